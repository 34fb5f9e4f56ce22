// Perturbed scores for the stochastic form of Algorithm 1 (tau tokens drawn per position from
// the nucleus of the temperature-scaled distribution, Sec. 3.1.2).
// For one logit row z and uniforms u: s = z / temperature; the nucleus keeps token v iff the
// tokens with a strictly larger s hold less than top_p of softmax(s), or fewer than tau tokens
// have a strictly larger s (so tau draws always exist); score = s - log(-log u) on kept tokens,
// -inf elsewhere.  Ordering a row's scores lists its tokens in the order successive draws
// without replacement would produce them, so the deterministic ranking kernels applied to the
// scores give Algorithm 1's "candidate is among the tau draws" and the first draw.
#include "common.h"

// Monotone map float -> uint32: a < b  <=>  key(a) < key(b) (no NaN expected).
__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t b = __float_as_uint(f);
    return b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
}

// One workgroup of 256 threads per row; the scaled row sits in LDS (V1 floats).
// The kept set is {v : s_v >= s*}; s* is found by a 16-way interval search over the 32-bit keys
// of the predicate "the tokens above this key hold less than top_p, or are fewer than tau",
// which is monotone in the key and changes only at values that occur in the row.
__global__ __launch_bounds__(256) void k_perturb(const float* __restrict__ logits, const float* __restrict__ u,
                                                 float* __restrict__ scores, int V1, float temperature,
                                                 float top_p, int tau) {
    extern __shared__ float s_s[];
    constexpr int NT = 15;
    __shared__ float s_f[2][4][NT + 1];
    __shared__ int s_i[2][4][NT + 1];
    const size_t row = blockIdx.x;
    const float* z = logits + row * V1;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    float m = -INFINITY;
    for (int v = tid; v < V1; v += 256) {
        const float s = z[v] / temperature + 0.f;   // -0 becomes +0: equal values, equal keys
        s_s[v] = s;
        m = fmaxf(m, s);
    }
    m = wave_max(m);
    if (lane == 0) s_f[0][wave][0] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_f[0][0][0], s_f[0][1][0]), fmaxf(s_f[0][2][0], s_f[0][3][0]));
    uint32_t kmin = 0;   // keep everything
    if (top_p < 1.f) {
        float zsum = 0.f;
        for (int v = tid; v < V1; v += 256) zsum += expf(s_s[v] - m);
        zsum = wave_sum(zsum);
        if (lane == 0) s_f[1][wave][0] = zsum;
        __syncthreads();
        const float target = top_p * (s_f[1][0][0] + s_f[1][1][0] + s_f[1][2][0] + s_f[1][3][0]);
        // Search for the smallest key at which the predicate holds.  It holds at hi (nothing lies
        // above the largest key) and is monotone; each round tries NT keys that cut [lo, hi] into
        // NT + 1 parts (their NT pairs of sums are reduced side by side, which costs little more
        // than one pair), so the interval shrinks 16-fold per round.  Every thread sees the same
        // sums, hence the same lo and hi: uniform control flow.
        uint32_t lo = 0, hi = 0xffffffffu;
        for (int it = 0; lo < hi; ++it) {
            const uint64_t span = (uint64_t)hi - lo;
            uint32_t mid[NT];
            float a[NT];
            int cnt[NT];
#pragma unroll
            for (int q = 0; q < NT; ++q) {
                mid[q] = lo + (uint32_t)((span * (uint64_t)(q + 1)) / (NT + 1));   // lo <= mid[q] < hi, non-decreasing
                a[q] = 0.f;
                cnt[q] = 0;
            }
            for (int v = tid; v < V1; v += 256) {
                const float s = s_s[v];
                const float e = expf(s - m);
                const uint32_t k = order_key(s);
#pragma unroll
                for (int q = 0; q < NT; ++q)
                    if (k > mid[q]) { a[q] += e; ++cnt[q]; }
            }
#pragma unroll
            for (int q = 0; q < NT; ++q) { a[q] = wave_sum_dpp(a[q]); cnt[q] = wave_sum_i_dpp(cnt[q]); }
            if (lane == 0) {
#pragma unroll
                for (int q = 0; q < NT; ++q) { s_f[it & 1][wave][q] = a[q]; s_i[it & 1][wave][q] = cnt[q]; }
            }
            __syncthreads();
            // the first key of the round at which the predicate holds bounds the answer from above,
            // the key before it (where it fails) from below
            uint32_t nlo = lo, nhi = hi;
            bool found = false;
#pragma unroll
            for (int q = 0; q < NT; ++q) {
                const float A = s_f[it & 1][0][q] + s_f[it & 1][1][q] + s_f[it & 1][2][q] + s_f[it & 1][3][q];
                const int C = s_i[it & 1][0][q] + s_i[it & 1][1][q] + s_i[it & 1][2][q] + s_i[it & 1][3][q];
                const bool holds = A < target || C < tau;
                if (!found) {
                    if (holds) { nhi = mid[q]; found = true; }
                    else nlo = mid[q] + 1;
                }
            }
            lo = nlo; hi = nhi;
        }
        kmin = hi;
    }
    float* y = scores + row * V1;
    const float* ur = u + row * V1;
    for (int v = tid; v < V1; v += 256) {
        const float s = s_s[v];
        y[v] = order_key(s) >= kmin ? s - logf(-logf(ur[v])) : -INFINITY;
    }
}


// Rows of up to 4096 logits: one WAVE per row, the row in registers (values of lane l: l, l + 64, ...), no LDS
// and no workgroup barrier.  The same search as in k_perturb, as a plain bisection over the 32-bit keys: a round is a
// compare and two conditional adds per value and two wave sums by lane permutations.  The values are kept as their
// keys (key_value gives a value back), entries beyond the row have key 0 (below every key) and mass 0.
__device__ __forceinline__ float key_value(uint32_t k) { return __uint_as_float(k ^ ((k >> 31) ? 0x80000000u : 0xffffffffu)); }
__device__ __forceinline__ float wave_max_dpp(float v) {
    v = fmaxf(v, __int_as_float(dpp_perm<0xB1>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_perm<0x4E>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_perm<0x141>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_perm<0x140>(__float_as_int(v))));
    return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0)), __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16))),
                 fmaxf(__int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32)), __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48))));
}
template <int GROUPS>   // groups of four 64-value chunks the row may have: GROUPS * 256 >= V1
__global__ __launch_bounds__(64) void k_perturb_wave(const float* __restrict__ logits, const float* __restrict__ u,
                                                     float* __restrict__ scores, int V1, float temperature, float top_p, int tau) {
    const size_t row = blockIdx.x;
    const int lane = threadIdx.x;
    const float* z = logits + row * V1;
    const float* ur = u + row * V1;
    float* y = scores + row * V1;
    float e[GROUPS][4];
    uint32_t key[GROUPS][4];
    float zv[GROUPS][4], gum[GROUPS][4];
    // logits and uniforms are asked for together (one memory latency, not one before and one after the search)
#pragma unroll
    for (int g = 0; g < GROUPS; ++g)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int v = g * 256 + q * 64 + lane;
            zv[g][q] = v < V1 ? z[v] : 0.f;
            gum[g][q] = v < V1 ? ur[v] : 0.5f;
        }
    float m = -INFINITY, mn = INFINITY;
#pragma unroll
    for (int g = 0; g < GROUPS; ++g)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int v = g * 256 + q * 64 + lane;
            const float sv = v < V1 ? zv[g][q] / temperature + 0.f : -INFINITY;   // -0 becomes +0: equal values, equal keys
            gum[g][q] = logf(-logf(gum[g][q]));
            key[g][q] = v < V1 ? order_key(sv) : 0u;
            m = fmaxf(m, sv);
            mn = fminf(mn, v < V1 ? sv : INFINITY);
        }
    m = wave_max_dpp(m);
    uint32_t kmin = 0;   // keep everything
    if (top_p < 1.f) {
        float zsum = 0.f;
#pragma unroll
        for (int g = 0; g < GROUPS; ++g)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                e[g][q] = g * 256 + q * 64 + lane < V1 ? expf(key_value(key[g][q]) - m) : 0.f;
                zsum += e[g][q];
            }
        const float target = top_p * wave_sum_dpp(zsum);
        // The search runs between the row's smallest and largest key: the predicate holds at the largest (nothing
        // lies above it), and below the smallest it is what it is at the smallest minus one (everything above), so a
        // result below the smallest key would keep the same tokens as the smallest key itself.  The answer is a key
        // of the row whenever the predicate fails just below the interval (it changes only at keys that occur), so
        // once the predicate has failed somewhere (lo has moved) and a single entry of the row is left in [lo, hi],
        // that entry's key is the answer: with ~1000 logits some 15 rounds instead of 32.
        uint32_t lo = order_key(-wave_max_dpp(-mn)), hi = order_key(m);
        // entries at or above lo and entries above hi, known from the rounds that set lo and hi: their difference is
        // the number of entries left in [lo, hi] (no count of its own per round)
        int c_lo = V1, c_hi = 0;
        bool failed = false;
        while (lo < hi) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            float a4[4] = {0.f, 0.f, 0.f, 0.f};   // four independent partial sums: no chain of dependent additions
            int c4[4] = {0, 0, 0, 0};
#pragma unroll
            for (int g = 0; g < GROUPS; ++g)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool above = key[g][q] > mid;
                    a4[q] += above ? e[g][q] : 0.f;
                    c4[q] += above ? 1 : 0;
                }
            const float A = wave_sum_dpp((a4[0] + a4[1]) + (a4[2] + a4[3]));
            const int C = wave_sum_i_dpp((c4[0] + c4[1]) + (c4[2] + c4[3]));
            if (A < target || C < tau) { hi = mid; c_hi = C; }
            else { lo = mid + 1; c_lo = C; failed = true; }
            if (failed && c_lo - c_hi == 1) {   // one entry left: its key (every other lane contributes 0)
                uint32_t kin = 0;
#pragma unroll
                for (int g = 0; g < GROUPS; ++g)
#pragma unroll
                    for (int q = 0; q < 4; ++q) kin = (key[g][q] >= lo && key[g][q] <= hi) ? key[g][q] : kin;
                hi = (uint32_t)wave_sum_i_dpp((int)kin);
                break;
            }
        }
        kmin = hi;
    }
#pragma unroll
    for (int g = 0; g < GROUPS; ++g)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int v = g * 256 + q * 64 + lane;
            if (v < V1) y[v] = key[g][q] >= kmin ? key_value(key[g][q]) - gum[g][q] : -INFINITY;
        }
}

void launch_perturb(const float* logits, const float* u, float* scores, int rows, int V1, float temperature,
                    float top_p, int tau, hipStream_t st) {
    if (V1 <= 1280) hipLaunchKernelGGL(k_perturb_wave<5>, dim3(rows), dim3(64), 0, st, logits, u, scores, V1, temperature, top_p, tau);
    else if (V1 <= 2304) hipLaunchKernelGGL(k_perturb_wave<9>, dim3(rows), dim3(64), 0, st, logits, u, scores, V1, temperature, top_p, tau);
    else if (V1 <= 4096) hipLaunchKernelGGL(k_perturb_wave<16>, dim3(rows), dim3(64), 0, st, logits, u, scores, V1, temperature, top_p, tau);
    else hipLaunchKernelGGL(k_perturb, dim3(rows), dim3(256), (size_t)V1 * sizeof(float), st, logits, u, scores, V1,
                            temperature, top_p, tau);
}
