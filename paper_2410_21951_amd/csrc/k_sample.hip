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

void launch_perturb(const float* logits, const float* u, float* scores, int rows, int V1, float temperature,
                    float top_p, int tau, hipStream_t st) {
    hipLaunchKernelGGL(k_perturb, dim3(rows), dim3(256), (size_t)V1 * sizeof(float), st, logits, u, scores, V1,
                       temperature, top_p, tau);
}
