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
// The kept set is {v : s_v >= s*}; s* is found by bisection over the 32-bit keys of the
// predicate "the tokens above this key hold less than top_p, or are fewer than tau", which is
// monotone in the key and changes only at values that occur in the row.
__global__ __launch_bounds__(256) void k_perturb(const float* __restrict__ logits, const float* __restrict__ u,
                                                 float* __restrict__ scores, int V1, float temperature,
                                                 float top_p, int tau) {
    extern __shared__ float s_s[];
    __shared__ float s_f[2][4];
    __shared__ int s_i[2][4];
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
    if (lane == 0) s_f[0][wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_f[0][0], s_f[0][1]), fmaxf(s_f[0][2], s_f[0][3]));
    uint32_t kmin = 0;   // keep everything
    if (top_p < 1.f) {
        float zsum = 0.f;
        for (int v = tid; v < V1; v += 256) zsum += expf(s_s[v] - m);
        zsum = wave_sum(zsum);
        if (lane == 0) s_f[1][wave] = zsum;
        __syncthreads();
        const float target = top_p * (s_f[1][0] + s_f[1][1] + s_f[1][2] + s_f[1][3]);
        uint32_t lo = 0, hi = 0xffffffffu;   // the predicate holds at hi (nothing lies above it)
        for (int it = 0; it < 32; ++it) {    // every thread sees the same sums: uniform control flow
            const uint32_t mid = lo + ((hi - lo) >> 1);
            float a = 0.f;
            int cnt = 0;
            for (int v = tid; v < V1; v += 256) {
                const float s = s_s[v];
                if (order_key(s) > mid) { a += expf(s - m); ++cnt; }
            }
            a = wave_sum(a);
            cnt = wave_sum_i(cnt);
            if (lane == 0) { s_f[it & 1][wave] = a; s_i[it & 1][wave] = cnt; }
            __syncthreads();
            const float A = s_f[it & 1][0] + s_f[it & 1][1] + s_f[it & 1][2] + s_f[it & 1][3];
            const int C = s_i[it & 1][0] + s_i[it & 1][1] + s_i[it & 1][2] + s_i[it & 1][3];
            if (A < target || C < tau) hi = mid; else lo = mid + 1;
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
