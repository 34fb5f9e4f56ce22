// bf16 MFMA linear map for small row counts (tree nodes x model width).
//
// Y[r][n] = sum_k X[r][k] W[n][k]: the weights are streamed once from HBM in a
// pre-tiled layout that matches the B operand of v_mfma_f32_16x16x32_bf16, the
// activations are staged in LDS (A operand), accumulation is fp32.
//
// Packed weight layout: [n-tile of 16 outputs][k-step of 32][64 lanes][8 bf16];
// lane (c = lane & 15, g = lane >> 4) of tile (nt, ks) holds
// W[nt*16 + c][ks*32 + 8g .. 8g+7], so one wave load is one contiguous KiB.
//
// One workgroup (4 waves) owns one n-tile and a group of up to 64 rows; its
// waves split the k-steps round-robin and their partial sums are combined in a
// fixed order through LDS (deterministic, no atomics).
#include <algorithm>

#include "common.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

#define GM_KC 1024                 // k-chunk staged in LDS at a time
#define GM_LDX (GM_KC + 8)         // padded LDS row stride in bf16 elements
#define GM_RT 64                   // rows per workgroup
#define GM_SMEM (GM_RT * GM_LDX * 2)

__device__ __forceinline__ float gelu_m(float v) { return 0.5f * v * (1.f + erff(v * 0.70710678118654752f)); }
__device__ __forceinline__ float silu_m(float v) { return v / (1.f + __expf(-v)); }

__device__ __forceinline__ void epilogue_bf16(const GemmArgs& a, int r, int n, float acc) {
    if (a.bias) acc += a.bias[n];
    bf16_t* out = (bf16_t*)a.out;
    switch (a.epi) {
    case EPI_STORE: out[(size_t)r * a.N + n] = f2bf(acc); break;
    case EPI_GELU: out[(size_t)r * a.N + n] = f2bf(gelu_m(acc)); break;
    case EPI_RESID: a.outf[(size_t)r * a.N + n] += acc; break;
    case EPI_F32: a.outf[(size_t)r * a.N + n] = acc; break;
    case EPI_SILU_RESID:
        out[(size_t)r * a.N + n] = f2bf(bf2f(((const bf16_t*)a.X)[(size_t)r * a.K + n]) + silu_m(acc));
        break;
    case EPI_QKV: {
        if (n < a.d) { out[(size_t)r * a.d + n] = f2bf(acc); break; }
        const int which = n / a.d - 1, c = n % a.d, head = c >> 6, dim = c & 63;
        const int b = r / a.M, node = r % a.M;
        const int pos = a.L[b] + node;
        if (pos < a.maxpos) {
            const size_t hb = ((size_t)b * a.nH + head) * a.maxpos * 64;
            if (which) ((bf16_t*)a.Vc)[hb + (size_t)dim * a.maxpos + pos] = f2bf(acc);
            else ((bf16_t*)a.Kc)[hb + (size_t)pos * 64 + dim] = f2bf(acc);
        }
        break;
    }
    }
}

__global__ __launch_bounds__(256) void k_gemm_mfma(GemmArgs a) {
    extern __shared__ uint4 smem[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, c = lane & 15;
    const int nt = blockIdx.x, r0 = blockIdx.y * GM_RT;
    const int nks = a.K >> 5;
    const uint4* Wp = (const uint4*)a.W + (size_t)nt * nks * 64 + lane;
    const bf16_t* X = (const bf16_t*)a.X;
    f32x4_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

    for (int kc0 = 0; kc0 < a.K; kc0 += GM_KC) {
        const int kcl = min(GM_KC, a.K - kc0);
        const int ks0 = kc0 >> 5, ksn = kcl >> 5;
        // weights first: these are the loads that go to HBM
        uint4 bw[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int ks = wave + 4 * i;
            bw[i] = ks < ksn ? Wp[(size_t)(ks0 + ks) * 64] : make_uint4(0, 0, 0, 0);
        }
        __syncthreads();   // readers of the previous chunk are done
        const int v8 = kcl >> 3;   // 16-byte vectors per row
        for (int idx = tid; idx < GM_RT * v8; idx += 256) {
            const int row = idx / v8, col = idx - row * v8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (r0 + row < a.R) v = *(const uint4*)(X + (size_t)(r0 + row) * a.K + kc0 + col * 8);
            smem[row * (GM_LDX / 8) + col] = v;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int ks = wave + 4 * i;
            if (ks < ksn) {
                const bf16x8_t b = __builtin_bit_cast(bf16x8_t, bw[i]);
#pragma unroll
                for (int rt = 0; rt < 4; ++rt) {
                    const uint4 av = smem[(rt * 16 + c) * (GM_LDX / 8) + ks * 4 + g];
                    acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av), b, acc[rt], 0, 0, 0);
                }
            }
        }
    }
    // combine the four waves' partial sums in wave order
    __syncthreads();
    float* red = (float*)smem;
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
        for (int i = 0; i < 4; ++i) red[((wave * 4 + rt) * 64 + lane) * 4 + i] = acc[rt][i];
    __syncthreads();
    const int row = tid >> 2;                 // 0..63
    const int rt = row >> 4, rr = row & 15;
    if (r0 + row < a.R) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = (tid & 3) * 4 + j;
            const int n = nt * 16 + col;
            if (n < a.N) {
                const int src = ((rt * 64) + (rr >> 2) * 16 + col) * 4 + (rr & 3);
                float v = red[src];
#pragma unroll
                for (int w = 1; w < 4; ++w) v += red[w * 1024 + src];
                epilogue_bf16(a, r0 + row, n, v);
            }
        }
    }
}

void launch_gemm_mfma(const GemmArgs& a, hipStream_t st) {
    static bool once = false;
    if (!once) {
        (void)hipFuncSetAttribute((const void*)k_gemm_mfma, hipFuncAttributeMaxDynamicSharedMemorySize, GM_SMEM);
        once = true;
    }
    dim3 grid((a.N + 15) / 16, (a.R + GM_RT - 1) / GM_RT), blk(256);
    hipLaunchKernelGGL(k_gemm_mfma, grid, blk, GM_SMEM, st, a);
}

// fp32 [N][K] row-major -> packed bf16 tiles (rows >= N are zero)
__global__ void k_pack_w(const float* __restrict__ src, uint4* __restrict__ dst, int N, int K) {
    const int nks = K >> 5;
    const size_t total = (size_t)((N + 15) / 16) * nks * 64;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(i & 63);
        const size_t tile = i >> 6;
        const int ks = (int)(tile % nks), nt = (int)(tile / nks);
        const int n = nt * 16 + (lane & 15), k0 = ks * 32 + 8 * (lane >> 4);
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float lo = 0.f, hi = 0.f;
            if (n < N) { lo = src[(size_t)n * K + k0 + 2 * j]; hi = src[(size_t)n * K + k0 + 2 * j + 1]; }
            w[j] = (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
        }
        dst[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

void launch_pack_w(const float* src, void* dst, int N, int K, hipStream_t st) {
    const size_t total = (size_t)((N + 15) / 16) * (K >> 5) * 64;
    int blocks = (int)std::min<size_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(k_pack_w, dim3(blocks), dim3(256), 0, st, src, (uint4*)dst, N, K);
}
