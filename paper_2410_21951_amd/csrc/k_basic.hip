// Element-wise and generic kernels: embedding / tree expansion, LayerNorm, the
// generic (non-MFMA) linear map and attention used by the fp32 model, and a
// few conversion helpers.  Templated on the storage type (float or bf16 bits);
// all arithmetic is fp32.
#include "common.h"

// ---------------------------------------------------------------------------
// Tree expansion + embedding (Sec. 2.1: the root is the base head's next token,
// depth D is filled from draft head D's top-k list; positions continue after
// the committed prefix).  In prefill mode the rows are consecutive prompt
// tokens: text ids are passed as -(id + 1), speech ids as they are.
// One block per row.
// ---------------------------------------------------------------------------
template <class T>
__global__ void k_embed(Dims D, DevState s, int prefill_mode, int table) {
    const int r = blockIdx.x, b = r / D.M, n = r % D.M;
    float* x = s.x + (size_t)r * D.d;
    int rows;
    if (prefill_mode) rows = s.n_rows[b];
    else rows = s.finished[b] ? 0 : D.M;
    if (!prefill_mode && n == 0 && threadIdx.x == 0) s.n_rows[b] = rows;
    if (n >= rows) {
        for (int i = threadIdx.x; i < D.d; i += blockDim.x) x[i] = 0.f;
        if (threadIdx.x == 0) s.tok[r] = 0;
        return;
    }
    int tok, pos;
    const T* E;
    if (prefill_mode) {
        int t = s.chunk_tok[r];
        pos = s.L[b] + n;
        if (t < 0) { tok = -t - 1; E = (const T*)s.E_text; }
        else { tok = t; E = (const T*)s.E_speech; }
    } else {
        int dep = s.t_depth[table][n];
        pos = s.L[b] + dep;
        if (n == 0) tok = s.root[b];
        else tok = s.draft_topk[((size_t)b * D.Hh + (dep - 1)) * VADUSA_MAX_TOPK + s.t_rank[table][n]];
        if ((unsigned)tok >= (unsigned)D.V1) tok = 0;   // rows of NaN logits have no arg-max and no draft lists: stay inside the table
        E = (const T*)s.E_speech;
    }
    if (pos >= D.maxpos) pos = D.maxpos - 1;   // never reached: the host checks capacity first
    if (threadIdx.x == 0) s.tok[r] = tok;
    const T* e = E + (size_t)tok * D.d;
    const T* p = (const T*)s.P + (size_t)pos * D.d;
    for (int i = threadIdx.x; i < D.d; i += blockDim.x) x[i] = ldf(e + i) + ldf(p + i);
}

void launch_embed(const Dims& D, const DevState& s, int dtype, int prefill_mode, int table, hipStream_t st) {
    dim3 g(D.B * D.M), blk(256);
    if (dtype) hipLaunchKernelGGL(k_embed<bf16_t>, g, blk, 0, st, D, s, prefill_mode, table);
    else hipLaunchKernelGGL(k_embed<float>, g, blk, 0, st, D, s, prefill_mode, table);
}

// ---------------------------------------------------------------------------
// LayerNorm over the last axis, one wave per row (biased variance, eps 1e-5).
// ---------------------------------------------------------------------------
template <class T>
__global__ void k_layernorm(const float* __restrict__ x, const float* __restrict__ g,
                            const float* __restrict__ bt, T* __restrict__ out, int R, int d) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = blockIdx.x * (blockDim.x >> 6) + wave;
    if (r >= R) return;
    const float* xr = x + (size_t)r * d;
    float sum = 0.f;
    for (int i = lane; i < d; i += 64) sum += xr[i];
    const float mu = wave_sum(sum) / d;
    float sq = 0.f;
    for (int i = lane; i < d; i += 64) { float t = xr[i] - mu; sq += t * t; }
    const float rstd = rsqrtf(wave_sum(sq) / d + LN_EPS);
    T* o = out + (size_t)r * d;
    for (int i = lane; i < d; i += 64) stf(o + i, (xr[i] - mu) * rstd * g[i] + bt[i]);
}

void launch_layernorm(const float* x, const float* g, const float* b, void* out, int R, int d, int dtype, hipStream_t st) {
    dim3 grid((R + 3) / 4), blk(256);
    if (dtype) hipLaunchKernelGGL(k_layernorm<bf16_t>, grid, blk, 0, st, x, g, b, (bf16_t*)out, R, d);
    else hipLaunchKernelGGL(k_layernorm<float>, grid, blk, 0, st, x, g, b, (float*)out, R, d);
}

// ---------------------------------------------------------------------------
// Generic linear map Y = X W^T (+ bias) with the epilogues of common.h.
// One wave per output column and tile of 16 rows; lanes stride over K and the
// 16 partial sums are reduced across the wave.  W is [N][K] row-major.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float gelu_f(float v) { return 0.5f * v * (1.f + erff(v * 0.70710678118654752f)); }
__device__ __forceinline__ float silu_f(float v) { return v / (1.f + __expf(-v)); }

template <class T>
__device__ __forceinline__ void epilogue(const GemmArgs& a, int r, int n, float acc) {
    if (a.bias) acc += a.bias[n];
    switch (a.epi) {
    case EPI_STORE: stf((T*)a.out + (size_t)r * a.N + n, acc); break;
    case EPI_GELU: stf((T*)a.out + (size_t)r * a.N + n, gelu_f(acc)); break;
    case EPI_RESID: a.outf[(size_t)r * a.N + n] += acc; break;
    case EPI_F32: a.outf[(size_t)r * a.N + n] = acc; break;
    case EPI_SILU_RESID:
        stf((T*)a.out + (size_t)r * a.N + n, ldf((const T*)a.X + (size_t)r * a.K + n) + silu_f(acc));
        break;
    case EPI_QKV: {
        if (n < a.d) { stf((T*)a.out + (size_t)r * a.d + n, acc); break; }
        const int which = n / a.d - 1, c = n % a.d, head = c >> 6, dim = c & 63;
        const int b = r / a.M, node = r % a.M;
        const int pos = a.L[b] + node;
        if (pos < a.maxpos) {
            const size_t hb = ((size_t)b * a.nH + head) * kv_cap(a.maxpos) * 64;
            if (which) stf((T*)a.Vc + hb + vc_off(pos, dim), acc);
            else stf((T*)a.Kc + hb + kc_off(pos, dim), acc);
        }
        break;
    }
    }
}

template <class T>
__global__ void k_gemm_simple(GemmArgs a) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + wave;
    const int r0 = blockIdx.y * 16;
    if (n >= a.N) return;
    const T* w = (const T*)a.W + (size_t)n * a.K;
    const T* X = (const T*)a.X;
    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    const T* xr[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) xr[i] = X + (size_t)min(r0 + i, a.R - 1) * a.K;
    for (int k = lane; k < a.K; k += 64) {
        const float wv = ldf(w + k);
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = fmaf(ldf(xr[i] + k), wv, acc[i]);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = wave_sum(acc[i]);
    if (lane < 16 && r0 + lane < a.R) {
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) if (lane == i) v = acc[i];
        epilogue<T>(a, r0 + lane, n, v);
    }
}

void launch_gemm_simple(const GemmArgs& a, int dtype, hipStream_t st) {
    dim3 grid((a.N + 3) / 4, (a.R + 15) / 16), blk(256);
    if (dtype) hipLaunchKernelGGL(k_gemm_simple<bf16_t>, grid, blk, 0, st, a);
    else hipLaunchKernelGGL(k_gemm_simple<float>, grid, blk, 0, st, a);
}

// ---------------------------------------------------------------------------
// Generic tree-masked attention (Sec. 2.1): one wave per (row, head).  A row
// sees cache positions [0, L) and, among the rows of this forward (stored at
// cache rows L + m), those whose bit is set in its mask row.  Lanes take keys
// round-robin with a private online softmax, then the 64 partial results are
// merged through LDS.
// ---------------------------------------------------------------------------
template <class T>
__global__ void k_attn_simple(Dims D, DevState s, int layer, int table) {
    __shared__ float so[64][65];
    const int n = blockIdx.x, head = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int r = b * D.M + n;
    T* out = (T*)s.att + (size_t)r * D.d + head * 64;
    if (n >= s.n_rows[b]) { stf(out + lane, 0.f); return; }
    const int L = s.L[b];
    const size_t hb = ((((size_t)layer * D.Bmax + b) * D.nH + head) * kv_cap(D.maxpos)) * 64;
    const T* Kh = (const T*)s.Kc + hb;
    const T* Vh = (const T*)s.Vc + hb;
    const T* qp = (const T*)s.q + (size_t)r * D.d + head * 64;
    float q[64];
#pragma unroll
    for (int i = 0; i < 64; ++i) q[i] = ldf(qp + i) * 0.125f;
    // table 1 is the causal chunk of the prefill (row n sees rows 0..n), which may have more rows
    // than the mask table has entries: no mask words are read for it
    const uint32_t* mrow = s.t_mask[0] + (size_t)(table == 1 ? 0 : n) * MASK_WORDS;
    float m = -INFINITY, l = 0.f, o[64];
#pragma unroll
    for (int i = 0; i < 64; ++i) o[i] = 0.f;
    const int T_all = L + D.M;
    for (int j = lane; j < T_all; j += 64) {
        if (j >= L) {
            const int mm = j - L;
            if (table == 1 ? mm > n : !((mrow[(mm >> 5) & (MASK_WORDS - 1)] >> (mm & 31)) & 1u)) continue;
        }
        float sc = 0.f;
#pragma unroll
        for (int i = 0; i < 64; ++i) sc = fmaf(q[i], ldf(Kh + kc_off(j, i)), sc);
        const float mn = fmaxf(m, sc);
        const float corr = __expf(m - mn), p = __expf(sc - mn);
        l = l * corr + p;
#pragma unroll
        for (int i = 0; i < 64; ++i) o[i] = o[i] * corr + p * ldf(Vh + vc_off(j, i));
        m = mn;
    }
    const float mx = wave_max(m);
    const float w = (m == -INFINITY) ? 0.f : __expf(m - mx);
    const float lt = wave_sum(l * w);
#pragma unroll
    for (int i = 0; i < 64; ++i) so[lane][i] = o[i] * w;
    __syncthreads();
    float acc = 0.f;
    for (int i = 0; i < 64; ++i) acc += so[i][lane];
    stf(out + lane, acc / lt);
}

void launch_attn_simple(const Dims& D, const DevState& s, int layer, int table, int dtype, hipStream_t st) {
    dim3 grid(D.M, D.nH, D.B), blk(64);
    if (dtype) hipLaunchKernelGGL(k_attn_simple<bf16_t>, grid, blk, 0, st, D, s, layer, table);
    else hipLaunchKernelGGL(k_attn_simple<float>, grid, blk, 0, st, D, s, layer, table);
}

// ---------------------------------------------------------------------------
// Helpers: fp32 -> storage conversion, storage -> fp32, prefill bookkeeping,
// KV read-back for inspection.
// ---------------------------------------------------------------------------
template <class T>
__global__ void k_convert(const float* __restrict__ src, T* __restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) stf(dst + i, src[i]);
}
void launch_convert(const float* src, void* dst, size_t n, int dtype, hipStream_t st) {
    int blocks = (int)((n + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    if (dtype) hipLaunchKernelGGL(k_convert<bf16_t>, dim3(blocks), dim3(256), 0, st, src, (bf16_t*)dst, n);
    else hipLaunchKernelGGL(k_convert<float>, dim3(blocks), dim3(256), 0, st, src, (float*)dst, n);
}

template <class T>
__global__ void k_to_float(const T* __restrict__ src, float* __restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = ldf(src + i);
}
void launch_to_float(const void* src, float* dst, size_t n, int dtype, hipStream_t st) {
    int blocks = (int)((n + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    if (dtype) hipLaunchKernelGGL(k_to_float<bf16_t>, dim3(blocks), dim3(256), 0, st, (const bf16_t*)src, dst, n);
    else hipLaunchKernelGGL(k_to_float<float>, dim3(blocks), dim3(256), 0, st, (const float*)src, dst, n);
}

__global__ void k_advance(DevState s, int B) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) s.L[b] += s.n_rows[b];
}
void launch_advance(const DevState& s, int B, hipStream_t st) {
    hipLaunchKernelGGL(k_advance, dim3((B + 63) / 64), dim3(64), 0, st, s, B);
}

// out[p][head*64 + dim] = K or V of (seq, head, position pos0 + p, dim)
template <class T>
__global__ void k_read_kv(Dims D, const T* __restrict__ cache, int seq, int which, int pos0, int npos, float* out) {
    const int p = blockIdx.x;
    for (int c = threadIdx.x; c < D.d; c += blockDim.x) {
        const int head = c >> 6, dim = c & 63;
        const size_t hb = ((size_t)seq * D.nH + head) * kv_cap(D.maxpos) * 64;
        out[(size_t)p * D.d + c] = which ? ldf(cache + hb + vc_off(pos0 + p, dim)) : ldf(cache + hb + kc_off(pos0 + p, dim));
    }
}
void launch_read_kv(const Dims& D, const void* cache_layer, int seq, int which, int pos0, int npos, float* out, int dtype, hipStream_t st) {
    if (dtype) hipLaunchKernelGGL(k_read_kv<bf16_t>, dim3(npos), dim3(256), 0, st, D, (const bf16_t*)cache_layer, seq, which, pos0, npos, out);
    else hipLaunchKernelGGL(k_read_kv<float>, dim3(npos), dim3(256), 0, st, D, (const float*)cache_layer, seq, which, pos0, npos, out);
}
