// Verification with tolerance (Algorithm 1), choice of the accepted path
// (Sec. 2.3), KV compaction to that path, continuation from the last accepted
// node (Sec. 2.1) and the draft heads' top-k lists.
#include "common.h"

// Total order used everywhere a "largest logit" is needed: value descending,
// then token id ascending.  before(a, b) = a ranks strictly ahead of b.
__device__ __forceinline__ bool before(float va, int ia, float vb, int ib) {
    return va > vb || (va == vb && ia < ib);
}

// Block-wide arg-best under the order above, restricted to entries that come
// strictly after (pv, pi).  Every thread returns the winner.  blockDim = 256.
__device__ int block_argbest(const float* __restrict__ z, int n, float pv, int pi, float* best_val) {
    __shared__ float sv[4];
    __shared__ int si[4];
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int v = threadIdx.x; v < n; v += blockDim.x) {
        const float zv = z[v];
        if (before(pv, pi, zv, v) && before(zv, v, bv, bi)) { bv = zv; bi = v; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (before(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    __syncthreads();   // protects sv/si against the previous call's readers
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    bv = sv[0]; bi = si[0];
    for (int w = 1; w < 4; ++w) if (before(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
    if (best_val) *best_val = bv;
    return bi;
}

// ---------------------------------------------------------------------------
// Algorithm 1 on every edge at once, then Sec. 2.3's choice.  One block (four
// waves) per sequence.  Edge n is accepted iff fewer than tau entries of the
// parent's logit row rank before the node's token; one wave counts one edge.
// path_ok[n] = every edge from the root to n accepted; the chosen node is the
// deepest such node, smallest index among equals (canonical order = leftmost).
// Output: path[b] = {count, node indices...}; count is cut after the first EOS.
// ---------------------------------------------------------------------------
__global__ void k_accept(Dims D, DevState s, int tau, int ignore_eos) {
    __shared__ int s_edge[VADUSA_MAX_TREE_NODES];
    __shared__ int s_ok[VADUSA_MAX_TREE_NODES];
    const int b = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int32_t* path = s.path + (size_t)b * (VADUSA_MAX_DRAFT_HEADS + 2);
    if (s.finished[b]) {
        if (threadIdx.x == 0) path[0] = 0;
        for (int n = threadIdx.x; n < D.M; n += blockDim.x) s.edge_ok[b * D.M + n] = 0;
        return;
    }
    const int32_t* parent = s.t_parent[0];
    const int32_t* depth = s.t_depth[0];
    const int32_t* tok = s.tok + (size_t)b * D.M;
    for (int n = wave; n < D.M; n += 4) {
        int edge = 1;
        if (n > 0) {
            const float* z = s.logits + ((size_t)b * D.M + parent[n]) * D.V1;
            const int t = tok[n];
            const float zt = z[t];
            int cnt = 0;
            for (int v = lane; v < D.V1; v += 64) cnt += before(z[v], v, zt, t) ? 1 : 0;
            edge = wave_sum_i(cnt) < tau;
        }
        if (lane == 0) { s_edge[n] = edge; s.edge_ok[b * D.M + n] = edge; }
    }
    __syncthreads();
    for (int n = threadIdx.x; n < D.M; n += blockDim.x) {
        int ok = 1, m = n;
        while (m > 0) { ok &= s_edge[m]; m = parent[m]; }
        s_ok[n] = ok;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int best = 0;
        for (int n = 1; n < D.M; ++n)
            if (s_ok[n] && depth[n] > depth[best]) best = n;
        int cnt = depth[best] + 1;
        int m = best;
        for (int j = cnt - 1; j >= 0; --j) { path[1 + j] = m; m = parent[m]; }
        if (!ignore_eos)
            for (int j = 0; j < cnt; ++j)
                if (tok[path[1 + j]] == D.V1 - 1) { cnt = j + 1; break; }
        path[0] = cnt;
    }
}

void launch_accept(const Dims& D, const DevState& s, int tau, int ignore_eos, hipStream_t st) {
    hipLaunchKernelGGL(k_accept, dim3(D.B), dim3(256), 0, st, D, s, tau, ignore_eos);
}

// ---------------------------------------------------------------------------
// KV compaction: cache row L + j <- row L + path[j] for the chosen path.
// path[j] >= j, so a destination row can be the source of an earlier j; every
// thread owns one column of one head and reads all its sources before writing.
// Grid (nH, nseq, Ly), 64 threads.
// ---------------------------------------------------------------------------
template <class T>
__global__ void k_commit_kv(Dims D, DevState s, int seq0) {
    const int head = blockIdx.x, b = seq0 + blockIdx.y, layer = blockIdx.z, dim = threadIdx.x;
    const int32_t* path = s.path + (size_t)b * (VADUSA_MAX_DRAFT_HEADS + 2);
    const int cnt = path[0];
    if (cnt <= 0) return;
    const int L = s.L[b];
    const size_t hb = ((((size_t)layer * D.Bmax + b) * D.nH + head) * D.maxpos) * 64;
    T* Kh = (T*)s.Kc + hb;
    T* Vh = (T*)s.Vc + hb;
    T kr[VADUSA_MAX_DRAFT_HEADS + 1], vr[VADUSA_MAX_DRAFT_HEADS + 1];
#pragma unroll
    for (int j = 0; j < VADUSA_MAX_DRAFT_HEADS + 1; ++j)
        if (j < cnt) {
            kr[j] = Kh[(size_t)(L + path[1 + j]) * 64 + dim];
            vr[j] = Vh[(size_t)(L + path[1 + j]) * 64 + dim];
        }
#pragma unroll
    for (int j = 0; j < VADUSA_MAX_DRAFT_HEADS + 1; ++j)
        if (j < cnt) {
            Kh[(size_t)(L + j) * 64 + dim] = kr[j];
            Vh[(size_t)(L + j) * 64 + dim] = vr[j];
        }
}

void launch_commit_kv(const Dims& D, const DevState& s, int seq0, int nseq, int dtype, hipStream_t st) {
    dim3 grid(D.nH, nseq, D.Ly), blk(64);
    if (dtype) hipLaunchKernelGGL(k_commit_kv<bf16_t>, grid, blk, 0, st, D, s, seq0);
    else hipLaunchKernelGGL(k_commit_kv<float>, grid, blk, 0, st, D, s, seq0);
}

// ---------------------------------------------------------------------------
// Continue from the last accepted node (Sec. 2.1): advance L, append the
// accepted tokens to the output, next root = best logit of that node's row,
// and copy its hidden state for the draft heads.  One block per sequence.
// In prefill mode the "path" is the chunk's last row and nothing is emitted.
// ---------------------------------------------------------------------------
template <class T>
__global__ void k_finalize(Dims D, DevState s, int seq0, int prefill_mode, int ignore_eos) {
    const int b = seq0 + blockIdx.x;
    int32_t* path = s.path + (size_t)b * (VADUSA_MAX_DRAFT_HEADS + 2);
    int cnt, last;
    if (prefill_mode) {
        cnt = s.n_rows[b];
        last = cnt - 1;
    } else {
        cnt = path[0];
        last = cnt > 0 ? path[cnt] : 0;
    }
    if (!prefill_mode && threadIdx.x == 0) s.acc_len[b] = cnt;
    if (cnt <= 0) return;
    const int32_t* tok = s.tok + (size_t)b * D.M;
    const int r = b * D.M + last;
    const int root = block_argbest(s.logits + (size_t)r * D.V1, D.V1, INFINITY, -1, nullptr);
    const T* h = (const T*)s.hn + (size_t)r * D.d;
    T* hb = (T*)s.hbest + (size_t)b * D.d;
    for (int i = threadIdx.x; i < D.d; i += blockDim.x) hb[i] = h[i];
    if (threadIdx.x == 0) {
        s.root[b] = root;
        s.L[b] += cnt;
        if (!prefill_mode) {
            int no = s.n_out[b];
            bool fin = false;
            for (int j = 0; j < cnt; ++j) {
                const int t = tok[path[1 + j]];
                s.acc_tok[b * (VADUSA_MAX_DRAFT_HEADS + 1) + j] = t;
                if (no < D.maxpos) s.out_tok[(size_t)b * D.maxpos + no++] = t;
                if (t == D.V1 - 1) fin = true;
            }
            s.n_out[b] = no;
            path[0] = 0;   // consumed
            if (fin && !ignore_eos) s.finished[b] = 1;
        }
    }
}

void launch_finalize(const Dims& D, const DevState& s, int seq0, int nseq, int prefill_mode, int ignore_eos, int dtype, hipStream_t st) {
    if (dtype) hipLaunchKernelGGL(k_finalize<bf16_t>, dim3(nseq), dim3(256), 0, st, D, s, seq0, prefill_mode, ignore_eos);
    else hipLaunchKernelGGL(k_finalize<float>, dim3(nseq), dim3(256), 0, st, D, s, seq0, prefill_mode, ignore_eos);
}

// ---------------------------------------------------------------------------
// Draft lists: the VADUSA_MAX_TOPK best ids of each draft head's logits,
// descending, equal logits: lower id first (Sec. 2.1).  Grid (Hh, nseq).
// ---------------------------------------------------------------------------
__global__ void k_topk(Dims D, DevState s, int seq0) {
    const int i = blockIdx.x, b = seq0 + blockIdx.y;
    const float* z = s.zdraft + ((size_t)i * D.Bmax + b) * D.V1;
    int32_t* out = s.draft_topk + ((size_t)b * D.Hh + i) * VADUSA_MAX_TOPK;
    float pv = INFINITY;
    int pi = -1;
    const int kmax = D.V1 < VADUSA_MAX_TOPK ? D.V1 : VADUSA_MAX_TOPK;
    for (int k = 0; k < kmax; ++k) {
        float bv;
        const int bi = block_argbest(z, D.V1, pv, pi, &bv);
        if (threadIdx.x == 0) out[k] = bi;
        pv = bv; pi = bi;
    }
}

void launch_topk(const Dims& D, const DevState& s, int seq0, int nseq, hipStream_t st) {
    hipLaunchKernelGGL(k_topk, dim3(D.Hh, nseq), dim3(256), 0, st, D, s, seq0);
}
