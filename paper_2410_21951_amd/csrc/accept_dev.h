// Device functions for verification with tolerance (Algorithm 1), choice of the
// accepted path (Sec. 2.3), continuation from the last accepted node (Sec. 2.1),
// KV compaction and the draft heads' top-k lists.  Each function is the body of
// one workgroup of 256 threads (64 for the compaction); the generic kernels and
// the persistent step kernel both call them.
#pragma once
#include "common.h"

// Total order used everywhere a "largest logit" is needed: value descending,
// then token id ascending.  before(a, b) = a ranks strictly ahead of b.
__device__ __forceinline__ bool before(float va, int ia, float vb, int ib) {
    return va > vb || (va == vb && ia < ib);
}

// Best (value, id) pair of a wave under the order above; every lane gets it.  Inside a row of 16
// lanes by DPP permutations (after each step twice as many lanes agree, so the mirrored partners
// serve as well as the xor partners), across the four rows by the row-swap instructions.
template <int CTRL>
__device__ __forceinline__ void argbest_step(float& bv, int& bi) {
    const float ov = __int_as_float(dpp_perm<CTRL>(__float_as_int(bv)));
    const int oi = dpp_perm<CTRL>(bi);
    if (before(ov, oi, bv, bi)) { bv = ov; bi = oi; }
}
__device__ __forceinline__ void row16_argbest(float& bv, int& bi) {
    argbest_step<0xB1>(bv, bi);
    argbest_step<0x4E>(bv, bi);
    argbest_step<0x141>(bv, bi);
    argbest_step<0x140>(bv, bi);
}
__device__ __forceinline__ void wave_argbest(float& bv, int& bi) {
    row16_argbest(bv, bi);
    {
        const vadusa_u32x2 rv = __builtin_amdgcn_permlane16_swap(__float_as_uint(bv), __float_as_uint(bv), false, false);
        const vadusa_u32x2 ri = __builtin_amdgcn_permlane16_swap((unsigned)bi, (unsigned)bi, false, false);
        const bool x = before(__uint_as_float(rv.x), (int)ri.x, __uint_as_float(rv.y), (int)ri.y);
        bv = __uint_as_float(x ? rv.x : rv.y); bi = (int)(x ? ri.x : ri.y);
    }
    {
        const vadusa_u32x2 rv = __builtin_amdgcn_permlane32_swap(__float_as_uint(bv), __float_as_uint(bv), false, false);
        const vadusa_u32x2 ri = __builtin_amdgcn_permlane32_swap((unsigned)bi, (unsigned)bi, false, false);
        const bool x = before(__uint_as_float(rv.x), (int)ri.x, __uint_as_float(rv.y), (int)ri.y);
        bv = __uint_as_float(x ? rv.x : rv.y); bi = (int)(x ? ri.x : ri.y);
    }
}

// Block-wide arg-best under the order above, restricted to entries that come
// strictly after (pv, pi).  Every thread returns the winner.  256 threads.
__device__ inline int block_argbest(const float* __restrict__ z, int n, float pv, int pi, float* best_val) {
    __shared__ float sv[4];
    __shared__ int si[4];
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int v0 = threadIdx.x; v0 < n; v0 += 256 * 4) {
        float zv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) zv[j] = v0 + 256 * j < n ? z[v0 + 256 * j] : 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int v = v0 + 256 * j;
            if (v < n && before(pv, pi, zv[j], v) && before(zv[j], v, bv, bi)) { bv = zv[j]; bi = v; }
        }
    }
    wave_argbest(bv, bi);
    __syncthreads();   // protects sv/si against the previous call's readers
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    bv = sv[0]; bi = si[0];
    for (int w = 1; w < 4; ++w) if (before(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
    if (bi == 0x7fffffff) bi = 0;   // no entry qualifies (a row of NaN): still an index of the row
    if (best_val) *best_val = bv;
    return bi;
}

// Algorithm 1, one edge: node n of sequence b is accepted iff fewer than tau entries of its
// parent's logit row rank before its token.  One wave; every lane returns the decision.
__device__ inline int dev_edge(const Dims& D, const DevState& s, int b, int n, int tau) {
    if (n == 0) return 1;
    const int lane = threadIdx.x & 63;
    const float* z = s.logits + ((size_t)b * D.M + s.t_parent[0][n]) * D.V1;
    const int t = s.tok[(size_t)b * D.M + n];
    const float zt = z[t];
    int cnt = 0;
    for (int v0 = lane; v0 < D.V1; v0 += 64 * 17) {
        float zv[17];
#pragma unroll
        for (int q = 0; q < 17; ++q) zv[q] = v0 + 64 * q < D.V1 ? z[v0 + 64 * q] : -INFINITY;
#pragma unroll
        for (int q = 0; q < 17; ++q) cnt += (v0 + 64 * q < D.V1 && before(zv[q], v0 + 64 * q, zt, t)) ? 1 : 0;
    }
    return wave_sum_i_dpp(cnt) < tau;
}

// Sec. 2.3's choice from the edge decisions in s_edge (LDS, complete and visible on entry):
// path_ok[n] = every edge from the root to n accepted; the chosen node is the deepest such
// node, smallest index among equals (canonical order = leftmost).
// Output: path[b] = {count, node indices...}; the count is cut after the first EOS.
__device__ inline void dev_choose(const Dims& D, const DevState& s, int b, int ignore_eos, const int* s_edge, int* s_ok) {
    int32_t* path = s.path + (size_t)b * (VADUSA_MAX_DRAFT_HEADS + 2);
    const int32_t* parent = s.t_parent[0];
    const int32_t* depth = s.t_depth[0];
    const int32_t* tok = s.tok + (size_t)b * D.M;
    // the tree tables go to LDS once: the walks below would otherwise pay a memory latency per hop
    __shared__ int s_par[VADUSA_MAX_TREE_NODES];
    __shared__ int s_key[VADUSA_MAX_TREE_NODES];
    for (int n = threadIdx.x; n < D.M; n += 256) s_par[n] = ldg(parent + n);
    __syncthreads();
    for (int n = threadIdx.x; n < D.M; n += 256) {
        int ok = 1, m = n;
        while (m > 0) { ok &= s_edge[m]; m = s_par[m]; }
        s_ok[n] = ok;
        // deepest accepted node, smallest index among equals: largest depth * 256 + (255 - n)
        s_key[n] = ok ? ldg(depth + n) * 256 + (255 - n) : -1;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int key = -1;
        for (int n0 = 0; n0 < D.M; n0 += 8) {
            int kq[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) kq[q] = s_key[(n0 + q) & (VADUSA_MAX_TREE_NODES - 1)];
#pragma unroll
            for (int q = 0; q < 8; ++q) if (n0 + q < D.M && kq[q] > key) key = kq[q];
        }
        const int best = key < 0 ? 0 : 255 - (key & 255);
        int cnt = (key < 0 ? 0 : key >> 8) + 1;
        int m = best;
        int nodes[VADUSA_MAX_DRAFT_HEADS + 1];
        for (int j = cnt - 1; j >= 0; --j) { nodes[j] = m; m = s_par[m]; }
        if (!ignore_eos)
            for (int j = 0; j < cnt; ++j)
                if (ldg(tok + nodes[j]) == D.V1 - 1) { cnt = j + 1; break; }
        for (int j = 0; j < cnt; ++j) stwi(path + 1 + j, nodes[j]);
        stwi(path, cnt);
    }
    __syncthreads();
}

// Algorithm 1 on every edge of sequence b at once, then Sec. 2.3's choice.
// Edge n is accepted iff fewer than tau entries of the parent's logit row rank
// before the node's token (one wave counts one edge).  path_ok[n] = every edge
// from the root to n accepted; the chosen node is the deepest such node,
// smallest index among equals (canonical order = leftmost).
// Output: path[b] = {count, node indices...}; the count is cut after the first EOS.
__device__ inline void dev_accept(const Dims& D, const DevState& s, int b, int tau, int ignore_eos) {
    __shared__ int s_edge[VADUSA_MAX_TREE_NODES];
    __shared__ int s_ok[VADUSA_MAX_TREE_NODES];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int32_t* path = s.path + (size_t)b * (VADUSA_MAX_DRAFT_HEADS + 2);
    if (s.finished[b]) {
        if (threadIdx.x == 0) stwi(path, 0);
        for (int n = threadIdx.x; n < D.M; n += 256) stwi(s.edge_ok + b * D.M + n, 0);
        return;
    }
    const int32_t* parent = s.t_parent[0];
    const int32_t* tok = s.tok + (size_t)b * D.M;
    // Wave w owns the edges n = w + 4j.  Lane j first fetches parent, token and the token's logit
    // of edge j, so that chain of three dependent loads is paid once per wave, not once per
    // edge; then the wave streams the parents' rows, two edges at a time, 17 values per lane and
    // batch (one batch covers 1088 logits).
    const int nj = (D.M - wave + 3) / 4;   // edges of this wave, at most 32
    int my_par = 0, my_t = 0;
    float my_zt = 0.f;
    if (lane < nj && wave + 4 * lane > 0) {
        const int n = wave + 4 * lane;
        my_par = parent[n];
        my_t = tok[n];
        my_zt = s.logits[((size_t)b * D.M + my_par) * D.V1 + my_t];
    }
    for (int j0 = 0; j0 < nj; j0 += 2) {
        int cnt[2] = {0, 0};
        const float* zrow[2];
        int tt[2];
        float ztv[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int j = j0 + e < nj ? j0 + e : j0;   // an odd tail repeats the edge (result unused)
            zrow[e] = s.logits + ((size_t)b * D.M + __shfl(my_par, j, 64)) * D.V1;
            tt[e] = __shfl(my_t, j, 64);
            ztv[e] = __shfl(my_zt, j, 64);
        }
        for (int v0 = lane; v0 < D.V1; v0 += 64 * 17) {
            float zv[2][17];
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int q = 0; q < 17; ++q) zv[e][q] = v0 + 64 * q < D.V1 ? zrow[e][v0 + 64 * q] : -INFINITY;
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int q = 0; q < 17; ++q)
                    cnt[e] += (v0 + 64 * q < D.V1 && before(zv[e][q], v0 + 64 * q, ztv[e], tt[e])) ? 1 : 0;
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int n = wave + 4 * (j0 + e);
            const int total = wave_sum_i_dpp(cnt[e]);
            if (j0 + e < nj && lane == 0) {
                const int edge = n == 0 ? 1 : (total < tau);
                s_edge[n] = edge;   // stored to memory after the loop: a store inside it would
            }                       // put a write acknowledgement into every wait for the next rows
        }
    }
    __syncthreads();
    for (int n = threadIdx.x; n < D.M; n += 256) stwi(s.edge_ok + b * D.M + n, s_edge[n]);
    dev_choose(D, s, b, ignore_eos, s_edge, s_ok);
}

// Sec. 2.3's choice for sequence b when the edge decisions were taken by other workgroups
// (dev_edge) and sit in edge_ok.
__device__ inline void dev_select(const Dims& D, const DevState& s, int b, int ignore_eos) {
    __shared__ int s_edge[VADUSA_MAX_TREE_NODES];
    __shared__ int s_ok[VADUSA_MAX_TREE_NODES];
    if (s.finished[b]) {
        if (threadIdx.x == 0) stwi(s.path + (size_t)b * (VADUSA_MAX_DRAFT_HEADS + 2), 0);
        return;
    }
    for (int n = threadIdx.x; n < D.M; n += 256) s_edge[n] = s.edge_ok[b * D.M + n];
    __syncthreads();
    dev_choose(D, s, b, ignore_eos, s_edge, s_ok);
}

// Continue from the last accepted node (Sec. 2.1): advance L, append the
// accepted tokens to the output, next root = best logit of that node's row, and
// its final-LayerNorm'd hidden state for the draft heads (copied from hn, or, if
// from_x, computed here from the residual stream).  acc_len[b] keeps the number
// of committed rows for the compaction that follows.  In prefill mode the
// "path" is the chunk's last row and nothing is emitted.
template <class T>
__device__ inline void dev_finalize(const Dims& D, const DevState& s, int b, int prefill_mode, int ignore_eos,
                                    int from_x) {
    __shared__ float s_red[8];
    int32_t* path = s.path + (size_t)b * (VADUSA_MAX_DRAFT_HEADS + 2);
    int cnt, last;
    if (prefill_mode) {
        cnt = s.n_rows[b];
        last = cnt - 1;
    } else {
        cnt = ldci(path);
        last = cnt > 0 ? ldci(path + cnt) : 0;
    }
    if (threadIdx.x == 0) stwi(s.acc_len + b, prefill_mode ? 0 : cnt);
    if (cnt <= 0) return;
    const int32_t* tok = s.tok + (size_t)b * D.M;
    const int r = b * D.M + last;
    const int root = block_argbest(s.logits + (size_t)r * D.V1, D.V1, INFINITY, -1, nullptr);
    T* hb = (T*)s.hbest + (size_t)b * D.d;
    if (from_x) {
        // final LayerNorm of the accepted node's residual row.  The row was written by other
        // workgroups of this launch: coherent loads, once, into registers (up to 16 values per
        // thread, d <= 4096; larger rows take the three-pass route below)
        const float* xr = s.x + (size_t)r * D.d;
        if (D.d <= 4096) {
            float xv[16];
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = threadIdx.x * 2 + 512 * j;
                xv[2 * j] = i < D.d ? ldcf(xr + i) : 0.f;
                xv[2 * j + 1] = i < D.d ? ldcf(xr + i + 1) : 0.f;
                sum += xv[2 * j] + xv[2 * j + 1];
            }
            sum = wave_sum_dpp(sum);
            if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = sum;
            __syncthreads();
            const float mu = (s_red[0] + s_red[1] + s_red[2] + s_red[3]) / D.d;
            float sq = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = threadIdx.x * 2 + 512 * j;
                if (i < D.d) { const float t0 = xv[2 * j] - mu, t1 = xv[2 * j + 1] - mu; sq += t0 * t0 + t1 * t1; }
            }
            sq = wave_sum_dpp(sq);
            if ((threadIdx.x & 63) == 0) s_red[4 + (threadIdx.x >> 6)] = sq;
            __syncthreads();
            const float rstd = rsqrtf((s_red[4] + s_red[5] + s_red[6] + s_red[7]) / D.d + LN_EPS);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = threadIdx.x * 2 + 512 * j;
                if (i < D.d) {
                    const float a = (xv[2 * j] - mu) * rstd * ldg(s.lnf_g + i) + ldg(s.lnf_b + i);
                    const float c2 = (xv[2 * j + 1] - mu) * rstd * ldg(s.lnf_g + i + 1) + ldg(s.lnf_b + i + 1);
                    stw32((bf16_t*)s.hbest + toff(b, i, D.d >> 5), pack_bf16(a, c2));   // tiled for the draft maps
                }
            }
        } else {
        float sum = 0.f;
        for (int i = threadIdx.x; i < D.d; i += 256) sum += ldcf(xr + i);
        sum = wave_sum_dpp(sum);
        if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = sum;
        __syncthreads();
        const float mu = (s_red[0] + s_red[1] + s_red[2] + s_red[3]) / D.d;
        float sq = 0.f;
        for (int i = threadIdx.x; i < D.d; i += 256) { const float t = ldcf(xr + i) - mu; sq += t * t; }
        sq = wave_sum_dpp(sq);
        if ((threadIdx.x & 63) == 0) s_red[4 + (threadIdx.x >> 6)] = sq;
        __syncthreads();
        const float rstd = rsqrtf((s_red[4] + s_red[5] + s_red[6] + s_red[7]) / D.d + LN_EPS);
        for (int i = threadIdx.x * 2; i < D.d; i += 512) {
            const float a = (ldcf(xr + i) - mu) * rstd * s.lnf_g[i] + s.lnf_b[i];
            const float c2 = (ldcf(xr + i + 1) - mu) * rstd * s.lnf_g[i + 1] + s.lnf_b[i + 1];
            stw32((bf16_t*)s.hbest + toff(b, i, D.d >> 5), pack_bf16(a, c2));   // tiled for the draft maps
        }
        }
    } else {
        const T* h = (const T*)s.hn + (size_t)r * D.d;
        for (int i = threadIdx.x; i < D.d; i += 256) hb[i] = h[i];
    }
    if (threadIdx.x == 0) {
        stwi(s.root + b, root);
        stwi(s.L + b, s.L[b] + cnt);
        if (!prefill_mode) {
            int no = s.n_out[b];
            bool fin = false;
            for (int j = 0; j < cnt; ++j) {
                const int t = tok[ldci(path + 1 + j)];
                stwi(s.acc_tok + b * (VADUSA_MAX_DRAFT_HEADS + 1) + j, t);
                if (no < D.maxpos) stwi(s.out_tok + (size_t)b * D.maxpos + no++, t);
                if (t == D.V1 - 1) fin = true;
            }
            stwi(s.n_out + b, no);
            stwi(path, 0);   // consumed
            if (fin && !ignore_eos) stwi(s.finished + b, 1);
        }
    }
}

// KV compaction after dev_finalize: cache row L0 + j <- row L0 + path[j], where
// L0 = L - acc_len is the length before this step and acc_len the number of
// committed rows.  path[j] >= j, so a destination row can be the source of an
// earlier j: every thread owns one column of one head and reads all its sources
// before writing.  64 threads (one per head dimension).
template <class T>
__device__ inline void dev_commit_kv(const Dims& D, const DevState& s, int layer, int b, int head, int dim) {
    const int32_t* path = s.path + (size_t)b * (VADUSA_MAX_DRAFT_HEADS + 2);
    const int cnt = ldci(s.acc_len + b);
    if (cnt <= 0) return;
    const int L0 = ldci(s.L + b) - cnt;
    const size_t hb = ((((size_t)layer * D.Bmax + b) * D.nH + head) * kv_cap(D.maxpos)) * 64;
    T* Kh = (T*)s.Kc + hb;
    T* Vh = (T*)s.Vc + hb;
    T kr[VADUSA_MAX_DRAFT_HEADS + 1], vr[VADUSA_MAX_DRAFT_HEADS + 1];
#pragma unroll
    for (int j = 0; j < VADUSA_MAX_DRAFT_HEADS + 1; ++j)
        if (j < cnt) {
            const int src = ldci(path + 1 + j);
            kr[j] = Kh[kc_off(L0 + src, dim)];
            vr[j] = Vh[vc_off(L0 + src, dim)];
        }
#pragma unroll
    for (int j = 0; j < VADUSA_MAX_DRAFT_HEADS + 1; ++j)
        if (j < cnt) {
            Kh[kc_off(L0 + j, dim)] = kr[j];
            Vh[vc_off(L0 + j, dim)] = vr[j];
        }
}

// The same for nl consecutive layers from layer0 on (the step kernel's compaction units: with many sequences a unit
// takes several layers, so that a workgroup has one unit instead of a chain of them, each a few dependent trips to
// memory).  The path is read once; four layers' rows are in flight together; a path whose rows already sit where they
// belong (the root alone, or nodes 0, 1, .. of the tree) moves nothing.
template <class T>
__device__ inline void dev_commit_kv_layers(const Dims& D, const DevState& s, int layer0, int nl, int b, int head, int dim) {
    constexpr int W = VADUSA_MAX_DRAFT_HEADS + 1, LB = 4;
    const int32_t* path = s.path + (size_t)b * (VADUSA_MAX_DRAFT_HEADS + 2);
    const int cnt = ldci(s.acc_len + b);
    if (cnt <= 0) return;
    const int L0 = ldci(s.L + b) - cnt;
    int src[W];
    bool moves = false;
#pragma unroll
    for (int j = 0; j < W; ++j) {
        src[j] = j < cnt ? ldci(path + 1 + j) : j;
        moves |= src[j] != j;
    }
    if (!moves) return;
    size_t so_k[W], so_v[W], do_k[W], do_v[W];
#pragma unroll
    for (int j = 0; j < W; ++j) {
        so_k[j] = kc_off(L0 + src[j], dim); so_v[j] = vc_off(L0 + src[j], dim);
        do_k[j] = kc_off(L0 + j, dim); do_v[j] = vc_off(L0 + j, dim);
    }
    const size_t lstride = (size_t)D.Bmax * D.nH * kv_cap(D.maxpos) * 64;
    const size_t hb0 = ((((size_t)layer0 * D.Bmax + b) * D.nH + head) * kv_cap(D.maxpos)) * 64;
    for (int l0 = 0; l0 < nl; l0 += LB) {
        T kr[LB][W], vr[LB][W];
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const size_t hb = hb0 + (size_t)(l0 + i < nl ? l0 + i : nl - 1) * lstride;
            const T* Kh = (const T*)s.Kc + hb;
            const T* Vh = (const T*)s.Vc + hb;
#pragma unroll
            for (int j = 0; j < W; ++j)
                if (j < cnt) { kr[i][j] = Kh[so_k[j]]; vr[i][j] = Vh[so_v[j]]; }
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            if (l0 + i >= nl) break;
            const size_t hb = hb0 + (size_t)(l0 + i) * lstride;
            T* Kh = (T*)s.Kc + hb;
            T* Vh = (T*)s.Vc + hb;
#pragma unroll
            for (int j = 0; j < W; ++j)
                if (j < cnt) { Kh[do_k[j]] = kr[i][j]; Vh[do_v[j]] = vr[i][j]; }
        }
    }
}

// Draft list of head i, sequence b: the VADUSA_MAX_TOPK best ids of its logits,
// descending, equal logits: lower id first (Sec. 2.1).
// Up to 4096 logits sit in registers (16 per thread).  The 256 threads form 64 quads; the 64
// quad maxima are distinct entries of the row, so the row's 16th best entry is not after the
// 16th best of them, T.  Every entry not after T is a candidate (two dozen for random logits);
// each candidate counts the candidates before it, which is its place in the list.
// More than 256 candidates (many equal or missing values), or more than 4096 logits: the
// list is built one entry per round by re-scanning (block_argbest); with SLICED, rows of up to
// 65536 logits first try the candidate scheme slice by slice (used by the stand-alone top-k
// kernel, which serves large vocabularies).
template <bool SLICED = false>
__device__ inline void dev_topk(const Dims& D, const DevState& s, int i, int b) {
    __shared__ float c_v[256];
    __shared__ int c_i[256];
    __shared__ float g_v[64];
    __shared__ int g_i[64];
    __shared__ int c_n;
    __shared__ float t_v;
    __shared__ int t_i;
    const float* z = s.zdraft + ((size_t)i * D.Bmax + b) * D.V1;
    int32_t* out = s.draft_topk + ((size_t)b * D.Hh + i) * VADUSA_MAX_TOPK;
    const int kmax = D.V1 < VADUSA_MAX_TOPK ? D.V1 : VADUSA_MAX_TOPK;
    bool rescan = D.V1 > 256 * 16;
    if constexpr (SLICED) {
        if (rescan) {
            // More than 4096 logits: the same scheme over slices of 4096.  First pass: the 16 group
            // maxima of every slice go to LDS (at most 256 of them: V1 <= 65536) and T is the 16th
            // best of these, again an entry of the row with at least 15 others before it.  Second
            // pass: every entry not after T is a candidate.
            const int nsl = (D.V1 + 4095) / 4096;
            if (nsl <= 16) {
                for (int sl = 0; sl < nsl; ++sl) {
                    float lv = -INFINITY;
                    int li = 0x7fffffff;
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const int v = sl * 4096 + (int)threadIdx.x + 256 * j;
                        const float zv = v < D.V1 ? ldg(z + v) : -INFINITY;
                        if (v < D.V1 && before(zv, v, lv, li)) { lv = zv; li = v; }
                    }
#pragma unroll
                    for (int o = 1; o < 16; o <<= 1) {
                        const float ov = __shfl_xor(lv, o, 64);
                        const int oi = __shfl_xor(li, o, 64);
                        if (before(ov, oi, lv, li)) { lv = ov; li = oi; }
                    }
                    if ((threadIdx.x & 15) == 0) { c_v[sl * 16 + (threadIdx.x >> 4)] = lv; c_i[sl * 16 + (threadIdx.x >> 4)] = li; }
                }
                if (threadIdx.x == 0) c_n = 0;
                __syncthreads();
                // thread t ranks maximum t among the nsl * 16 maxima; the one 15 are before is T
                // (a slice tail without entries leaves (-inf, 0x7fffffff), which ranks last)
                const int nm = nsl * 16;
                if ((int)threadIdx.x < nm) {
                    const float mv = c_v[threadIdx.x];
                    const int mi = c_i[threadIdx.x];
                    int r = 0;
                    for (int t = 0; t < nm; ++t) r += before(c_v[t], c_i[t], mv, mi) ? 1 : 0;
                    if (r == 15) { g_v[0] = mv; g_i[0] = mi; }
                }
                __syncthreads();
                const float tv = g_v[0];
                const int ti = g_i[0];
                __syncthreads();   // every thread holds T: the candidate list may overwrite the maxima
                for (int sl = 0; sl < nsl; ++sl) {
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const int v = sl * 4096 + (int)threadIdx.x + 256 * j;
                        const float zv = v < D.V1 ? ldg(z + v) : -INFINITY;
                        if (v < D.V1 && !before(tv, ti, zv, v)) {
                            const int slot = atomicAdd(&c_n, 1);
                            if (slot < 256) { c_v[slot] = zv; c_i[slot] = v; }
                        }
                    }
                }
                __syncthreads();
                const int n = c_n;
                if (n <= 256) {
                    rescan = false;
                    if ((int)threadIdx.x < n) {
                        const float mv = c_v[threadIdx.x];
                        const int mi = c_i[threadIdx.x];
                        int r = 0;
                        for (int t = 0; t < n; ++t) r += before(c_v[t], c_i[t], mv, mi) ? 1 : 0;
                        if (r < kmax) stwi(out + r, mi);
                    }
                }
                __syncthreads();
            }
        }
    }
    if (D.V1 <= 256 * 16) {
        float zr[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int v = threadIdx.x + 256 * j;
            zr[j] = v < D.V1 ? ldg(z + v) : -INFINITY;
        }
        float lv = -INFINITY;
        int li = 0x7fffffff;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int v = threadIdx.x + 256 * j;
            if (v < D.V1 && before(zr[j], v, lv, li)) { lv = zr[j]; li = v; }
        }
        // best of each quad: 64 group maxima (fewer for fewer than 253 logits; empty groups leave
        // (-inf, 0x7fffffff), which ranks after every real entry)
        argbest_step<0xB1>(lv, li);
        argbest_step<0x4E>(lv, li);
        if ((threadIdx.x & 3) == 0) { g_v[threadIdx.x >> 2] = lv; g_i[threadIdx.x >> 2] = li; }
        if (threadIdx.x == 0) { c_n = 0; t_v = -INFINITY; t_i = 0x7fffffff; }   // default T: keep everything
        __syncthreads();
        // T = the 16th best of the group maxima: an entry of the row with at least 15 others before
        // it, so the row's 16th best is not after T.  Wave 0 ranks the 64 maxima against each other
        // with lane broadcasts (no LDS traffic in the loop).  With fewer than 16 real maxima T stays
        // at its default.
        if (threadIdx.x < 64 && D.V1 >= 64) {
            const float gv = g_v[threadIdx.x];
            const int gi = g_i[threadIdx.x];
            int r = 0;
            for (int j = 0; j < 64; ++j) {
                const float bv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(gv), j));
                const int bi = __builtin_amdgcn_readlane(gi, j);
                r += before(bv, bi, gv, gi) ? 1 : 0;
            }
            if (r == 15) { t_v = gv; t_i = gi; }
        }
        __syncthreads();
        const float tv = t_v;
        const int ti = t_i;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int v = threadIdx.x + 256 * j;
            if (v < D.V1 && !before(tv, ti, zr[j], v)) {
                const int slot = atomicAdd(&c_n, 1);
                if (slot < 256) { c_v[slot] = zr[j]; c_i[slot] = v; }
            }
        }
        __syncthreads();
        const int n = c_n;
        if (n <= 64) {
            // the usual case (a few dozen candidates): wave 0 holds one candidate per lane and ranks
            // them against each other with lane broadcasts; a candidate's rank is its place in the list
            if (threadIdx.x < 64) {
                const bool have = (int)threadIdx.x < n;
                const float mv = have ? c_v[threadIdx.x] : -INFINITY;
                const int mi = have ? c_i[threadIdx.x] : 0x7fffffff;
                int r = 0;
                for (int j = 0; j < n; ++j) {
                    const float bv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mv), j));
                    const int bi = __builtin_amdgcn_readlane(mi, j);
                    r += before(bv, bi, mv, mi) ? 1 : 0;
                }
                if (have && r < kmax) stwi(out + r, mi);
            }
        } else if (n <= 256) {
            if ((int)threadIdx.x < n) {
                const float mv = c_v[threadIdx.x];
                const int mi = c_i[threadIdx.x];
                int r = 0;
                for (int t0 = 0; t0 < n; t0 += 8) {   // eight candidates per round: LDS reads overlap
                    float cv[8];
                    int ci[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) { cv[q] = c_v[(t0 + q) & 255]; ci[q] = c_i[(t0 + q) & 255]; }
#pragma unroll
                    for (int q = 0; q < 8; ++q) r += (t0 + q < n && before(cv[q], ci[q], mv, mi)) ? 1 : 0;
                }
                if (r < kmax) stwi(out + r, mi);
            }
        } else {
            rescan = true;   // n is the same for every thread
        }
        __syncthreads();     // the LDS arrays are free for the next unit
    }
    if (rescan) {
        float pv = INFINITY;
        int pi = -1;
        for (int k = 0; k < kmax; ++k) {
            float bv;
            const int bi = block_argbest(z, D.V1, pv, pi, &bv);
            if (threadIdx.x == 0) stwi(out + k, bi);
            pv = bv; pi = bi;
        }
    }
}
