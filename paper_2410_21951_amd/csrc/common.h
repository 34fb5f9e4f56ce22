// Internal declarations shared by the HIP translation units of libvadusa.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "vadusa.h"

typedef uint16_t bf16_t;   // raw bfloat16 bits

#define MASK_WORDS (VADUSA_MAX_TREE_NODES / 32)
#define LN_EPS 1e-5f

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);   // round to nearest, ties to even
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const bf16_t* p) { return bf2f(*p); }
__device__ __forceinline__ void stf(float* p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t* p, float v) { *p = f2bf(v); }

// Every pointer the kernels dereference points into device (global) memory.  A pointer that
// reaches a function as an argument, or is read from a parameter block in LDS, is a generic
// pointer to the compiler and would be accessed with FLAT instructions (slower to issue, and
// tied to the LDS counter as well); the helpers below state the address space.
#if defined(__HIP_DEVICE_COMPILE__)
#define VADUSA_GLOBAL __attribute__((address_space(1)))
#else
#define VADUSA_GLOBAL
#endif
template <class T>
__device__ __forceinline__ T ldg(const T* p) { return *(const VADUSA_GLOBAL T*)p; }   // scalar T only
// A pointer that is the same in every lane (read from the parameter block, derived from the unit
// number): moved to scalar registers, so that loads can use "scalar base + lane offset" addresses.
template <class T>
__device__ __forceinline__ T* uniform_ptr(T* p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (T*)(((uint64_t)hi << 32) | lo);
}
// Makes a loaded value count as used (the load stays, and is waited for here) without storing it anywhere.
__device__ __forceinline__ void keep_alive(uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" : : "v"(v));
#else
    (void)v;
#endif
}
// 8- and 16-byte loads (HIP's uint2 / uint4 / float2 are classes: their copy would go back to a generic reference)
typedef uint32_t vadusa_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t vadusa_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 ldg4(const void* p) {
    const vadusa_u32x4 v = *(const VADUSA_GLOBAL vadusa_u32x4*)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 ldg2(const void* p) {
    const vadusa_u32x2 v = *(const VADUSA_GLOBAL vadusa_u32x2*)p;
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ float2 ldgf2(const void* p) {
    const vadusa_u32x2 v = *(const VADUSA_GLOBAL vadusa_u32x2*)p;
    return make_float2(__uint_as_float(v.x), __uint_as_float(v.y));
}

// Stores / loads that are coherent across the whole GPU without cache maintenance
// (write-through to / read from the memory side).  The persistent step kernel uses them
// for every value that crosses workgroups inside one launch.
__device__ __forceinline__ void stw32(void* p, uint32_t v) {
    __hip_atomic_store((VADUSA_GLOBAL uint32_t*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void stw64(void* p, uint64_t v) {
    __hip_atomic_store((VADUSA_GLOBAL uint64_t*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16 bytes at once (no atomic type is that wide: the store instruction itself, with the same agent-scope bit; the
// compiler does not count it among the outstanding memory operations, which only makes its later waits stricter).
// A store of more than 8 bytes reads its data registers a little after it issues, and a vector instruction that
// overwrites them must keep two wait states' distance: the compiler inserts those after the stores it knows, not
// after inline assembly, so they are part of the statement.
__device__ __forceinline__ void stw128(void* p, uint4 v) {
#if defined(__HIP_DEVICE_COMPILE__)
    typedef uint32_t u32x4_st __attribute__((ext_vector_type(4)));
    const u32x4_st d = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(d) : "memory");
#else
    *(uint4*)p = v;
#endif
}
__device__ __forceinline__ void stw16(void* p, uint16_t v) {
    __hip_atomic_store((VADUSA_GLOBAL uint16_t*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void stwi(int32_t* p, int32_t v) { stw32(p, (uint32_t)v); }
__device__ __forceinline__ void stwf(float* p, float v) { stw32(p, __float_as_uint(v)); }
__device__ __forceinline__ void stwf2(float* p, float a, float b) {
    stw64(p, (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32));
}
__device__ __forceinline__ int32_t ldci(const int32_t* p) {
    return __hip_atomic_load((const VADUSA_GLOBAL int32_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ldcf(const float* p) {
    return __uint_as_float(__hip_atomic_load((const VADUSA_GLOBAL uint32_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
// Offset of element (r, k) of a bf16 activation matrix kept in MFMA-operand tiles:
// [row tile of 16][k-step of 32][lane = (r & 15) + 16 * ((k & 31) >> 3)][k & 7], nks = K / 32.
// A wave reads one (row tile, k-step) as the A operand with one contiguous KiB load.
__device__ __forceinline__ size_t toff(int r, int k, int nks) {
    return ((size_t)((r >> 4) * nks + (k >> 5)) * 64 + (r & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}
// KV cache of one (layer, sequence, head): kv_cap(max_positions) positions (whole blocks of 32) x 64 dimensions,
// kept in the operand tiles of the attention units, so that every operand of a 32-key block is one contiguous KiB
// per wave load (a row-major cache makes such a load touch 16 cache lines and use half of each):
//   K: [block of 32 keys][key tile t][k-step s][lane][8]: key k = pos & 31 sits in tile t = (k >> 2) & 1 (tile 0:
//      keys 0-3, 8-11, 16-19, 24-27 of the block; tile 1: the others) at row c = ((k >> 3) << 2) | (k & 3); k-step
//      s = dim >> 5; lane = c + 16 * ((dim & 31) >> 3).  (With this row order the lane that holds query c's scores
//      after S^T = K Q^T holds them for eight consecutive keys: exactly a B fragment of P^T for O^T += V^T P^T.)
//   V: [block of 32 keys][dimension tile dt = dim >> 4][lane][8]: lane = (dim & 15) + 16 * ((pos & 31) >> 3),
//      element pos & 7 (V transposed: a lane holds eight consecutive positions of one dimension).
__host__ __device__ inline int kv_cap(int maxpos) { return (maxpos + 31) & ~31; }
__host__ __device__ inline size_t kc_off(int pos, int dim) {
    const int k = pos & 31, t = (k >> 2) & 1, c = ((k >> 3) << 2) | (k & 3);
    return (size_t)(pos >> 5) * 2048 + (size_t)(((t * 2 + (dim >> 5)) * 64 + c + 16 * ((dim & 31) >> 3)) * 8 + (dim & 7));
}
__host__ __device__ inline size_t vc_off(int pos, int dim) {
    return (size_t)(pos >> 5) * 2048 + (size_t)((((dim >> 4) * 64) + (dim & 15) + 16 * ((pos & 31) >> 3)) * 8 + (pos & 7));
}
// Two floats to a pair of bf16 (round to nearest even): one v_cvt_pk_bf16_f32 on the device.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_cvt;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_cvt;
    const f32x2_cvt v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_cvt));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// The same sums without LDS traffic: DPP lane permutations inside each row of 16 lanes (swap
// with the quad neighbour, the other pair of the quad, the mirrored half row, the mirrored row:
// after each step twice as many lanes hold the same partial sum), then the four row sums are
// read from lanes 0, 16, 32 and 48.  Every lane returns the total; all 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ int dpp_perm(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false); }
// sums over the 4 lanes of a quad and over the 16 lanes of a row; every lane gets the total.  The
// additions pair the same values as an xor-butterfly of __shfl_xor would, so the results are the same bits.
__device__ __forceinline__ float quad_sum(float v) {
    v += __int_as_float(dpp_perm<0xB1>(__float_as_int(v)));
    v += __int_as_float(dpp_perm<0x4E>(__float_as_int(v)));
    return v;
}
__device__ __forceinline__ float pair_sum(float v) { return v + __int_as_float(dpp_perm<0xB1>(__float_as_int(v))); }
__device__ __forceinline__ float row16_sum(float v) {
    v = quad_sum(v);
    v += __int_as_float(dpp_perm<0x141>(__float_as_int(v)));
    v += __int_as_float(dpp_perm<0x140>(__float_as_int(v)));
    return v;
}
// Combining a value with the ones 16 and 32 lanes away (the four rows of a wave), every lane gets
// the result.  gfx950 swaps rows between two registers in the vector ALU: with both operands the
// same value, one register then holds rows {0, 0, 2, 2} and the other rows {1, 1, 3, 3} (16-lane
// swap), or halves {lo, lo} and {hi, hi} (32-lane swap), and combining the two registers lane by
// lane is the exchange, without a trip through the LDS permute unit.
typedef unsigned int vadusa_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float rows_max(float v) {
    vadusa_u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float rows_sum(float v) {
    vadusa_u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(r.x) + __uint_as_float(r.y);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r.x) + __uint_as_float(r.y);
}
__device__ __forceinline__ int wave_sum_i_dpp(int v) {
    v += dpp_perm<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_perm<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_perm<0x141>(v);   // row_half_mirror
    v += dpp_perm<0x140>(v);   // row_mirror
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
           __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}
__device__ __forceinline__ float wave_sum_dpp(float v) {
    v += __int_as_float(dpp_perm<0xB1>(__float_as_int(v)));
    v += __int_as_float(dpp_perm<0x4E>(__float_as_int(v)));
    v += __int_as_float(dpp_perm<0x141>(__float_as_int(v)));
    v += __int_as_float(dpp_perm<0x140>(__float_as_int(v)));
    return (__int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0)) +
            __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32)) +
            __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48)));
}

// Shapes that every kernel needs (passed by value).
struct Dims {
    int Ly, d, nH, F, V1, Hh, maxpos, Bmax, Mmax;   // model / capacity
    int B, M;                                        // current batch, rows per sequence
};

// Pointers to one layer's parameters on the device.
struct LayerW {
    const float *ln1_g, *ln1_b, *bqkv, *bo, *ln2_g, *ln2_b, *b1, *b2;
    const void *Wqkv, *Wo, *W1, *W2;   // element type follows the context dtype
    // bf16 model only: LayerNorm folded into the following linear map (see k_step.hip)
    float *cs_qkv, *t_qkv, *cs_w1, *t_w1;
};
struct DraftW {
    const void* W1; const float* b1; const void* W2;
};

// Decoding state and scratch on the device (all inside the caller's arena).
struct DevState {
    // model
    const void *E_text, *E_speech, *P;
    const float *lnf_g, *lnf_b;
    const void* W_out;
    float *cs_out, *t_out;          // bf16 model: folded final LayerNorm for the vocabulary map
    const LayerW* layers_dev;       // bf16 model: the layer table in device memory
    const DraftW* draft_dev;
    // KV cache, element type = dtype: K [Ly][Bmax][nH][maxpos][64], V [Ly][Bmax][nH][64][maxpos]
    void *Kc, *Vc;
    // activations
    float* x;        // [R][d]  residual stream
    // bf16 model, persistent step kernel.  Buffers that cross workgroups are written once
    // per launch, so there is one instance per producer: xb / stats have 2*Ly+1 slots
    // (embedding, then after the out-projection and after FFN2 of every layer), q / att /
    // hid one slot per layer.  Slot strides are in elements.
    bf16_t* xb;      // [2Ly+1][R][d]  bf16 copy of the residual stream
    float* stats;    // [2Ly+1][d/16][R][2] per 16-column tile: mean, sum of squared deviations
    size_t act_stride, stats_stride, hid_stride, draft_stride;   // rows padded to a multiple of 16
    uint32_t* bar;   // grid barrier: VADUSA_BAR_WORDS words; counters 64 words apart: 8 group counters, then 8 copies of the top counter
    int32_t* kerr;   // [4] error flag raised by a kernel (barrier time-out)
    const uint32_t* gtab;   // bf16 model: [5][VADUSA_GREC_WORDS] descriptors of the layers' linear maps (null: none)
    long long* tprof; // [128][8] timing points of workgroup 0 in the last launch (device clock, 100 MHz)
    void* xn;        // [R][d]  LayerNorm output
    void* q;         // [R][d]   (bf16 model: one slot per layer)
    void* att;       // [R][d]   (bf16 model: one slot per layer)
    void* hid;       // [R][F]   (bf16 model: one slot per layer)
    void* hn;        // [R][d]  final-LayerNorm'd node states
    float* logits;   // [R][V1]
    void* hbest;     // [Bmax][d]
    void* rdraft;    // [Hh][Bmax][d]
    float* zdraft;   // [Bmax][Hh][V1]
    // integer state
    int32_t *L, *root, *finished, *draft_topk /*[Bmax][Hh][MAX_TOPK]*/;
    int32_t *tok /*[R]*/, *n_rows /*[Bmax]*/, *edge_ok /*[R]*/, *path /*[Bmax][MAX_DRAFT_HEADS+2]*/;
    int32_t *out_tok /*[Bmax][maxpos]*/, *n_out /*[Bmax]*/;
    int32_t *acc_tok /*[Bmax][MAX_DRAFT_HEADS+1]*/, *acc_len /*[Bmax]*/;
    int32_t *chunk_tok /*[R]*/, *override_topk /*[Bmax][Hh][MAX_TOPK]*/;
    // tree tables (index 0: current tree, 1: causal chunk used by prefill)
    int32_t *t_parent[2], *t_depth[2], *t_rank[2];
    uint32_t* t_mask[2];   // [Mmax][MASK_WORDS]
    float* staging;        // weight conversion staging
};

struct vadusa_ctx {
    vadusa_config cfg;
    hipStream_t stream;
    char* arena;
    size_t arena_bytes;
    DevState s;
    std::vector<LayerW> layers;
    std::vector<DraftW> draft;
    size_t elem;                 // bytes per stored element (4 or 2)
    int state;                   // 0 created, 1 weights loaded, 2 ready, 3 verification pending
    int batch;                   // current batch
    int M;                       // nodes of the pending / last verification
    std::vector<int32_t> L_ub;   // host upper bound of each sequence's committed length
    std::vector<char> pending;   // per sequence: verification waits for compaction
    std::vector<int32_t> tree_parent, tree_rank, tree_depth;   // last uploaded tree
    size_t staging_floats;
    int n_cus;                   // workgroups of the persistent step kernel (one per compute unit)
    int persistent;              // 0: one launch per phase (debugging aid)
    int profile;                 // 1: the step kernel records timing points (environment VADUSA_PHASE_CLOCK)
    float* uniforms;             // [max_batch * max_tree_nodes][V+1]: the caller's random numbers of a stochastic step
    float* scores;               // same shape: perturbed scores that replace the logits in such a step
    int sampled;                 // the pending / last verification was a stochastic one
    int gtab_ready;              // the descriptor table of the layer maps has been written (after the weights are placed)
    int big_min, allq_min;       // StepParams::big_min, allq_min (environment VADUSA_BIG_MIN_UNITS sets both, for tests of small shapes)
    uint32_t epoch;              // grid-barrier epoch reached so far
    int errored;                 // a step kernel gave up at a grid barrier: every call but vadusa_prefill refuses until that resets the context
    std::string err;
};

// Epilogues of the linear-map kernels.
enum {
    EPI_STORE = 0,      // out[r][n] = acc + bias              (stored in the context dtype)
    EPI_GELU = 1,       // out[r][n] = gelu(acc + bias)
    EPI_RESID = 2,      // x[r][n] += acc + bias               (fp32 residual stream)
    EPI_F32 = 3,        // outf[r][n] = acc (+ bias if given)
    EPI_SILU_RESID = 4, // out[r][n] = in[r][n] + silu(acc + bias)   (needs N == K)
    EPI_QKV = 5         // n < d: q[r][n]; else key / value rows of the KV cache at L[b] + node
};

struct GemmArgs {
    const void* X;      // [R][K] context dtype
    const void* W;      // [N][K] context dtype (layout depends on the kernel)
    const float* bias;  // [N] or null
    int R, K, N;
    int epi;
    void* out;          // context dtype, [R][N]
    float* outf;        // fp32 target (EPI_RESID: x, EPI_F32: logits)
    // EPI_QKV
    void *Kc, *Vc;      // layer base of the cache
    const int32_t* L;
    int M, nH, maxpos, d;
};

// Parameters of the persistent step kernel (bf16 model).
struct StepParams {
    Dims D;
    DevState s;
    int table;          // which tree table the rows use (0 tree, 1 causal chunk)
    int prefill_mode;
    int tau, ignore_eos;
    int ph_lo, ph_hi;   // phases to run: [ph_lo, ph_hi)
    int persistent;     // 1: one cooperative launch with grid barriers between phases
    int wide;           // 1: B * M >= 256 rows: the layer maps and the base head use 64 x 64 output tiles
    int mid;            // 1: 65 to 255 rows: QKV / FFN1 in 64 x 32 units, out-projection / FFN2 in 32 x 16 units
    int profile;        // n > 0: workgroup n - 1 records timing points (costs a few hundred ns each)
    uint32_t epoch;     // barrier epoch before the first barrier of this launch
    int seq0, nseq;     // sequences the compaction phases act on
    // Every layer's parameters sit at the same offsets from the previous layer's:
    // layer l = layer 0 advanced by l * lw_stride bytes (likewise the draft heads), so no
    // kernel has to fetch a parameter table from memory before it can address its weights.
    LayerW lw0;
    DraftW dw0;
    size_t lw_stride, dw_stride;
    int big_min;        // many-row kernel: a map takes 128 x 128 units if it has at least this many of them
    int allq_min;       // many-row kernel: an attention unit is a whole (sequence, head) if there are at least this many
    int topk_apart;     // 1: the last phase only compacts the KV cache; the draft lists come from the stand-alone top-k kernel
    int fuse_select;    // 1: the continuation units choose their sequence's path themselves (the selection phase has no units)
};
// Phases of the step kernel after the decoder layers, as offsets from H = 1 + 5 * n_layers.
// TP_COMMIT: first map of the draft heads; TP_TOPK: draft lists and, beside them (most workgroups
// are idle in that phase), the compaction of the KV cache.
enum { TP_HEAD = 0, TP_EDGES, TP_SELECT, TP_FINAL, TP_COMMIT, TP_DRAFT2, TP_TOPK, TP_COUNT };
int step_num_phases(int n_layers);
// Phases of [ph_lo, ph_hi) that have units: a phase without units is skipped together with its grid barrier, so a
// persistent launch passes this many barriers less one.
int step_live_phases(const StepParams& p);
// words of DevState::bar, the grid barrier's counters (16 of them, 64 words apart)
#define VADUSA_BAR_WORDS 4096
// One record per kind of layer phase: everything about a linear map that does not depend on the
// launch (operand and result pointers of layer 0 with their advance per layer, K, N, epilogue),
// written once per context by launch_build_gtab from the same code that otherwise derives it per unit.
#define VADUSA_GREC_WORDS 32
void launch_build_gtab(const StepParams& p, uint32_t* tab, hipStream_t st);
// phase index: 0 embed; 1+5l.. layer l (qkv, attn, wo, ffn1, ffn2); then H + TP_*
void launch_step(const StepParams& p, int n_cus, hipStream_t st, hipError_t* err);
void launch_pack_w_ln(const float* src, const float* gamma, const float* beta, void* dst, float* colsum,
                      float* tvec, int N, int K, hipStream_t st);
void launch_add_vec(float* dst, const float* src, int n, hipStream_t st);

// ---- launch wrappers (each enqueues on `st`, no synchronisation) ----
void launch_embed(const Dims& D, const DevState& s, int dtype, int prefill_mode, int table, hipStream_t st);
void launch_layernorm(const float* x, const float* g, const float* b, void* out, int R, int d, int dtype, hipStream_t st);
void launch_gemm_simple(const GemmArgs& a, int dtype, hipStream_t st);
void launch_pack_w(const float* src, void* dst, int N, int K, hipStream_t st);
void launch_attn_simple(const Dims& D, const DevState& s, int layer, int table, int dtype, hipStream_t st);
void launch_accept(const Dims& D, const DevState& s, int tau, int ignore_eos, hipStream_t st);
void launch_commit_kv(const Dims& D, const DevState& s, int seq0, int nseq, int dtype, hipStream_t st);
void launch_finalize(const Dims& D, const DevState& s, int seq0, int nseq, int prefill_mode, int ignore_eos, int dtype, hipStream_t st);
void launch_topk(const Dims& D, const DevState& s, int seq0, int nseq, hipStream_t st);
void launch_perturb(const float* logits, const float* u, float* scores, int rows, int V1, float temperature,
                    float top_p, int tau, hipStream_t st);
void launch_convert(const float* src, void* dst, size_t n, int dtype, hipStream_t st);
void launch_advance(const DevState& s, int B, hipStream_t st);
void launch_read_kv(const Dims& D, const void* cache_layer, int seq, int which, int pos0, int npos, float* out, int dtype, hipStream_t st);
void launch_to_float(const void* src, float* dst, size_t n, int dtype, hipStream_t st);
