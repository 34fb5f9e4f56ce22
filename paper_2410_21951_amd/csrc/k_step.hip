// The speculative step of the bf16 model as ONE persistent kernel.
//
// A step is a fixed sequence of phases; every phase is a set of independent
// units that the workgroups of the grid take round-robin, and a grid barrier
// separates dependent phases.  Phases:
//   0                 embed: tree expansion + token/position embedding (Sec. 2.1)
//   1+5l .. 5+5l      layer l: QKV, attention, out-projection, FFN1, FFN2
//   H = 1+5*Ly        base head (logits of every node; Algorithm 1 line 1)
//   H+1               acceptance: Algorithm 1 on every edge, one wave per edge
//   H+2               Sec. 2.3 path choice per sequence (a phase of its own only in a launch that ends with it;
//                     otherwise the continuation unit chooses the path, and a phase without units is skipped
//                     together with its barrier)
//   H+3               continuation from the last accepted node (Sec. 2.1)
//   H+4               draft heads, first map
//   H+5               draft heads, vocabulary map
//   H+6               draft top-k lists || KV compaction to the accepted path
//
// Linear maps stream pre-tiled bf16 weights straight from HBM into the B
// operand of v_mfma_f32_16x16x32_bf16 and the activations (kept in memory in A-operand tiles) from L2
// likewise; the many-row kernel's 128 x 128 units stage both through LDS.
// LayerNorm is folded into the map that follows it:
//   LN(x) W^T = rstd * (x (g*W)^T - mu * colsum(g*W)) + (beta W^T + bias),
// so the map reads the bf16 copy of the raw residual stream and applies the
// row statistics in its epilogue.  The statistics are produced, per 16-column
// tile, by whoever wrote the residual stream (exact fp32 values), and merged
// by the consumer (mean of the tile means; squared deviations = the tiles' own plus 16 x the
// spread of the tile means, summed as distances from the row's first tile mean).
// No atomics combine data: results are bit-reproducible.
//
// Coherence inside the one launch: the eight XCDs have private L2 caches and a
// cache write-back / invalidate at every barrier costs several microseconds.
// Instead every value that crosses workgroups is stored write-through (agent
// scope) into a buffer that is written exactly once per launch and was never
// read before in this launch (one activation slot per layer), so a plain cached
// load after the barrier can only miss and fetch the fresh line.  Values that
// are re-read after having been cached (L, the residual row of the accepted
// node) are loaded at agent scope.  (Hence warm_kv, which reads cache blocks ahead of the attention phase,
// touches only blocks that no row of the step is written into.)
#include <algorithm>
#include <cstdlib>

#include <type_traits>
#include "accept_dev.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

#define ST_TILE_BYTES (20 * 1024)           // reduction buffer of the linear maps (16 KiB), attention merge buffers
#define ST_LDS_BYTES (ST_TILE_BYTES + 1024)  // + row statistics
#define ST_MID_TILE_BYTES (32 * 1024)       // reduction buffer of the 64 x 32 units (65 to 255 rows): 4 waves x 8 tiles x 1 KiB
#define ST_MID_LDS_BYTES (ST_MID_TILE_BYTES + 1024)
#define ST_WIDE_TILE_BYTES (64 * 1024)      // reduction buffer of the 64 x 64 units: 4 waves x 16 tiles x 1 KiB
#define ST_WIDE_LDS_BYTES (ST_WIDE_TILE_BYTES + 1024)
#define ST_SPIN_LIMIT (1 << 22)

enum { SE_QKV = 0, SE_GELU, SE_LOGITS, SE_RESID, SE_SILU_RESID, SE_F32 };

struct GemmD {
    const bf16_t* X;      // [R][K]
    int K, N, R;
    const uint4* Wp;      // packed weights
    const float* bias;    // [N] or null (LN-folded maps: beta W^T + bias)
    const float* colsum;  // [N], LN-folded maps only
    const float* stats;   // [K/16][R][2] statistics of X's rows, or null: no LayerNorm
    int epi;
    bf16_t* out;          // SE_GELU / SE_SILU_RESID / SE_QKV (q)
    float* outf;          // SE_LOGITS / SE_F32
    float* stats_out;     // SE_RESID
    int layer;
    int ph;               // phase index (timing points only)
    int G;                // 64-row-kernel units only: column tiles per unit (4: 64 x 64 unit; 8: 128 x 128 unit)
};

// The kernel's parameters, copied once per workgroup from the kernel-argument segment (which
// may live in host memory) into LDS.  Every device function reads them from here.
__shared__ StepParams sP;
// Committed length and row count of the first ST_SEQ_CACHE sequences, read once per launch: both
// are fixed while the decoder layers run (the continuation phase advances L after them), and the
// attention units need them before they can ask for their first key block.
#define ST_SEQ_CACHE 256
__shared__ int s_seqL[ST_SEQ_CACHE], s_seqRows[ST_SEQ_CACHE];

// GELU with the exact (erf) definition; erf by the rational approximation 7.1.26 of Abramowitz &
// Stegun (absolute error below 1.5e-7, the size of an fp32 rounding of the result, which is then
// stored as bf16): one exponential, one reciprocal and a fifth-degree polynomial instead of the
// library routine's two branches.
__device__ __forceinline__ float gelu_s(float v) {
    const float x = fabsf(v) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(1.f + 0.3275911f * x);   // one instruction, 1 ulp: far below the approximation's own error
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float erfc_x = poly * __expf(-x * x);            // 1 - erf(|x|)
    const float one_plus_erf = v < 0.f ? erfc_x : 2.f - erfc_x;
    return 0.5f * v * one_plus_erf;
}
__device__ __forceinline__ float silu_s(float v) { return v / (1.f + __expf(-v)); }

// ---------------------------------------------------------------------------
// phase bookkeeping (host and device)
// ---------------------------------------------------------------------------
__host__ __device__ inline int cdiv(int a, int b) { return (a + b - 1) / b; }
// Units of a linear map are numbered (row block) * pad8(column tiles) + column tile: workgroup i
// runs on XCD i mod 8, so the row blocks that share a weight tile share an XCD and its L2, and
// the tile leaves HBM once.  Numbers whose column tile is padding are empty units.
__host__ __device__ inline int pad8(int a) { return (a + 7) & ~7; }

int step_num_phases(int n_layers) { return 1 + 5 * n_layers + TP_COUNT; }

// Maps of the many-row kernel with at least StepParams::big_min 128 x 128 output units (more than half the compute
// units) take those (operands staged through LDS and shared by the four waves); smaller ones keep the 64 x 64 units
// whose waves split the reduction.  The base head (its epilogue stores single floats of rows that are not 16-byte
// aligned, which a 128 x 128 unit does 64 times per lane) takes them only with one per compute unit (allq_min).
__host__ __device__ inline bool wide_big(int R, int N, int min_units) { return cdiv(R, 128) * cdiv(N, 128) >= min_units; }
// Attention units of the many-row kernel are whole (sequence, head)s once there is one per compute unit
// (up to four query tiles: one per wave).
__host__ __device__ inline bool attn_allq(const StepParams& P) { return P.wide && P.D.M <= 64 && P.D.B * P.D.nH >= P.allq_min; }
// (sequence, head) pairs per whole-head attention unit: a tree of up to 32 (16) nodes has two (one) query tiles, so a
// workgroup's four waves can take two (four) pairs, each wave a query tile over all its key blocks, as long as that
// still leaves a unit for every compute unit; otherwise the waves that a pair does not need split its key blocks.
__host__ __device__ inline int attn_ppu(const StepParams& P) {
    const int n_qt = (P.D.M + 15) >> 4;
    int ppu = n_qt >= 3 ? 1 : n_qt == 2 ? 2 : 4;
    while (ppu > 1 && cdiv(P.D.B * P.D.nH, ppu) < P.allq_min) ppu >>= 1;
    return ppu;
}
// Few-row kernel, maps with more than 32 rows whose width is a multiple of 32 (QKV, FFN1): units
// of 32 rows x 32 columns instead of 64 x 16.  What bounds such a phase is the bytes the compute
// units pull through L2 (every unit reads its rows of X and its columns of W over the whole K):
// a square unit needs (32 + 32) K values for the same 1024 outputs, not (64 + 16) K.
__host__ __device__ inline bool sq_units(const StepParams& P, int N) { return !P.wide && P.D.B * P.D.M > 32 && N % 32 == 0; }
// Units of the last phase that rank the draft heads' logits (none when a stand-alone kernel does it).
__host__ __device__ inline int topk_units(const StepParams& P) { return P.topk_apart ? 0 : P.D.Hh * P.D.B; }
// Layers per KV compaction unit (a unit: four heads of one sequence): one in the few-row kernels and while all units of
// the step fit one round of the 256 workgroups, more with more sequences, so that a workgroup still has a single unit.
__host__ __device__ inline int commit_layers(const StepParams& P) {
    if (!P.wide) return 1;
    const int per_layer = cdiv(P.D.nH, 4) * P.nseq;
    const int lg = cdiv(P.D.Ly * per_layer, 256);
    return lg < 1 ? 1 : lg > P.D.Ly ? P.D.Ly : lg;
}
__host__ __device__ inline int phase_units(const StepParams& P, int ph) {
    const Dims& D = P.D;
    const int R = D.B * D.M, RG = cdiv(R, 64), RB = cdiv(R, 16), H = 1 + 5 * D.Ly;
    if (ph == 0) return P.wide ? cdiv(R, 4) : R;
    if (P.wide && ph >= 1 && ph <= H && (ph == H || (ph - 1) % 5 != 1)) {
        // 64 x 64 output tiles: groups of four column tiles; 128 x 128: groups of eight
        const int N = ph == H ? D.V1 : (ph - 1) % 5 == 0 ? 3 * D.d : (ph - 1) % 5 == 3 ? D.F : D.d;
        if (wide_big(R, N, ph == H ? P.allq_min : P.big_min)) return pad8(cdiv(cdiv(N, 16), 8)) * cdiv(R, 128);
        return pad8(cdiv(cdiv(N, 16), 4)) * RG;
    }
    if (ph < H) {
        switch ((ph - 1) % 5) {
        case 0: return sq_units(P, 3 * D.d) ? pad8(3 * D.d / 32) * cdiv(R, P.mid ? 64 : 32) : pad8(3 * D.d / 16) * RG;
        case 1: return attn_allq(P) ? pad8(cdiv(D.B * D.nH, attn_ppu(P))) : pad8(D.B * D.nH) * cdiv(D.M, 16);
        case 2: return pad8(D.d / 16) * (P.mid ? cdiv(R, 32) : RB);
        case 3: return sq_units(P, D.F) ? pad8(D.F / 32) * cdiv(R, P.mid ? 64 : 32) : pad8(D.F / 16) * RG;
        default: return pad8(D.d / 16) * (P.mid ? cdiv(R, 32) : RB);
        }
    }
    const int RGb = cdiv(D.B, 64);
    switch (ph - H) {
    case TP_HEAD: return pad8(cdiv(D.V1, 16)) * RG;
    case TP_EDGES: return P.prefill_mode ? 0 : cdiv(R, 4);
    case TP_SELECT: return (P.prefill_mode || P.fuse_select) ? 0 : P.nseq;
    case TP_FINAL: return P.nseq;
    case TP_COMMIT: return D.Hh * (D.d / 16) * RGb;
    case TP_DRAFT2: return D.Hh * cdiv(D.V1, 16) * RGb;
    default: return topk_units(P) + cdiv(D.Ly, commit_layers(P)) * cdiv(D.nH, 4) * P.nseq;   // TP_TOPK: draft lists, then KV compaction
    }
}

int step_live_phases(const StepParams& p) {
    const int H = 1 + 5 * p.D.Ly;
    int n = 0;
    for (int ph = p.ph_lo; ph < p.ph_hi; ++ph) n += (ph < H || phase_units(p, ph) > 0) ? 1 : 0;
    return n;
}

// Timing points of one workgroup (StepParams::profile - 1; device clock, 100 MHz): tprof[phase][k]; k = 0 phase start,
// 1 own units done, 2.. points inside a unit.  Read back through vadusa_debug_read.  They exist only in the library
// built with -DVADUSA_CLOCK_BUILD (libvadusa_clock.so): a point that is switched off still costs a read of the
// parameter block, a compare and a branch, nine of them per phase: 20 us per step at valle_b1.
__device__ __forceinline__ void tp(int ph, int k) {
#ifdef VADUSA_CLOCK_BUILD
    const StepParams& P = sP;
    if (P.profile && (int)blockIdx.x == P.profile - 1 && threadIdx.x == 0 && ph < 128) P.s.tprof[ph * 8 + k] = wall_clock64();
#else
    (void)ph; (void)k;
#endif
}

// ---------------------------------------------------------------------------
// grid barrier, two levels, no cache maintenance (see the coherence note above):
// workgroups arrive on one of 8 group counters (number mod 8); the last of a
// group adds one to each of 8 copies of the top counter, and every workgroup
// waits on one copy (its number mod 8) until all groups are in.  Between the
// last arrival and everybody's release lie one atomic with a result, one without
// and one read; a release flag per group, written by the group's last member
// after it has seen the top counter, put a further round trip there (+36 us per
// step of 67 barriers).  Additions to one address are served one after another
// (~5 ns each) and slow down under many watchers, which sets the shape: measured
// 16 x 8 (groups x copies) 518 us per step, 8 x 8 513, 8 x 16 513, 4 x 8 519,
// 32 x 8 527; arriving directly on the 8 copies (256 additions each) 612; one
// level of 16 group counters in 8 copies, watched by 16 lanes, 533.
// All counters grow monotonically (epoch = number of barriers so far).
// Bounded: after ST_SPIN_LIMIT polls, or when another workgroup has raised the
// error flag, the workgroup gives up and the kernel ends (the host reports it).
// Inlined: as a called function (the kernel's only call) it cost the step 10 us: what is live at
// the end of a phase was parked in lanes of a vector register around each of the 66 calls.
// ---------------------------------------------------------------------------
#define BAR_GROUPS 8
#define BAR_TOPS 8
#define BAR_STRIDE 64   // words between counters
__device__ __forceinline__ bool grid_sync(uint32_t epoch, int ph) {
    const StepParams& P = sP;
    __shared__ int s_ok;
    // The workgroup barrier does not wait for global stores (only for LDS traffic): every thread
    // first waits until its own write-through stores have been acknowledged, so that nothing is
    // in flight when thread 0 announces this workgroup's arrival.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();   // every wave's stores have completed (write-through: at the memory side)
    tp(ph, 4);
    if (threadIdx.x == 0) {
        uint32_t* bar = P.s.bar;
        const int g = blockIdx.x % BAR_GROUPS;
        const uint32_t members = (gridDim.x - g + BAR_GROUPS - 1) / BAR_GROUPS;
        const uint32_t ngroups = gridDim.x < BAR_GROUPS ? gridDim.x : BAR_GROUPS;
        int ok = 1, spins = 0;
        const uint32_t old = __hip_atomic_fetch_add(&bar[g * BAR_STRIDE], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == epoch * members) {
#pragma unroll
            for (int x = 0; x < BAR_TOPS; ++x)
                __hip_atomic_fetch_add(&bar[(BAR_GROUPS + x) * BAR_STRIDE], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        const uint32_t* top = &bar[(BAR_GROUPS + blockIdx.x % BAR_TOPS) * BAR_STRIDE];
        while ((int32_t)(__hip_atomic_load(top, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch * ngroups) < 0) {
            if (++spins > ST_SPIN_LIMIT || ((spins & 255) == 0 && ldci(P.s.kerr) != 0)) { ok = 0; break; }
            __builtin_amdgcn_s_sleep(1);
        }
        if (!ok) stwi(P.s.kerr, 1);
        s_ok = ok;
    }
    __syncthreads();
    return s_ok != 0;
}

// ---------------------------------------------------------------------------
// embed (phase 0): one unit per row.  Writes x (fp32), its bf16 copy and the
// per-tile row statistics.
// ---------------------------------------------------------------------------
// WIDE (many-row kernel): a unit is four rows, one per wave, so that a workgroup has four rows' chains of dependent
// loads (row count, tree tables, token, embedding rows) in flight at once instead of one.
template <bool WIDE>
__device__ __forceinline__ void embed_unit(int r_) {
    const StepParams& P = sP;
    const Dims& D = P.D;
    const DevState& s = P.s;
    const int r = WIDE ? __builtin_amdgcn_readfirstlane(r_) * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))
                       : __builtin_amdgcn_readfirstlane(r_);
    if (WIDE && r >= D.B * D.M) return;
    constexpr int NTH = WIDE ? 64 : 256;   // threads per row
    const int b = r / D.M, n = r % D.M, tid = WIDE ? (int)(threadIdx.x & 63) : (int)threadIdx.x;
    int rows;
    if (P.prefill_mode) rows = ldg(s.n_rows + b);
    else rows = s.finished[b] ? 0 : D.M;
    if (!P.prefill_mode && n == 0 && tid == 0) stwi(s.n_rows + b, rows);
    const bool valid = n < rows;
    int tok = 0, pos = 0;
    const bf16_t* E = (const bf16_t*)s.E_speech;
    if (valid) {
        if (P.prefill_mode) {
            const int t = s.chunk_tok[r];
            pos = ldg(s.L + b) + n;
            if (t < 0) { tok = -t - 1; E = (const bf16_t*)s.E_text; }
            else tok = t;
        } else {
            const int dep = s.t_depth[P.table][n];
            pos = ldg(s.L + b) + dep;
            tok = n == 0 ? s.root[b]
                         : s.draft_topk[((size_t)b * D.Hh + (dep - 1)) * VADUSA_MAX_TOPK + s.t_rank[P.table][n]];
            // a row of logits without a largest entry (all NaN) leaves the arg-max and the draft lists without an
            // answer: whatever they hold then, the row read below is one of the table's
            if ((unsigned)tok >= (unsigned)D.V1) tok = 0;
        }
        if (pos >= D.maxpos) pos = D.maxpos - 1;   // the host checks capacity before launching
    }
    if (tid == 0) stwi(s.tok + r, tok);
    const bf16_t* e = E + (size_t)tok * D.d;
    const bf16_t* p = (const bf16_t*)s.P + (size_t)pos * D.d;
    float* x = s.x + (size_t)r * D.d;
    bf16_t* xb = s.xb;                      // slot 0, tiled
    float* st = s.stats;                    // slot 0
    const int R = D.B * D.M;
    for (int c0 = tid * 4; c0 < D.d; c0 += NTH * 4) {
        float v[4];
        const uint2 ev = ldg2(e + c0), pv = ldg2(p + c0);
        v[0] = bf2f((bf16_t)ev.x) + bf2f((bf16_t)pv.x);
        v[1] = bf2f((bf16_t)(ev.x >> 16)) + bf2f((bf16_t)(pv.x >> 16));
        v[2] = bf2f((bf16_t)ev.y) + bf2f((bf16_t)pv.y);
        v[3] = bf2f((bf16_t)(ev.y >> 16)) + bf2f((bf16_t)(pv.y >> 16));
        if (!valid) v[0] = v[1] = v[2] = v[3] = 0.f;
        float sum = v[0] + v[1] + v[2] + v[3];
        sum = quad_sum(sum);
        const float mean = sum * (1.f / 16.f);
        float m2 = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) { const float t = v[j] - mean; m2 += t * t; }
        m2 = quad_sum(m2);
        stwf2(x + c0, v[0], v[1]);
        stwf2(x + c0 + 2, v[2], v[3]);
        stw64(xb + toff(r, c0, D.d >> 5), (uint64_t)pack_bf16(v[0], v[1]) | ((uint64_t)pack_bf16(v[2], v[3]) << 32));
        if ((tid & 3) == 0) stwf2(st + ((size_t)(c0 >> 4) * R + r) * 2, mean, m2);
    }
}

// The context's descriptor table: one record of 32 words for each kind of layer phase (QKV 0,
// out-projection 2, FFN1 3, FFN2 4; slot 1 is unused), holding what does not depend on the launch:
//   words 4i .. 4i+3, i = 0..6: pointer for layer 0 and its advance per layer in bytes, for
//       X, Wp, bias, colsum, stats, out, stats_out (a null pointer has advance 0)
//   words 28..31: K, N, epilogue, -
#if defined(__HIP_DEVICE_COMPILE__)
#define VADUSA_CONSTANT __attribute__((address_space(4)))
#else
#define VADUSA_CONSTANT
#endif

// Descriptor of linear-map unit u of phase ph (all values are workgroup-uniform).  Returns false
// for an empty unit (padding of the XCD-aware numbering) and for phases that are not linear maps.
template <bool WIDE, bool MID = false>   // MID: few-row kernel for 65 to 255 rows (residual maps in 32-row units)
__device__ __forceinline__ bool describe_gemm(int ph, int u, GemmD& g, int& nt, int& row0, const uint32_t* gtab = nullptr) {
    const StepParams& P = sP;
    const Dims& D = P.D;
    const DevState& s = P.s;
    const int R = D.B * D.M, H = 1 + 5 * D.Ly;
    if (ph == 0) return false;
    if (!WIDE && gtab != nullptr && ph < H) {
        // The table never changes while kernels run and its address is workgroup-uniform: read
        // through the constant address space, i.e. by scalar loads into scalar registers; the
        // same four records serve every layer, so they stay in the scalar cache.
        const int l = (ph - 1) / 5, k = (ph - 1) % 5;
        const VADUSA_CONSTANT vadusa_u32x4* t = (const VADUSA_CONSTANT vadusa_u32x4*)(gtab + k * VADUSA_GREC_WORDS);
        vadusa_u32x4 w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = t[i];
        auto at = [&](int i) {
            const uint64_t base = (uint64_t)w[i].x | ((uint64_t)w[i].y << 32), adv = (uint64_t)w[i].z | ((uint64_t)w[i].w << 32);
            return base + (uint64_t)l * adv;
        };
        g.R = R; g.outf = nullptr; g.ph = ph; g.G = 4; g.layer = l;
        g.X = (const bf16_t*)at(0); g.Wp = (const uint4*)at(1); g.bias = (const float*)at(2); g.colsum = (const float*)at(3);
        g.stats = (const float*)at(4); g.out = (bf16_t*)at(5); g.stats_out = (float*)at(6);
        g.K = (int)w[7].x; g.N = (int)w[7].y; g.epi = (int)w[7].z;
        const int NT = g.N >> 4, NTp = pad8(NT);
        int rb;
        if (u < NTp) { nt = u; rb = 0; }
        else if ((NTp & (NTp - 1)) == 0) { nt = u & (NTp - 1); rb = u >> __builtin_ctz(NTp); }
        else { nt = u % NTp; rb = u / NTp; }
        row0 = rb * (g.epi == SE_RESID ? (MID ? 32 : 16) : 64);
        return nt < NT;
    }
    g.R = R; g.stats = nullptr; g.colsum = nullptr; g.bias = nullptr; g.out = nullptr; g.outf = nullptr;
    g.stats_out = nullptr; g.layer = 0; g.ph = ph;
    // (column tile, row block) of unit u of a map with NT column tiles; false: empty unit
    int rb = 0;
    nt = 0; row0 = 0;
    const bool wide = WIDE && ph <= H;   // the draft maps have only B rows: always narrow
    g.G = 4;
    int wrows = 64;   // rows per unit of the many-row kernel
    auto split = [&](int NT) {
        if (wide) {   // unit = (row block) * pad8(tile groups) + group of G column tiles
            if (wide_big(R, g.N, ph == H ? P.allq_min : P.big_min)) { g.G = 8; wrows = 128; }
            const int NG = cdiv(NT, g.G), NGp = pad8(NG), gidx = u % NGp;
            rb = u / NGp;
            nt = gidx * g.G;
            return gidx < NG;
        }
        const int NTp = pad8(NT);
        if (u < NTp) { nt = u; rb = 0; }                                            // a single row block
        else if ((NTp & (NTp - 1)) == 0) { nt = u & (NTp - 1); rb = u >> __builtin_ctz(NTp); }   // power of two
        else { nt = u % NTp; rb = u / NTp; }
        return nt < NT;
    };
    if (ph < H) {
        const int l = (ph - 1) / 5, k = (ph - 1) % 5;
        LayerW w;   // layer l = layer 0 advanced by l * lw_stride bytes
        {
            const size_t off = (size_t)l * P.lw_stride;
            w.Wqkv = (const char*)P.lw0.Wqkv + off; w.Wo = (const char*)P.lw0.Wo + off;
            w.W1 = (const char*)P.lw0.W1 + off; w.W2 = (const char*)P.lw0.W2 + off;
            w.bo = (const float*)((const char*)P.lw0.bo + off); w.b2 = (const float*)((const char*)P.lw0.b2 + off);
            w.t_qkv = (float*)((char*)P.lw0.t_qkv + off); w.cs_qkv = (float*)((char*)P.lw0.cs_qkv + off);
            w.t_w1 = (float*)((char*)P.lw0.t_w1 + off); w.cs_w1 = (float*)((char*)P.lw0.cs_w1 + off);
        }
        g.layer = l;
        // slots: xb / stats 2l = input of the layer, 2l+1 = after the out-projection, 2l+2 = after FFN2
        bf16_t* xb0 = s.xb + (size_t)(2 * l) * s.act_stride;
        float* st0 = s.stats + (size_t)(2 * l) * s.stats_stride;
        bf16_t* q_l = (bf16_t*)s.q + (size_t)l * s.act_stride;
        bf16_t* att_l = (bf16_t*)s.att + (size_t)l * s.act_stride;
        bf16_t* hid_l = (bf16_t*)s.hid + (size_t)l * s.hid_stride;
        switch (k) {
        case 0:
            g.X = xb0; g.K = D.d; g.N = 3 * D.d; g.Wp = (const uint4*)w.Wqkv; g.bias = w.t_qkv; g.colsum = w.cs_qkv;
            g.stats = st0; g.epi = SE_QKV; g.out = q_l;
            return split(3 * D.d / 16) ? (row0 = rb * wrows, true) : false;
        case 1: return false;
        case 2:
            g.X = att_l; g.K = D.d; g.N = D.d; g.Wp = (const uint4*)w.Wo; g.bias = w.bo;
            g.epi = SE_RESID; g.out = xb0 + s.act_stride; g.stats_out = st0 + s.stats_stride;
            return split(D.d / 16) ? (row0 = rb * (wide ? wrows : MID ? 32 : 16), true) : false;
        case 3:
            g.X = xb0 + s.act_stride; g.K = D.d; g.N = D.F; g.Wp = (const uint4*)w.W1; g.bias = w.t_w1; g.colsum = w.cs_w1;
            g.stats = st0 + s.stats_stride; g.epi = SE_GELU; g.out = hid_l;
            return split(D.F / 16) ? (row0 = rb * wrows, true) : false;
        default:
            g.X = hid_l; g.K = D.F; g.N = D.d; g.Wp = (const uint4*)w.W2; g.bias = w.b2;
            g.epi = SE_RESID; g.out = xb0 + 2 * s.act_stride; g.stats_out = st0 + 2 * s.stats_stride;
            return split(D.d / 16) ? (row0 = rb * (wide ? wrows : MID ? 32 : 16), true) : false;
        }
    }
    const int RGb = cdiv(D.B, 64);
    switch (ph - H) {
    case TP_HEAD:
        g.X = s.xb + (size_t)(2 * D.Ly) * s.act_stride; g.K = D.d; g.N = D.V1; g.Wp = (const uint4*)s.W_out;
        g.bias = s.t_out; g.colsum = s.cs_out;
        g.stats = s.stats + (size_t)(2 * D.Ly) * s.stats_stride; g.epi = SE_LOGITS; g.outf = s.logits;
        return split(cdiv(D.V1, 16)) ? (row0 = rb * wrows, true) : false;
    case TP_COMMIT: {
        const int per = (D.d / 16) * RGb, i = u / per, v = u % per;
        DraftW dw;
        dw.W1 = (const char*)P.dw0.W1 + (size_t)i * P.dw_stride;
        dw.b1 = (const float*)((const char*)P.dw0.b1 + (size_t)i * P.dw_stride);
        g.R = D.B; g.X = (const bf16_t*)s.hbest; g.K = D.d; g.N = D.d;
        g.Wp = (const uint4*)dw.W1; g.bias = dw.b1; g.epi = SE_SILU_RESID;
        g.out = (bf16_t*)s.rdraft + (size_t)i * s.draft_stride;
        nt = v / RGb; row0 = (v % RGb) * 64;
        return true;
    }
    case TP_DRAFT2: {
        const int per = cdiv(D.V1, 16) * RGb, i = u / per, v = u % per;
        DraftW dw;
        dw.W2 = (const char*)P.dw0.W2 + (size_t)i * P.dw_stride;
        g.R = D.B; g.X = (const bf16_t*)s.rdraft + (size_t)i * s.draft_stride; g.K = D.d; g.N = D.V1;
        g.Wp = (const uint4*)dw.W2; g.epi = SE_F32;
        g.outf = s.zdraft + (size_t)i * D.Bmax * D.V1;
        nt = v / RGb; row0 = (v % RGb) * 64;
        return true;
    }
    default: return false;
    }
}


// ---------------------------------------------------------------------------
// linear-map unit.  NRT = 4: 64 rows x one 16-column tile (QKV, FFN1, heads).
// NRT = 1: 16 rows x one tile (out-projection, FFN2: residual update +
// statistics of the new rows).  Wave w owns a contiguous quarter of the
// k-steps and loads BOTH operands straight from global memory into the MFMA
// register layout: B (weights, one contiguous KiB per wave load, from HBM) and
// A (activations, 16 bytes per lane, from L2).  Every load of a chunk is issued
// before the first MFMA, so a unit pays one memory latency per chunk.  Partial
// sums are combined in wave order through LDS.
// ---------------------------------------------------------------------------
// Where lane l's four accumulator floats of a 16 x 16 tile sit in a reduction buffer (in units of 16 bytes).  A
// thread of the 64-row epilogues reads, for one of its four columns, word (row & 3) of lane (row >> 2) * 16 + column:
// with the lanes in order the 64 reads of a wave fall into 8 of the 32 banks; with bits 3-5 of the lane folded
// onto bits 0-2 they cover all of them, and a wave's 16-byte writes stay a permutation inside each group of eight.
__device__ __forceinline__ int red_slot(int l) {
    return l ^ ((l >> 3) & 7);
}
template <int NRT>
__device__ __forceinline__ void gemm_unit(int ph_, int u_, const uint32_t* gtab) {
    // arguments arrive in vector registers: make them (and all that follows from them) scalar
    const int ph_u = __builtin_amdgcn_readfirstlane(ph_), u_u = __builtin_amdgcn_readfirstlane(u_);
    const StepParams& P = sP;
    GemmD g;
    int nt, row0;
    if (!describe_gemm<false, NRT == 2>(ph_u, u_u, g, nt, row0, gtab)) return;
    extern __shared__ uint4 smem[];
    float* s_stat = (float*)((char*)smem + ST_TILE_BYTES);
    constexpr int CH = NRT == 4 ? 8 : NRT == 2 ? 8 : 16;     // k-steps per chunk
    constexpr int ROWS = NRT * 16;
    const Dims& D = P.D;
    const DevState& s = P.s;
    // the wave index is the same for all lanes of a wave: say so, and everything derived from it
    // (k-step range, loop bounds) stays in scalar registers and branches are scalar
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int nks = g.K >> 5;
    const int ks_lo = (nks * wave) >> 2, ks_hi = (nks * (wave + 1)) >> 2;
    // Operand addresses are kept as a workgroup-uniform base (scalar registers) plus a 32-bit
    // per-lane index, so that a load needs no vector address arithmetic.
    const uint4* Wp = uniform_ptr(g.Wp + (size_t)nt * nks * 64);
    // A operand: tile (row tile, k-step) of the tiled activation layout = 64 lanes x 16 bytes
    const uint4* Ap[NRT];
    bool rowok[NRT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
        rowok[rt] = row0 + rt * 16 < g.R;   // whole tile beyond the last row: skipped
        Ap[rt] = uniform_ptr((const uint4*)g.X + (size_t)(rowok[rt] ? (row0 >> 4) + rt : 0) * nks * 64);
    }
    const uint32_t ulane = (uint32_t)lane;
    f32x4_t acc[NRT];
#pragma unroll
    for (int i = 0; i < NRT; ++i) acc[i] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    tp(g.ph, 5);
    // epilogue inputs, requested now so that they arrive with the operands (the vectors are
    // padded to whole 16-column tiles)
    uint4 cs4 = make_uint4(0, 0, 0, 0), b4 = cs4;
    float xres[NRT == 4 ? 1 : NRT], bres = 0.f;
    int kv_b = 0, kv_L = 0, kv_rows = 0, kv_which = 0, kv_cc = 0;   // QKV map: where this thread's key / value row goes
    if (NRT == 4) {
        const int n0 = nt * 16 + (tid & 3) * 4;
        if (g.colsum) cs4 = ldg4(g.colsum + n0);
        if (g.bias) b4 = ldg4(g.bias + n0);
        if (g.epi == SE_QKV && nt * 16 >= D.d) {
            const int r = row0 + (tid >> 2) < g.R ? row0 + (tid >> 2) : g.R - 1;   // no branch on the row: see gemm_unit22
            kv_which = (nt * 16) / D.d - 1;            // workgroup-uniform: 0 keys, 1 values
            kv_cc = (nt * 16) % D.d;
            kv_b = r / D.M;
            kv_L = s_seqL[kv_b];                       // (a few-row kernel has fewer than 256 rows, so all its sequences are cached)
            kv_rows = s_seqRows[kv_b];
        }
    } else {
        const int n = nt * 16 + (tid & 15);
#pragma unroll
        for (int it = 0; it < (NRT == 4 ? 1 : NRT); ++it) {
            const int r = row0 + it * 16 + (tid >> 4);
            xres[it] = r < g.R ? ldg(s.x + (size_t)r * g.N + n) : 0.f;
        }
        bres = ldg(g.bias + n);
    }

    // row statistics of the LayerNorm folded into this map: four threads per row, each
    // merges a quarter of the 16-column tiles (loads issued with the first operand chunk)
    // The tile means are summed as distances from c0 = the row's first tile mean (a shift close to the row mean):
    // the spread between the tiles then comes out of small numbers, also for rows whose mean is far larger than
    // their spread (sum m_t^2 - tiles mean^2 would lose it to cancellation).
    float s1 = 0.f, s2 = 0.f, s3 = 0.f, c0 = 0.f;
    const int tiles = g.K >> 4;
    const bool do_stats = g.stats != nullptr && tid < ROWS * 4;

    auto merge_stats = [&]() {
        const int row = tid >> 2, part = tid & 3, r = row0 + row;
        if (r < g.R) {
            const float2* sp = (const float2*)g.stats + r;
            c0 = ldgf2(sp).x;
            for (int t0 = part; t0 < tiles; t0 += 32) {
                float2 v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int t = t0 + 4 * j;
                    v[j] = t < tiles ? ldgf2(sp + (size_t)t * g.R) : make_float2(0.f, 0.f);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (t0 + 4 * j < tiles) { const float dv = v[j].x - c0; s1 += dv; s2 += v[j].y; s3 += dv * dv; }
            }
        }
    };
    // Up to 64 tiles (K <= 1024) a thread's share of the statistics is at most 16 entries: they are
    // requested here, ahead of the operands, so that they are back before the operands are (asked
    // for after them they would return last and the reduction's result would wait for them), and
    // summed after the MFMAs.  Addresses are clamped instead of guarded: no branch per load.
    const bool stats_early = do_stats && tiles <= 64;
    float2 sv[16];
    if (stats_early) {
        // addresses as the statistics' base (the same for the workgroup: scalar registers) plus a 32-bit byte offset per
        // thread and tile: no 64-bit multiplication per load (with one wave per SIMD, seventeen of them cost 0.6 us)
        const int r = row0 + (tid >> 2);
        const char* sb = (const char*)uniform_ptr(g.stats);
        const uint32_t roff = (uint32_t)(r < g.R ? r : 0) * 8u, tstride = (uint32_t)g.R * 8u;
        c0 = ldgf2(sb + roff).x;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int t = (tid & 3) + 4 * j;
            sv[j] = ldgf2(sb + (roff + (uint32_t)(t < tiles ? t : 0) * tstride));
        }
    }
    // the first pass always runs: a wave without k-steps (K < 128) loads nothing in it but still
    // merges the statistics of its rows
    for (int kb = ks_lo; kb == ks_lo || kb < ks_hi; kb += CH) {
        uint4 bw[CH], aw[NRT][CH];
        if (kb + CH <= ks_hi) {   // a whole chunk (the usual case): straight-line loads
#pragma unroll
            for (int i = 0; i < CH; ++i) bw[i] = ldg4((const char*)Wp + ((uint32_t)(kb + i) * 1024u + ulane * 16u));
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    aw[rt][i] = rowok[rt] ? ldg4((const char*)Ap[rt] + ((uint32_t)(kb + i) * 1024u + ulane * 16u)) : make_uint4(0, 0, 0, 0);
        } else {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int ks = kb + i;
                bw[i] = ks < ks_hi ? ldg4((const char*)Wp + ((uint32_t)ks * 1024u + ulane * 16u)) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    const int ks = kb + i;
                    aw[rt][i] = (ks < ks_hi && rowok[rt]) ? ldg4((const char*)Ap[rt] + ((uint32_t)ks * 1024u + ulane * 16u)) : make_uint4(0, 0, 0, 0);
                }
        }
        if (kb == ks_lo) tp(g.ph, 6);
        if (kb == ks_lo && do_stats && !stats_early) merge_stats();
        if (kb == ks_lo) tp(g.ph, 7);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, bw[i]);
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt)
                acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, aw[rt][i]), bfrag,
                                                                  acc[rt], 0, 0, 0);
        }
    }
    tp(g.ph, 2);   // operands arrived, MFMAs issued
    if (stats_early && row0 + (tid >> 2) < g.R) {
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if ((tid & 3) + 4 * j < tiles) { const float dv = sv[j].x - c0; s1 += dv; s2 += sv[j].y; s3 += dv * dv; }
    }
    if (g.stats) {
        s1 = quad_sum(s1);
        s2 = quad_sum(s2);
        s3 = quad_sum(s3);
        if (do_stats && (tid & 3) == 0) {
            // mean of tile means; M2 = sum M2_t + 16 sum (mean_t - mean)^2
            const float mean = c0 + s1 / tiles;   // s1, s3: sums of the tile means' distances from c0 and of their squares
            const float m2 = s2 + 16.f * fmaxf(s3 - s1 * s1 / tiles, 0.f);
            s_stat[tid >> 2] = mean;
            s_stat[64 + (tid >> 2)] = rsqrtf(m2 / g.K + LN_EPS);
        }
    }
    __syncthreads();
    float* red = (float*)smem;   // [wave][rt][lane][4]
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
        for (int i = 0; i < 4; ++i) red[((wave * NRT + rt) * 64 + (NRT == 4 ? red_slot(lane) : lane)) * 4 + i] = acc[rt][i];
    __syncthreads();
    tp(g.ph, 3);   // partial sums exchanged

    if (NRT == 4) {
        const int row = tid >> 2, rt = row >> 4, rr = row & 15, r = row0 + row;
        const int n0 = nt * 16 + (tid & 3) * 4;       // four consecutive output columns
        if (r < g.R && n0 < g.N) {
            const float mu = g.stats ? s_stat[row] : 0.f, rstd = g.stats ? s_stat[64 + row] : 1.f;
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = (tid & 3) * 4 + j;
                const int src = ((rt * 64) + red_slot((rr >> 2) * 16 + col)) * 4 + (rr & 3);
                float a = red[src];
#pragma unroll
                for (int w = 1; w < 4; ++w) a += red[w * 1024 + src];
                const float csj = __uint_as_float(j == 0 ? cs4.x : j == 1 ? cs4.y : j == 2 ? cs4.z : cs4.w);
                const float bj = __uint_as_float(j == 0 ? b4.x : j == 1 ? b4.y : j == 2 ? b4.z : b4.w);
                if (g.stats) a = rstd * (a - mu * csj);
                v[j] = a + bj;   // columns beyond N (ragged last tile of a vocabulary map) are never stored
            }
            const bool full = n0 + 3 < g.N;   // only the vocabulary maps have a ragged last tile
            switch (g.epi) {
            case SE_GELU:
                stw64(g.out + toff(r, n0, g.N >> 5),
                      (uint64_t)pack_bf16(gelu_s(v[0]), gelu_s(v[1])) | ((uint64_t)pack_bf16(gelu_s(v[2]), gelu_s(v[3])) << 32));
                break;
            case SE_LOGITS:
            case SE_F32:
                // rows of V+1 floats are only 4-byte aligned: single-word write-through stores
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (full || n0 + j < g.N) stwf(g.outf + (size_t)r * g.N + n0 + j, v[j]);
                break;
            case SE_SILU_RESID: {
                const uint2 xin = ldg2(g.X + toff(r, n0, g.K >> 5));
                const float h0 = bf2f((bf16_t)xin.x) + silu_s(v[0]), h1 = bf2f((bf16_t)(xin.x >> 16)) + silu_s(v[1]);
                const float h2 = bf2f((bf16_t)xin.y) + silu_s(v[2]), h3 = bf2f((bf16_t)(xin.y >> 16)) + silu_s(v[3]);
                stw64(g.out + toff(r, n0, g.N >> 5), (uint64_t)pack_bf16(h0, h1) | ((uint64_t)pack_bf16(h2, h3) << 32));
                break;
            }
            case SE_QKV: {
                const uint64_t pk = (uint64_t)pack_bf16(v[0], v[1]) | ((uint64_t)pack_bf16(v[2], v[3]) << 32);
                if (n0 < D.d) { stw64(g.out + toff(r, n0, D.d >> 5), pk); break; }
                const int b = kv_b, node = r - b * D.M;
                const int which = kv_which, cc = kv_cc + (tid & 3) * 4, head = cc >> 6, dim = cc & 63;
                const int pos = kv_L + node;
                if (pos < D.maxpos && kv_rows > 0) {
                    const size_t hb = ((((size_t)g.layer * D.Bmax + b) * D.nH + head) * kv_cap(D.maxpos)) * 64;
                    if (which) {
                        bf16_t* vp = (bf16_t*)s.Vc + hb + vc_off(pos, dim);   // four dimensions of one position: four lanes of a value tile
#pragma unroll
                        for (int j = 0; j < 4; ++j) stw16(vp + j * 8, f2bf(v[j]));
                    } else {
                        stw64((bf16_t*)s.Kc + hb + kc_off(pos, dim), pk);   // four dimensions of one key: half of a lane's piece
                    }
                }
                break;
            }
            default: break;
            }
        }
    } else {
        // residual update: one element per thread and row tile, statistics over the 16 columns of the tile
#pragma unroll
        for (int it = 0; it < (NRT == 4 ? 1 : NRT); ++it) {
            const int row = tid >> 4, col = tid & 15, r = row0 + it * 16 + row, n = nt * 16 + col;
            const int src = it * 256 + ((row >> 2) * 16 + col) * 4 + (row & 3);
            float v = red[src];
#pragma unroll
            for (int w = 1; w < 4; ++w) v += red[w * (NRT * 256) + src];
            const bool ok = r < g.R;
            float xn = 0.f;
            if (ok) {
                xn = xres[it] + v + bres;
                stwf(s.x + (size_t)r * g.N + n, xn);
            }
            {
                const float nb = __int_as_float(dpp_perm<0xB1>(__float_as_int(xn)));   // the neighbouring column (used by even columns): a pair -> one 32-bit store
                if (ok && !(col & 1)) stw32(g.out + toff(r, n, g.N >> 5), pack_bf16(xn, nb));
            }
            float sum = xn;
            sum = row16_sum(sum);
            const float mean = sum * (1.f / 16.f);
            float m2 = (xn - mean) * (xn - mean);
            m2 = row16_sum(m2);
            if (ok && col == 0) stwf2(g.stats_out + ((size_t)nt * g.R + r) * 2, mean, m2);
        }
    }
}

// ---------------------------------------------------------------------------
// 32 x 32 unit of the few-row kernel (two row tiles x two column tiles; QKV and FFN1 when
// sq_units): the same scheme as gemm_unit (wave w owns a quarter of the k-steps, operands
// straight into MFMA registers, partial sums added in wave order through LDS), with every A
// fragment used for two column tiles and every B fragment for two row tiles.  Units are
// numbered (row block) * pad8(column pairs) + column pair.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void gemm_unit22(int ph_, int u_, const uint32_t* gtab) {
    const int ph_u = __builtin_amdgcn_readfirstlane(ph_), u_u = __builtin_amdgcn_readfirstlane(u_);
    const StepParams& P = sP;
    GemmD g;
    int nt, row0;
    if (!describe_gemm<false>(ph_u, 0, g, nt, row0, gtab)) return;   // unit 0 always exists: the map itself
    {
        const int NG = g.N >> 5, NGp = pad8(NG);
        int gi, rb;
        if (u_u < NGp) { gi = u_u; rb = 0; }
        else if ((NGp & (NGp - 1)) == 0) { gi = u_u & (NGp - 1); rb = u_u >> __builtin_ctz(NGp); }
        else { gi = u_u % NGp; rb = u_u / NGp; }
        if (gi >= NG) return;
        nt = gi * 2; row0 = rb * 32;
    }
    extern __shared__ uint4 smem[];
    float* s_stat = (float*)((char*)smem + ST_TILE_BYTES);
    constexpr int CH = 8;
    const Dims& D = P.D;
    const DevState& s = P.s;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int nks = g.K >> 5;
    const int ks_lo = (nks * wave) >> 2, ks_hi = (nks * (wave + 1)) >> 2;
    const uint4* Wp[2];
    const uint4* Ap[2];
    bool rowok[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        Wp[t] = uniform_ptr(g.Wp + (size_t)(nt + t) * nks * 64);
        rowok[t] = row0 + t * 16 < g.R;
        Ap[t] = uniform_ptr((const uint4*)g.X + (size_t)(rowok[t] ? (row0 >> 4) + t : 0) * nks * 64);
    }
    const uint32_t ulane = (uint32_t)lane;
    f32x4_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    tp(g.ph, 5);
    // epilogue inputs of this thread's four columns, requested with the operands
    const int erow = tid >> 3, ecg = tid & 7;                 // row of the unit, group of four columns (of 32)
    const int n0 = nt * 16 + ecg * 4;
    uint4 cs4 = make_uint4(0, 0, 0, 0), b4 = cs4;
    if (g.colsum) cs4 = ldg4(g.colsum + n0);
    if (g.bias) b4 = ldg4(g.bias + n0);
    int kv_b = 0, kv_L = 0, kv_rows = 0, kv_which = 0, kv_cc = 0;
    if (g.epi == SE_QKV && nt * 16 >= D.d) {
        // (no branch on the row: behind a divergent branch the compiler waits for every load that is under way, here
        // the column sums and bias just requested, before the statistics and operands are asked for; the sequence's
        // length and row count come from the copy in LDS, not from memory)
        const int r = row0 + erow < g.R ? row0 + erow : g.R - 1;
        kv_which = (nt * 16) / D.d - 1;
        kv_cc = (nt * 16) % D.d;
        kv_b = r / D.M;
        kv_L = s_seqL[kv_b];          // (this unit runs with up to 64 rows, so at most 64 sequences: all of them cached)
        kv_rows = s_seqRows[kv_b];
    }
    // LayerNorm statistics of the unit's 32 rows: four threads per row (threads 0..127)
    float s1 = 0.f, s2 = 0.f, s3 = 0.f, c0 = 0.f;   // c0: shift of the tile means, see gemm_unit
    const int tiles = g.K >> 4;
    const bool do_stats = g.stats != nullptr && tid < 128;
    const bool stats_early = do_stats && tiles <= 64;
    float2 sv[16];
    if (stats_early) {
        // addresses as the statistics' base (the same for the workgroup: scalar registers) plus a 32-bit byte offset per
        // thread and tile: no 64-bit multiplication per load (with one wave per SIMD, seventeen of them cost 0.6 us)
        const int r = row0 + (tid >> 2);
        const char* sb = (const char*)uniform_ptr(g.stats);
        const uint32_t roff = (uint32_t)(r < g.R ? r : 0) * 8u, tstride = (uint32_t)g.R * 8u;
        c0 = ldgf2(sb + roff).x;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int t = (tid & 3) + 4 * j;
            sv[j] = ldgf2(sb + (roff + (uint32_t)(t < tiles ? t : 0) * tstride));
        }
    }
    for (int kb = ks_lo; kb == ks_lo || kb < ks_hi; kb += CH) {
        uint4 bw[2][CH], aw[2][CH];
        if (kb + CH <= ks_hi) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < CH; ++i) bw[t][i] = ldg4((const char*)Wp[t] + ((uint32_t)(kb + i) * 1024u + ulane * 16u));
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    aw[t][i] = rowok[t] ? ldg4((const char*)Ap[t] + ((uint32_t)(kb + i) * 1024u + ulane * 16u)) : make_uint4(0, 0, 0, 0);
        } else {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    const int ks = kb + i;
                    bw[t][i] = ks < ks_hi ? ldg4((const char*)Wp[t] + ((uint32_t)ks * 1024u + ulane * 16u)) : make_uint4(0, 0, 0, 0);
                    aw[t][i] = (ks < ks_hi && rowok[t]) ? ldg4((const char*)Ap[t] + ((uint32_t)ks * 1024u + ulane * 16u)) : make_uint4(0, 0, 0, 0);
                }
        }
        if (kb == ks_lo) tp(g.ph, 6);
        if (kb == ks_lo && do_stats && !stats_early) {
            const int r = row0 + (tid >> 2);
            if (r < g.R) {
                const float2* sp = (const float2*)g.stats + r;
                c0 = ldgf2(sp).x;
                for (int t = tid & 3; t < tiles; t += 4) {
                    const float2 v = ldgf2(sp + (size_t)t * g.R);
                    const float dv = v.x - c0; s1 += dv; s2 += v.y; s3 += dv * dv;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i)
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int ct = 0; ct < 2; ++ct)
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, aw[rt][i]),
                                                                          __builtin_bit_cast(bf16x8_t, bw[ct][i]), acc[rt][ct], 0, 0, 0);
    }
    tp(g.ph, 2);
    if (stats_early && row0 + (tid >> 2) < g.R) {
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if ((tid & 3) + 4 * j < tiles) { const float dv = sv[j].x - c0; s1 += dv; s2 += sv[j].y; s3 += dv * dv; }
    }
    if (g.stats) {
        s1 = quad_sum(s1);
        s2 = quad_sum(s2);
        s3 = quad_sum(s3);
        if (do_stats && (tid & 3) == 0) {
            const float mean = c0 + s1 / tiles;   // s1, s3: sums of the tile means' distances from c0 and of their squares
            const float m2 = s2 + 16.f * fmaxf(s3 - s1 * s1 / tiles, 0.f);
            s_stat[tid >> 2] = mean;
            s_stat[64 + (tid >> 2)] = rsqrtf(m2 / g.K + LN_EPS);
        }
    }
    __syncthreads();
    float* red = (float*)smem;   // [wave][row tile][column tile][lane][4]
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[((wave * 4 + rt * 2 + ct) * 64 + red_slot(lane)) * 4 + i] = acc[rt][ct][i];
    __syncthreads();
    tp(g.ph, 3);
    {
        const int rt = erow >> 4, rr = erow & 15, ct = ecg >> 2, r = row0 + erow;
        if (r < g.R) {
            const float mu = g.stats ? s_stat[erow] : 0.f, rstd = g.stats ? s_stat[64 + erow] : 1.f;
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = (ecg & 3) * 4 + j;
                const int src = (((rt * 2 + ct) * 64) + red_slot((rr >> 2) * 16 + col)) * 4 + (rr & 3);
                float a = red[src];
#pragma unroll
                for (int w = 1; w < 4; ++w) a += red[w * 1024 + src];
                const float csj = __uint_as_float(j == 0 ? cs4.x : j == 1 ? cs4.y : j == 2 ? cs4.z : cs4.w);
                const float bj = __uint_as_float(j == 0 ? b4.x : j == 1 ? b4.y : j == 2 ? b4.z : b4.w);
                if (g.stats) a = rstd * (a - mu * csj);
                v[j] = a + bj;
            }
            if (g.epi == SE_GELU) {
                stw64(g.out + toff(r, n0, g.N >> 5),
                      (uint64_t)pack_bf16(gelu_s(v[0]), gelu_s(v[1])) | ((uint64_t)pack_bf16(gelu_s(v[2]), gelu_s(v[3])) << 32));
            } else if (g.epi == SE_QKV) {
                const uint64_t pk = (uint64_t)pack_bf16(v[0], v[1]) | ((uint64_t)pack_bf16(v[2], v[3]) << 32);
                if (n0 < D.d) {
                    stw64(g.out + toff(r, n0, D.d >> 5), pk);
                } else {
                    const int b = kv_b, node = r - b * D.M;
                    const int cc = kv_cc + ecg * 4, head = cc >> 6, dim = cc & 63;
                    const int pos = kv_L + node;
                    if (pos < D.maxpos && kv_rows > 0) {
                        const size_t hb = ((((size_t)g.layer * D.Bmax + b) * D.nH + head) * kv_cap(D.maxpos)) * 64;
                        if (kv_which) {
                            bf16_t* vp = (bf16_t*)s.Vc + hb + vc_off(pos, dim);   // four dimensions of one position: four lanes of a value tile
#pragma unroll
                            for (int j = 0; j < 4; ++j) stw16(vp + j * 8, f2bf(v[j]));
                        } else {
                            stw64((bf16_t*)s.Kc + hb + kc_off(pos, dim), pk);   // four dimensions of one key: half of a lane's piece
                        }
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// 64 x 32 unit (four row tiles x two column tiles) of the few-row kernels for 65 to 255 rows (trees of
// more than 64 nodes, small batches): gemm_unit22 with twice the rows, so that QKV and FFN1 of a 128-row step
// are one round of units (192 and 256) instead of two, and a weight fragment feeds four row tiles.  Units are
// numbered (row block of 64) * pad8(column pairs) + column pair.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void gemm_unit42(int ph_, int u_, const uint32_t* gtab) {
    const int ph_u = __builtin_amdgcn_readfirstlane(ph_), u_u = __builtin_amdgcn_readfirstlane(u_);
    const StepParams& P = sP;
    GemmD g;
    int nt, row0;
    if (!describe_gemm<false>(ph_u, 0, g, nt, row0, gtab)) return;   // unit 0 always exists: the map itself
    {
        const int NG = g.N >> 5, NGp = pad8(NG);
        int gi, rb;
        if (u_u < NGp) { gi = u_u; rb = 0; }
        else if ((NGp & (NGp - 1)) == 0) { gi = u_u & (NGp - 1); rb = u_u >> __builtin_ctz(NGp); }
        else { gi = u_u % NGp; rb = u_u / NGp; }
        if (gi >= NG) return;
        nt = gi * 2; row0 = rb * 64;
    }
    extern __shared__ uint4 smem[];
    float* s_stat = (float*)((char*)smem + ST_MID_TILE_BYTES);
    constexpr int CH = 8;
    const Dims& D = P.D;
    const DevState& s = P.s;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int nks = g.K >> 5;
    const int ks_lo = (nks * wave) >> 2, ks_hi = (nks * (wave + 1)) >> 2;
    const uint4* Wp[2];
    const uint4* Ap[4];
    bool rowok[4];
#pragma unroll
    for (int t = 0; t < 2; ++t) Wp[t] = uniform_ptr(g.Wp + (size_t)(nt + t) * nks * 64);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        rowok[t] = row0 + t * 16 < g.R;
        Ap[t] = uniform_ptr((const uint4*)g.X + (size_t)(rowok[t] ? (row0 >> 4) + t : 0) * nks * 64);
    }
    const uint32_t ulane = (uint32_t)lane;
    f32x4_t acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    tp(g.ph, 5);
    // epilogue inputs of this thread's four columns, requested with the operands
    const int erow = tid >> 3, ecg = tid & 7;                 // rows erow and erow + 32 of the unit, group of four columns (of 32)
    const int n0 = nt * 16 + ecg * 4;
    uint4 cs4 = make_uint4(0, 0, 0, 0), b4 = cs4;
    if (g.colsum) cs4 = ldg4(g.colsum + n0);
    if (g.bias) b4 = ldg4(g.bias + n0);
    int kv_b[2] = {0, 0}, kv_L[2] = {0, 0}, kv_rows[2] = {0, 0}, kv_which = 0, kv_cc = 0;
    if (g.epi == SE_QKV && nt * 16 >= D.d) {
        kv_which = (nt * 16) / D.d - 1;
        kv_cc = (nt * 16) % D.d;
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const int r = row0 + 32 * hh + erow < g.R ? row0 + 32 * hh + erow : g.R - 1;   // no branch on the row: see gemm_unit22
            kv_b[hh] = r / D.M;
            kv_L[hh] = s_seqL[kv_b[hh]];
            kv_rows[hh] = s_seqRows[kv_b[hh]];
        }
    }
    // LayerNorm statistics of the unit's 64 rows: four threads per row
    float s1 = 0.f, s2 = 0.f, s3 = 0.f, c0 = 0.f;   // c0: shift of the tile means, see gemm_unit
    const int tiles = g.K >> 4;
    const bool do_stats = g.stats != nullptr;
    const bool stats_early = do_stats && tiles <= 64;
    float2 sv[16];
    if (stats_early) {
        // addresses as the statistics' base (the same for the workgroup: scalar registers) plus a 32-bit byte offset per
        // thread and tile: no 64-bit multiplication per load (with one wave per SIMD, seventeen of them cost 0.6 us)
        const int r = row0 + (tid >> 2);
        const char* sb = (const char*)uniform_ptr(g.stats);
        const uint32_t roff = (uint32_t)(r < g.R ? r : 0) * 8u, tstride = (uint32_t)g.R * 8u;
        c0 = ldgf2(sb + roff).x;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int t = (tid & 3) + 4 * j;
            sv[j] = ldgf2(sb + (roff + (uint32_t)(t < tiles ? t : 0) * tstride));
        }
    }
    for (int kb = ks_lo; kb == ks_lo || kb < ks_hi; kb += CH) {
        uint4 bw[2][CH], aw[4][CH];
        if (kb + CH <= ks_hi) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < CH; ++i) bw[t][i] = ldg4((const char*)Wp[t] + ((uint32_t)(kb + i) * 1024u + ulane * 16u));
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    aw[t][i] = rowok[t] ? ldg4((const char*)Ap[t] + ((uint32_t)(kb + i) * 1024u + ulane * 16u)) : make_uint4(0, 0, 0, 0);
        } else {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    const int ks = kb + i;
                    bw[t][i] = ks < ks_hi ? ldg4((const char*)Wp[t] + ((uint32_t)ks * 1024u + ulane * 16u)) : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    const int ks = kb + i;
                    aw[t][i] = (ks < ks_hi && rowok[t]) ? ldg4((const char*)Ap[t] + ((uint32_t)ks * 1024u + ulane * 16u)) : make_uint4(0, 0, 0, 0);
                }
        }
        if (kb == ks_lo) tp(g.ph, 6);
        if (kb == ks_lo && do_stats && !stats_early) {
            const int r = row0 + (tid >> 2);
            if (r < g.R) {
                const float2* sp = (const float2*)g.stats + r;
                c0 = ldgf2(sp).x;
                for (int t = tid & 3; t < tiles; t += 4) {
                    const float2 v = ldgf2(sp + (size_t)t * g.R);
                    const float dv = v.x - c0; s1 += dv; s2 += v.y; s3 += dv * dv;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i)
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)
#pragma unroll
                for (int ct = 0; ct < 2; ++ct)
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, aw[rt][i]),
                                                                          __builtin_bit_cast(bf16x8_t, bw[ct][i]), acc[rt][ct], 0, 0, 0);
    }
    tp(g.ph, 2);
    if (stats_early && row0 + (tid >> 2) < g.R) {
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if ((tid & 3) + 4 * j < tiles) { const float dv = sv[j].x - c0; s1 += dv; s2 += sv[j].y; s3 += dv * dv; }
    }
    if (g.stats) {
        s1 = quad_sum(s1);
        s2 = quad_sum(s2);
        s3 = quad_sum(s3);
        if (do_stats && (tid & 3) == 0) {
            const float mean = c0 + s1 / tiles;   // s1, s3: sums of the tile means' distances from c0 and of their squares
            const float m2 = s2 + 16.f * fmaxf(s3 - s1 * s1 / tiles, 0.f);
            s_stat[tid >> 2] = mean;
            s_stat[64 + (tid >> 2)] = rsqrtf(m2 / g.K + LN_EPS);
        }
    }
    __syncthreads();
    float* red = (float*)smem;   // [wave][row tile][column tile][lane][4]
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[((wave * 8 + rt * 2 + ct) * 64 + red_slot(lane)) * 4 + i] = acc[rt][ct][i];
    __syncthreads();
    tp(g.ph, 3);
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        const int urow = erow + 32 * hh, rt = urow >> 4, rr = urow & 15, ct = ecg >> 2, r = row0 + urow;
        if (r < g.R) {
            const float mu = g.stats ? s_stat[urow] : 0.f, rstd = g.stats ? s_stat[64 + urow] : 1.f;
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = (ecg & 3) * 4 + j;
                const int src = (((rt * 2 + ct) * 64) + red_slot((rr >> 2) * 16 + col)) * 4 + (rr & 3);
                float a = red[src];
#pragma unroll
                for (int w = 1; w < 4; ++w) a += red[w * 2048 + src];
                const float csj = __uint_as_float(j == 0 ? cs4.x : j == 1 ? cs4.y : j == 2 ? cs4.z : cs4.w);
                const float bj = __uint_as_float(j == 0 ? b4.x : j == 1 ? b4.y : j == 2 ? b4.z : b4.w);
                if (g.stats) a = rstd * (a - mu * csj);
                v[j] = a + bj;
            }
            if (g.epi == SE_GELU) {
                stw64(g.out + toff(r, n0, g.N >> 5),
                      (uint64_t)pack_bf16(gelu_s(v[0]), gelu_s(v[1])) | ((uint64_t)pack_bf16(gelu_s(v[2]), gelu_s(v[3])) << 32));
            } else if (g.epi == SE_QKV) {
                const uint64_t pk = (uint64_t)pack_bf16(v[0], v[1]) | ((uint64_t)pack_bf16(v[2], v[3]) << 32);
                if (n0 < D.d) {
                    stw64(g.out + toff(r, n0, D.d >> 5), pk);
                } else {
                    const int b = kv_b[hh], node = r - b * D.M;
                    const int cc = kv_cc + ecg * 4, head = cc >> 6, dim = cc & 63;
                    const int pos = kv_L[hh] + node;
                    if (pos < D.maxpos && kv_rows[hh] > 0) {
                        const size_t hb = ((((size_t)g.layer * D.Bmax + b) * D.nH + head) * kv_cap(D.maxpos)) * 64;
                        if (kv_which) {
                            bf16_t* vp = (bf16_t*)s.Vc + hb + vc_off(pos, dim);   // four dimensions of one position: four lanes of a value tile
#pragma unroll
                            for (int j = 0; j < 4; ++j) stw16(vp + j * 8, f2bf(v[j]));
                        } else {
                            stw64((bf16_t*)s.Kc + hb + kc_off(pos, dim), pk);   // four dimensions of one key: half of a lane's piece
                        }
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// linear-map unit for many rows (B * M >= 256): 64 rows x 64 columns (four column tiles).
// Same scheme as above (wave w owns a quarter of the k-steps, operands straight into MFMA
// registers, partial sums added in wave order through LDS), but every A fragment is used for
// four column tiles, so a compute unit ingests 256 KB per 64 x 64 outputs instead of 640 KB.
// All epilogues, including the residual update with the statistics of the new rows.
// ---------------------------------------------------------------------------
// Epilogue of the many-row units for one thread's four outputs v[0..3] of row r, columns
// n0 .. n0 + 3 (inside column tile `tile`): activation / residual / cache scatter as the map
// asks.  The four threads of a row (tid & 3) hold a tile's 16 columns between them; ACC: the four lanes c, c + 16,
// c + 32, c + 48 of a wave do (the layout of an MFMA result whose first operand was the weight tile), and for the
// residual update every lane of the wave calls (its tile statistics are lane exchanges), `live` saying whether the
// lane's outputs exist.
// Cache row of row r of the QKV map: sequence and position, or a negative position if the row has none (beyond the
// map's rows or the cache, or a finished sequence).  Asked once per row before the stores: the two loads are a trip to
// L2 each, and between the write-through stores of an epilogue the compiler does not move or merge them.
__device__ __forceinline__ void wide_kv_row(const GemmD& g, int r, int& kv_b, int& kv_pos) {
    const Dims& D = sP.D;
    const DevState& s = sP.s;
    kv_b = 0; kv_pos = -1;
    if (g.epi != SE_QKV || r >= g.R) return;
    kv_b = r / D.M;
    const int pos = ldg(s.L + kv_b) + (r - kv_b * D.M);
    if (pos < D.maxpos && ldg(s.n_rows + kv_b) > 0) kv_pos = pos;
}
template <bool ACC = false, int EPI = -1>   // EPI >= 0: the map's epilogue as a compile-time constant (the caller has branched on it once)
__device__ __forceinline__ void wide_store(const GemmD& g, int r, int n0, int tile, const float (&v)[4], const uint4& xr, bool live = true,
                                           int kv_b = 0, int kv_pos = -1) {
    const StepParams& P = sP;
    const Dims& D = P.D;
    const DevState& s = P.s;
    const int tid = threadIdx.x;
    {
        const bool full = n0 + 3 < g.N;
        switch (EPI >= 0 ? EPI : g.epi) {
        case SE_GELU:
            stw64(g.out + toff(r, n0, g.N >> 5),
                  (uint64_t)pack_bf16(gelu_s(v[0]), gelu_s(v[1])) | ((uint64_t)pack_bf16(gelu_s(v[2]), gelu_s(v[3])) << 32));
            break;
        case SE_LOGITS:
        case SE_F32:
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (full || n0 + j < g.N) stwf(g.outf + (size_t)r * g.N + n0 + j, v[j]);
            break;
        case SE_RESID: {
            // residual update; the statistics of the tile's 16 columns come from the four threads of the row
            const float x0 = __uint_as_float(xr.x) + v[0], x1 = __uint_as_float(xr.y) + v[1];
            const float x2 = __uint_as_float(xr.z) + v[2], x3 = __uint_as_float(xr.w) + v[3];
            if (live) {
                stwf2(s.x + (size_t)r * g.N + n0, x0, x1);
                stwf2(s.x + (size_t)r * g.N + n0 + 2, x2, x3);
                stw64(g.out + toff(r, n0, g.N >> 5), (uint64_t)pack_bf16(x0, x1) | ((uint64_t)pack_bf16(x2, x3) << 32));
            }
            float sum = x0 + x1 + x2 + x3;
            sum = ACC ? rows_sum(sum) : quad_sum(sum);
            const float mean = sum * (1.f / 16.f);
            float m2 = (x0 - mean) * (x0 - mean) + (x1 - mean) * (x1 - mean) + (x2 - mean) * (x2 - mean) + (x3 - mean) * (x3 - mean);
            m2 = ACC ? rows_sum(m2) : quad_sum(m2);
            if (live && (ACC ? (tid & 48) == 0 : (tid & 3) == 0)) stwf2(g.stats_out + ((size_t)tile * g.R + r) * 2, mean, m2);
            break;
        }
        case SE_QKV: {
            const uint64_t pk = (uint64_t)pack_bf16(v[0], v[1]) | ((uint64_t)pack_bf16(v[2], v[3]) << 32);
            if (n0 < D.d) { stw64(g.out + toff(r, n0, D.d >> 5), pk); break; }
            // key / value columns: row r is position kv_pos of sequence kv_b's cache (wide_kv_row; negative: no such row)
            const int which = n0 >= 2 * D.d, cc = n0 - (which + 1) * D.d, head = cc >> 6, dim = cc & 63;
            if (kv_pos >= 0) {
                const size_t hb = ((((size_t)g.layer * D.Bmax + kv_b) * D.nH + head) * kv_cap(D.maxpos)) * 64;
                if (which) {
                    bf16_t* vp = (bf16_t*)s.Vc + hb + vc_off(kv_pos, dim);   // four dimensions of one position: four lanes of a value tile
#pragma unroll
                    for (int j = 0; j < 4; ++j) stw16(vp + j * 8, f2bf(v[j]));
                } else {
                    stw64((bf16_t*)s.Kc + hb + kc_off(kv_pos, dim), pk);   // four dimensions of one key: half of a lane's piece
                }
            }
            break;
        }
        default: break;
        }
    }
}

// ---------------------------------------------------------------------------
// 128 x 128 unit of the many-row kernel (maps with at least 128 such units).  The reduction
// runs in stages of two k-steps: a stage is 16 activation tiles and 16 weight tiles of 1 KiB
// (tile = one MFMA operand, already in register layout in memory), copied by the four waves
// into LDS and read from there by all of them: wave (wr, wc) owns rows 64 wr.., columns 64 wc..
// (4 x 4 MFMA tiles), so every operand byte fetched from memory feeds four times as many MFMAs
// as in the 64 x 64 unit.  Two stages sit in LDS (2 x 32 KiB) and four more are in flight in
// registers.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void gemm_big_impl(const GemmD& g, int nt, int row0) {
    constexpr int NRT = 4, NCT = 4;
    const StepParams& P = sP;
    extern __shared__ uint4 smem[];
    float* s_stat = (float*)((char*)smem + ST_WIDE_TILE_BYTES);   // [2][128]: mean, 1/std of the unit's rows
    const DevState& s = P.s;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int nks = g.K >> 5, NT = cdiv(g.N, 16), RT = cdiv(g.R, 16);
    const int nch = nks >> 1;
    const int wr = wave >> 1, wc = wave & 1;
    const uint32_t ulane = (uint32_t)lane;
    // loader: wave w copies tiles T = w + 4 j of a stage; T < 16: activation tile T >> 1 of the
    // unit's eight row tiles, k-step T & 1 of the stage; T >= 16: weight tile (T - 16) >> 1
    const uint4* src[8];
    bool ok[8];
    const int kk_w = wave & 1;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int T = wave + 4 * j;
        if (j < 4) {
            const int rt = (row0 >> 4) + (T >> 1);
            ok[j] = rt < RT;
            src[j] = uniform_ptr((const uint4*)g.X + ((size_t)(ok[j] ? rt : 0) * nks + kk_w) * 64);
        } else {
            const int ct = nt + ((T - 16) >> 1);
            ok[j] = ct < NT;
            src[j] = uniform_ptr(g.Wp + ((size_t)(ok[j] ? ct : 0) * nks + kk_w) * 64);
        }
    }
    // Every load is unconditional (a branch per load would serialise them): tiles beyond the map's
    // last row or column tile re-read tile 0 and stages beyond the last re-read the last one; such
    // operands only reach accumulators of rows and columns that the epilogue never stores, or
    // stages that are never multiplied.  K is a multiple of 64 here, so a stage is always whole.
    auto gload = [&](int c, uint4 (&G)[8]) {
        const uint32_t off = (uint32_t)(c < nch ? c : nch - 1) * 2048u + ulane * 16u;
#pragma unroll
        for (int j = 0; j < 8; ++j) G[j] = ldg4((const char*)src[j] + off);
    };
    auto lstore = [&](int st, const uint4 (&G)[8]) {
#pragma unroll
        for (int j = 0; j < 8; ++j) smem[(st * 32 + wave + 4 * j) * 64 + lane] = G[j];
    };
    f32x4_t acc[NCT][NRT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) acc[ct][rt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    auto compute = [&](int st) {
        uint4 a[2][NRT], b[2][NCT];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt) a[kk][rt] = smem[(st * 32 + (wr * 4 + rt) * 2 + kk) * 64 + lane];
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) b[kk][ct] = smem[(st * 32 + 16 + (wc * 4 + ct) * 2 + kk) * 64 + lane];
        }
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, b[kk][ct]);
#pragma unroll
                for (int rt = 0; rt < NRT; ++rt)   // weights first: a lane then holds four consecutive columns of one row
                    acc[ct][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfrag, __builtin_bit_cast(bf16x8_t, a[kk][rt]),
                                                                          acc[ct][rt], 0, 0, 0);
            }
    };
    // four stages are in flight in registers besides the one being multiplied: with ~2 us from a
    // load's issue to its data under load, a compute unit needs over 100 KB outstanding to keep
    // its matrix cores fed
    // row statistics of the LayerNorm folded into the map: two threads per row merge the row's tile statistics.
    // Their first 64 tiles (all of them up to K = 1024) are requested BEFORE the operand stages: asked for after
    // them they would return behind 128 KB of operands and the first stage's copy into LDS would wait for them.
    const bool do_stats = g.stats != nullptr;
    const int tiles = g.K >> 4;
    const int srow = tid >> 1, sr = row0 + srow;
    const float2* sp = (const float2*)g.stats + (sr < g.R ? sr : 0);
    float2 sv[32];
    float c0 = 0.f;   // shift of the tile means, see gemm_unit
    if (do_stats) {
        c0 = ldgf2(sp).x;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const int t = (tid & 1) + 2 * j;
            sv[j] = ldgf2(sp + (size_t)(t < tiles ? t : 0) * g.R);
        }
    }
    uint4 G0[8], G1[8], G2[8], G3[8];
    gload(0, G0);
    gload(1, G1);
    gload(2, G2);
    gload(3, G3);
    if (do_stats) {
        float s1 = 0.f, s2 = 0.f, s3 = 0.f;
        if (sr < g.R) {
#pragma unroll
            for (int j = 0; j < 32; ++j)
                if ((tid & 1) + 2 * j < tiles) { const float dv = sv[j].x - c0; s1 += dv; s2 += sv[j].y; s3 += dv * dv; }
            for (int t = 64 + (tid & 1); t < tiles; t += 2) {   // K > 1024
                const float2 v = ldgf2(sp + (size_t)t * g.R);
                const float dv = v.x - c0; s1 += dv; s2 += v.y; s3 += dv * dv;
            }
        }
        s1 = pair_sum(s1);
        s2 = pair_sum(s2);
        s3 = pair_sum(s3);
        if ((tid & 1) == 0) {
            const float mean = c0 + s1 / tiles;   // s1, s3: sums of the tile means' distances from c0 and of their squares
            const float m2 = s2 + 16.f * fmaxf(s3 - s1 * s1 / tiles, 0.f);
            s_stat[srow] = mean;
            s_stat[128 + srow] = rsqrtf(m2 / g.K + LN_EPS);
        }
    }
    lstore(0, G0);
    if (4 < nch) gload(4, G0);
    __syncthreads();
    // One round = four stages.  On entry stage c sits in LDS half 0 and G1, G2, G3, G0 hold (or
    // await) stages c + 1 .. c + 4.  While all of a round's loads exist they are issued without
    // a branch, so that the waits before the LDS copies count exactly the loads issued since;
    // the last rounds guard each group of loads and each multiplication.
    auto round = [&](int c, auto all) {
        constexpr bool ALL = decltype(all)::value;
        compute(0);
        lstore(1, G1);
        if (ALL || c + 5 < nch) gload(c + 5, G1);
        __syncthreads();
        if (ALL || c + 1 < nch) compute(1);
        lstore(0, G2);
        if (ALL || c + 6 < nch) gload(c + 6, G2);
        __syncthreads();
        if (ALL || c + 2 < nch) compute(0);
        lstore(1, G3);
        if (ALL || c + 7 < nch) gload(c + 7, G3);
        __syncthreads();
        if (ALL || c + 3 < nch) compute(1);
        lstore(0, G0);
        if (ALL || c + 8 < nch) gload(c + 8, G0);
        __syncthreads();
    };
    tp(g.ph, 7);
    int c = 0;
    for (; c + 8 < nch; c += 4) round(c, std::true_type{});
    for (; c < nch; c += 4) round(c, std::false_type{});
    tp(g.ph, 2);   // reduction done
    // Epilogue straight from the accumulators: with the weight tile as the MFMA's first operand, lane (lc, gq) of wave
    // (wr, wc) holds, for each of its 4 x 4 tiles, row 16 rt + lc of the wave's 64 rows and columns 4 gq .. 4 gq + 3 of
    // the tile: four consecutive outputs of one row, which is what every store of the epilogue takes (no trip of
    // the 128 x 128 results through LDS).
    const int lc = lane & 15, gq = lane >> 4;
    const bool resid = g.epi == SE_RESID;
    uint4 cs4[NCT], b4[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int tile = nt + 4 * wc + ct, n0 = tile * 16 + 4 * gq;
        cs4[ct] = b4[ct] = make_uint4(0, 0, 0, 0);
        if (tile < NT) {
            if (g.colsum) cs4[ct] = ldg4(g.colsum + n0);
            if (g.bias) b4[ct] = ldg4(g.bias + n0);
        }
    }
    tp(g.ph, 3);
    if (g.epi == SE_QKV && nt * 16 >= 2 * P.D.d) {
        // A unit of value columns.  The value cache keeps eight consecutive positions of one dimension together
        // (16 bytes), and a lane holds four dimensions of one position: stored from here the unit would be 64
        // two-byte stores per lane.  The unit's values go through LDS instead ([dimension][row], rows padded to
        // 130 so that a wave's dimensions fall into different banks) and leave as whole 16-byte pieces: a thread
        // owns one dimension (tid & 127), each half of the workgroup every other piece of eight positions of every
        // sequence that has rows in the unit; a piece that the unit's rows cover only in part (the sequence's
        // length is not a multiple of eight, or its rows continue in another unit) is stored position by position.
        const Dims& D = P.D;
        constexpr int VT = 130;
        bf16_t* vt = (bf16_t*)smem;
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
            const int urow = 64 * wr + 16 * rt + lc;
            const float mu = do_stats ? s_stat[urow] : 0.f;
            const float rstd = do_stats ? s_stat[128 + urow] : 1.f;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct)
            {
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float a = acc[ct][rt][j];
                    const float csj = __uint_as_float(j == 0 ? cs4[ct].x : j == 1 ? cs4[ct].y : j == 2 ? cs4[ct].z : cs4[ct].w);
                    const float bj = __uint_as_float(j == 0 ? b4[ct].x : j == 1 ? b4[ct].y : j == 2 ? b4[ct].z : b4[ct].w);
                    if (do_stats) a = rstd * (a - mu * csj);
                    v[j] = a + bj;
                }
                const uint32_t p01 = pack_bf16(v[0], v[1]), p23 = pack_bf16(v[2], v[3]);
                bf16_t* w = vt + (64 * wc + 16 * ct + 4 * gq) * VT + urow;
                w[0] = (bf16_t)p01; w[VT] = (bf16_t)(p01 >> 16); w[2 * VT] = (bf16_t)p23; w[3 * VT] = (bf16_t)(p23 >> 16);
            }
        }
        __syncthreads();
        const int udim = tid & 127, half = wave >> 1;
        const int col = nt * 16 + udim - 2 * D.d, head = col >> 6, dd = col & 63;
        const bool col_ok = nt * 16 + udim < g.N;
        const int r_end = row0 + 128 < g.R ? row0 + 128 : g.R;
        const bf16_t* vrow = vt + udim * VT;
        for (int b = row0 / D.M; b * D.M < r_end; ++b) {
            const int n_lo = row0 > b * D.M ? row0 - b * D.M : 0, n_hi = r_end - b * D.M < D.M ? r_end - b * D.M : D.M;
            if (ldg(s.n_rows + b) <= 0) continue;
            const int L = ldg(s.L + b);
            const int p_lo = L + n_lo, p_hi = L + n_hi < D.maxpos ? L + n_hi : D.maxpos;
            if (p_hi <= p_lo) continue;
            const size_t hb = ((((size_t)g.layer * D.Bmax + b) * D.nH + head) * kv_cap(D.maxpos)) * 64;
            const int ubase = b * D.M - L - row0;   // position p is row p + ubase of the unit
            for (int o = (p_lo >> 3) + half; o <= ((p_hi - 1) >> 3); o += 2) {
                const int p0 = o * 8;
                uint32_t hw[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    int i = p0 + e + ubase;
                    i = i < 0 ? 0 : i > 127 ? 127 : i;
                    hw[e] = vrow[i];
                }
                bf16_t* dst = (bf16_t*)s.Vc + hb + vc_off(p0, dd);
                if (!col_ok) continue;
                if (p0 >= p_lo && p0 + 8 <= p_hi) {
                    stw64(dst, (uint64_t)(hw[0] | (hw[1] << 16)) | ((uint64_t)(hw[2] | (hw[3] << 16)) << 32));
                    stw64(dst + 4, (uint64_t)(hw[4] | (hw[5] << 16)) | ((uint64_t)(hw[6] | (hw[7] << 16)) << 32));
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (p0 + e >= p_lo && p0 + e < p_hi) stw16(dst + e, (bf16_t)hw[e]);
                }
            }
        }
        return;
    }
    // one copy of the loops per kind of epilogue, chosen once: inside them the kind is a compile-time constant, so
    // the 16 stores of a lane are straight-line code (no branch chain and no read of the parameter block per store)
    int kv_b[NRT], kv_pos[NRT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) wide_kv_row(g, row0 + 64 * wr + 16 * rt + lc, kv_b[rt], kv_pos[rt]);
    auto finish = [&](auto kind) {
        constexpr int EPI = decltype(kind)::value;
        if constexpr (EPI == SE_GELU || EPI == SE_QKV) {
            // bf16 outputs in 16-byte pieces (eight consecutive columns of a row: a lane's piece of an operand tile, or
            // of a key tile of the cache).  A lane holds four columns, the lane 16 further on the other four of the
            // piece: two row tiles at a time, the lanes of the even 16-lane rows hand over their half of the second
            // tile's piece and get the other half of the first tile's (one row swap per register), so that every lane
            // stores one whole piece instead of two halves: half as many store requests.
            const Dims& D = P.D;
#pragma unroll
            for (int rp = 0; rp < NRT / 2; ++rp) {
                const int urow0 = 64 * wr + 32 * rp + lc;   // the pair's rows: urow0 and urow0 + 16
                float mu[2], rstd[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    mu[h] = do_stats ? s_stat[urow0 + 16 * h] : 0.f;
                    rstd[h] = do_stats ? s_stat[128 + urow0 + 16 * h] : 1.f;
                }
                const int mine = gq & 1;   // which of the two rows this lane stores
                const int r = row0 + urow0 + 16 * mine;
                const int my_b = mine ? kv_b[2 * rp + 1] : kv_b[2 * rp], my_pos = mine ? kv_pos[2 * rp + 1] : kv_pos[2 * rp];
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct) {
                    const int tile = nt + 4 * wc + ct;
                    uint32_t w[2][2];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        float v[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            float a = acc[ct][2 * rp + h][j];
                            const float csj = __uint_as_float(j == 0 ? cs4[ct].x : j == 1 ? cs4[ct].y : j == 2 ? cs4[ct].z : cs4[ct].w);
                            const float bj = __uint_as_float(j == 0 ? b4[ct].x : j == 1 ? b4[ct].y : j == 2 ? b4[ct].z : b4[ct].w);
                            if (do_stats) a = rstd[h] * (a - mu[h] * csj);
                            v[j] = EPI == SE_GELU ? gelu_s(a + bj) : a + bj;
                        }
                        w[h][0] = pack_bf16(v[0], v[1]);
                        w[h][1] = pack_bf16(v[2], v[3]);
                    }
                    // first row's halves of the odd lane rows <-> second row's halves of the even lane rows
                    const vadusa_u32x2 s0 = __builtin_amdgcn_permlane16_swap(w[0][0], w[1][0], false, false);
                    const vadusa_u32x2 s1 = __builtin_amdgcn_permlane16_swap(w[0][1], w[1][1], false, false);
                    const uint4 piece = make_uint4(s0.x, s1.x, s0.y, s1.y);   // columns np .. np + 7 of row r
                    const int np = tile * 16 + 8 * (gq >> 1);
                    if (r >= g.R || tile >= NT) continue;
                    if (EPI == SE_GELU) stw128(g.out + toff(r, np, g.N >> 5), piece);
                    else if (np < D.d) stw128(g.out + toff(r, np, D.d >> 5), piece);
                    else if (my_pos >= 0) {   // key columns (a unit of value columns went the other way above)
                        const int cc = np - D.d, head = cc >> 6, dim = cc & 63;
                        const size_t hb = ((((size_t)g.layer * D.Bmax + my_b) * D.nH + head) * kv_cap(D.maxpos)) * 64;
                        stw128((bf16_t*)s.Kc + hb + kc_off(my_pos, dim), piece);
                    }
                }
            }
            return;
        }
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
            const int urow = 64 * wr + 16 * rt + lc, r = row0 + urow;
            const float mu = do_stats ? s_stat[urow] : 0.f;
            const float rstd = do_stats ? s_stat[128 + urow] : 1.f;
            uint4 xr4[NCT];
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const int tile = nt + 4 * wc + ct, n0 = tile * 16 + 4 * gq;
                xr4[ct] = make_uint4(0, 0, 0, 0);
                if (EPI == SE_RESID && tile < NT && r < g.R) xr4[ct] = ldg4(s.x + (size_t)r * g.N + n0);
            }
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const int tile = nt + 4 * wc + ct, n0 = tile * 16 + 4 * gq;
                const bool live = r < g.R && tile < NT && n0 < g.N;
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float a = acc[ct][rt][j];
                    const float csj = __uint_as_float(j == 0 ? cs4[ct].x : j == 1 ? cs4[ct].y : j == 2 ? cs4[ct].z : cs4[ct].w);
                    const float bj = __uint_as_float(j == 0 ? b4[ct].x : j == 1 ? b4[ct].y : j == 2 ? b4[ct].z : b4[ct].w);
                    if (do_stats) a = rstd * (a - mu * csj);
                    v[j] = a + bj;
                }
                // the residual update's tile statistics are lane exchanges: every lane takes part, live or not
                if (EPI == SE_RESID || live) wide_store<true, EPI>(g, r, n0, tile, v, xr4[ct], live, kv_b[rt], kv_pos[rt]);
            }
        }
    };
    switch (g.epi) {
    case SE_GELU: finish(std::integral_constant<int, SE_GELU>{}); break;
    case SE_QKV: finish(std::integral_constant<int, SE_QKV>{}); break;
    case SE_RESID: finish(std::integral_constant<int, SE_RESID>{}); break;
    case SE_LOGITS: finish(std::integral_constant<int, SE_LOGITS>{}); break;
    default: finish(std::integral_constant<int, SE_F32>{}); break;
    }
}
__device__ __forceinline__ void gemm_wide_unit(int ph_, int u_) {
    constexpr int NRT = 4, NCT = 4, CH = 2;
    const int ph_u = __builtin_amdgcn_readfirstlane(ph_), u_u = __builtin_amdgcn_readfirstlane(u_);
    const StepParams& P = sP;
    GemmD g;
    int nt, row0;
    if (!describe_gemm<true>(ph_u, u_u, g, nt, row0)) return;
    if (g.G == 8) { gemm_big_impl(g, nt, row0); return; }
    extern __shared__ uint4 smem[];
    float* s_stat = (float*)((char*)smem + ST_WIDE_TILE_BYTES);
    const Dims& D = P.D;
    const DevState& s = P.s;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int nks = g.K >> 5, NT = cdiv(g.N, 16);
    const int ks_lo = (nks * wave) >> 2, ks_hi = (nks * (wave + 1)) >> 2;
    const uint4* Wp[NCT];
    bool tile_ok[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        tile_ok[ct] = nt + ct < NT;   // a tile beyond the last one: skipped
        Wp[ct] = uniform_ptr(g.Wp + (size_t)(tile_ok[ct] ? nt + ct : nt) * nks * 64);
    }
    const uint4* Ap[NRT];
    bool rowok[NRT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
        rowok[rt] = row0 + rt * 16 < g.R;
        Ap[rt] = uniform_ptr((const uint4*)g.X + (size_t)(rowok[rt] ? (row0 >> 4) + rt : 0) * nks * 64);
    }
    const uint32_t ulane = (uint32_t)lane;
    f32x4_t acc[NCT][NRT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) acc[ct][rt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    // epilogue inputs of this thread: row tid / 4, columns 4 (tid % 4) .. + 3 of every tile
    const int erow = tid >> 2, er = row0 + erow;
    uint4 cs4[NCT], b4[NCT], xr4[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int n0 = (nt + ct) * 16 + (tid & 3) * 4;
        cs4[ct] = b4[ct] = xr4[ct] = make_uint4(0, 0, 0, 0);
        if (tile_ok[ct]) {
            if (g.colsum) cs4[ct] = ldg4(g.colsum + n0);
            if (g.bias) b4[ct] = ldg4(g.bias + n0);
            if (g.epi == SE_RESID && er < g.R) xr4[ct] = ldg4(s.x + (size_t)er * g.N + n0);
        }
    }
    int kv_b, kv_pos;
    wide_kv_row(g, er, kv_b, kv_pos);
    float s1 = 0.f, s2 = 0.f, s3 = 0.f, c0 = 0.f;   // c0: shift of the tile means, see gemm_unit
    const int tiles = g.K >> 4;
    const bool do_stats = g.stats != nullptr;
    if (do_stats && er < g.R) {   // four threads per row, each merges a quarter of the row's tile statistics
        const float2* sp = (const float2*)g.stats + er;
        c0 = ldgf2(sp).x;
        for (int t0 = tid & 3; t0 < tiles; t0 += 32) {
            float2 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int t = t0 + 4 * j;
                v[j] = t < tiles ? ldgf2(sp + (size_t)t * g.R) : make_float2(0.f, 0.f);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
                    if (t0 + 4 * j < tiles) { const float dv = v[j].x - c0; s1 += dv; s2 += v[j].y; s3 += dv * dv; }
        }
    }
    // two chunks of CH k-steps in flight alternately: the loads of one chunk overlap the MFMAs of
    // the other (chunks beyond the wave's range load nothing and multiply zeros)
    // Every load is unconditional (a branch per load would serialise them): a tile beyond the
    // map's last row or column tile re-reads a valid one and only reaches accumulators that the
    // epilogue never stores; a k-step beyond the wave's range re-reads the map's last k-step and
    // is not multiplied.
    auto load_chunk = [&](int kb, uint4 (&bw)[NCT][CH], uint4 (&aw)[NRT][CH]) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const uint32_t off = (uint32_t)(kb + i < nks ? kb + i : nks - 1) * 1024u + ulane * 16u;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) bw[ct][i] = ldg4((const char*)Wp[ct] + off);
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt) aw[rt][i] = ldg4((const char*)Ap[rt] + off);
        }
    };
    auto mfma_chunk = [&](int kb, const uint4 (&bw)[NCT][CH], const uint4 (&aw)[NRT][CH]) {
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (kb + i < ks_hi)
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, bw[ct][i]);
#pragma unroll
                for (int rt = 0; rt < NRT; ++rt)
                    acc[ct][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, aw[rt][i]), bfrag,
                                                                          acc[ct][rt], 0, 0, 0);
            }
    };
    {
        uint4 bw0[NCT][CH], aw0[NRT][CH], bw1[NCT][CH], aw1[NRT][CH];
        load_chunk(ks_lo, bw0, aw0);
        for (int kb = ks_lo; kb < ks_hi; kb += 2 * CH) {
            load_chunk(kb + CH, bw1, aw1);
            mfma_chunk(kb, bw0, aw0);
            load_chunk(kb + 2 * CH, bw0, aw0);
            mfma_chunk(kb + CH, bw1, aw1);
        }
    }
    if (do_stats) {
        s1 = quad_sum(s1);
        s2 = quad_sum(s2);
        s3 = quad_sum(s3);
        if ((tid & 3) == 0) {
            const float mean = c0 + s1 / tiles;   // s1, s3: sums of the tile means' distances from c0 and of their squares
            const float m2 = s2 + 16.f * fmaxf(s3 - s1 * s1 / tiles, 0.f);
            s_stat[erow] = mean;
            s_stat[64 + erow] = rsqrtf(m2 / g.K + LN_EPS);
        }
    }
    __syncthreads();
    float* red = (float*)smem;   // [wave][ct][rt][lane][4]
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[(((wave * NCT + ct) * NRT + rt) * 64 + lane) * 4 + i] = acc[ct][rt][i];
    __syncthreads();

    const int rt = erow >> 4, rr = erow & 15, r = er;
    const float mu = do_stats ? s_stat[erow] : 0.f, rstd = do_stats ? s_stat[64 + erow] : 1.f;
    auto outputs = [&](int ct, float (&v)[4]) {   // the thread's four outputs of column tile ct
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = (tid & 3) * 4 + j;
            const int src = ((ct * NRT + rt) * 64 + (rr >> 2) * 16 + col) * 4 + (rr & 3);
            float a = red[src];
#pragma unroll
            for (int w = 1; w < 4; ++w) a += red[w * (NCT * NRT * 256) + src];
            const float csj = __uint_as_float(j == 0 ? cs4[ct].x : j == 1 ? cs4[ct].y : j == 2 ? cs4[ct].z : cs4[ct].w);
            const float bj = __uint_as_float(j == 0 ? b4[ct].x : j == 1 ? b4[ct].y : j == 2 ? b4[ct].z : b4[ct].w);
            if (do_stats) a = rstd * (a - mu * csj);
            v[j] = a + bj;
        }
    };
    const bool qk_unit = g.epi == SE_QKV && (nt + NCT) * 16 <= 2 * D.d;   // query or key columns only
    if ((g.epi == SE_GELU || g.epi == SE_RESID || qk_unit) && g.N % 16 == 0) {
        // bf16 outputs leave as whole 16-byte pieces (eight consecutive columns of a row): a thread holds four columns
        // of every tile, its neighbour the other four of the piece; two tiles at a time, the even thread hands over its
        // half of the second tile's piece and gets the other half of the first tile's, and stores that piece whole
        // (the odd thread the second tile's): half as many store requests.  The residual stream's four floats go out
        // as one 16-byte store as well.  Every thread takes part in the lane exchanges, with or without a row.
        const bool odd = tid & 1;
#pragma unroll
        for (int cp = 0; cp < NCT / 2; ++cp) {
            uint32_t w[2][2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int ct = 2 * cp + h, tile = nt + ct, n0 = tile * 16 + (tid & 3) * 4;
                float v[4];
                outputs(ct, v);
                if (g.epi == SE_GELU) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = gelu_s(v[j]);
                } else if (g.epi == SE_RESID) {
                    v[0] += __uint_as_float(xr4[ct].x); v[1] += __uint_as_float(xr4[ct].y);
                    v[2] += __uint_as_float(xr4[ct].z); v[3] += __uint_as_float(xr4[ct].w);
                    const bool live = r < g.R && tile_ok[ct];
                    if (live) stw128(s.x + (size_t)r * g.N + n0, make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])));
                    // the statistics of the tile's 16 columns come from the four threads of the row
                    const float mean = quad_sum(v[0] + v[1] + v[2] + v[3]) * (1.f / 16.f);
                    const float m2 = quad_sum((v[0] - mean) * (v[0] - mean) + (v[1] - mean) * (v[1] - mean) +
                                              (v[2] - mean) * (v[2] - mean) + (v[3] - mean) * (v[3] - mean));
                    if (live && (tid & 3) == 0) stwf2(g.stats_out + ((size_t)tile * g.R + r) * 2, mean, m2);
                }
                w[h][0] = pack_bf16(v[0], v[1]);
                w[h][1] = pack_bf16(v[2], v[3]);
            }
            const uint32_t t0 = (uint32_t)dpp_perm<0xB1>((int)(odd ? w[0][0] : w[1][0]));   // the neighbour's half of this thread's piece
            const uint32_t t1 = (uint32_t)dpp_perm<0xB1>((int)(odd ? w[0][1] : w[1][1]));
            const uint4 piece = odd ? make_uint4(t0, t1, w[1][0], w[1][1]) : make_uint4(w[0][0], w[0][1], t0, t1);
            const int ct = 2 * cp + (odd ? 1 : 0), np = (nt + ct) * 16 + ((tid & 3) >> 1) * 8;
            if (r >= g.R || !tile_ok[ct]) continue;
            if (g.epi != SE_QKV) stw128(g.out + toff(r, np, g.N >> 5), piece);
            else if (np < D.d) stw128(g.out + toff(r, np, D.d >> 5), piece);
            else if (kv_pos >= 0) {
                const int cc = np - D.d, head = cc >> 6, dim = cc & 63;
                const size_t hb = ((((size_t)g.layer * D.Bmax + kv_b) * D.nH + head) * kv_cap(D.maxpos)) * 64;
                stw128((bf16_t*)s.Kc + hb + kc_off(kv_pos, dim), piece);
            }
        }
        return;
    }
    if (r >= g.R) return;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int n0 = (nt + ct) * 16 + (tid & 3) * 4;
        if (!tile_ok[ct] || n0 >= g.N) continue;
        float v[4];
        outputs(ct, v);
        wide_store(g, r, n0, nt + ct, v, xr4[ct], true, kv_b, kv_pos);
    }
}

// ---------------------------------------------------------------------------
// tree-masked attention unit (Sec. 2.1): one head, 16 query rows of one
// sequence.  Keys: cache positions [0, L) and the rows of this forward at
// L + m where the query's mask bit m is set.  The four waves take 32-key blocks
// round-robin with a private online softmax (S^T = K Q^T, O^T += V^T P^T on
// MFMA), then merge through LDS.  The cache keeps K and V^T in blocks of 32 keys, each already in the
// layout of the MFMA operands (kc_off / vc_off in common.h).
// ---------------------------------------------------------------------------
// ALLQ (many-row kernel, at least one (sequence, head) per compute unit): a unit is one or more whole
// (sequence, head) pairs (attn_ppu); a wave takes a query tile over all its key blocks, so the waves of a pair
// read the same K / V blocks (once from L2, then from the compute unit's L1), nothing is merged across
// waves, and the result goes from the accumulators straight to memory.  (Where pairs are too few for that,
// the waves that a pair's query tiles do not need split the tiles' key blocks and merge through LDS.)
template <bool ALLQ, bool CAUSAL>
__device__ __forceinline__ void attn_unit(int ph_, int u_) {
    const int layer = (__builtin_amdgcn_readfirstlane(ph_) - 1) / 5, u = __builtin_amdgcn_readfirstlane(u_);
    const StepParams& P = sP;
    extern __shared__ uint4 smem[];
    const Dims& D = P.D;
    const DevState& s = P.s;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, gq = lane >> 4, c = lane & 15;
    // unit = (query tile) * pad8(B * nH) + (sequence, head): the query tiles of one head run on
    // one XCD (workgroup i is on XCD i mod 8) and share its L2 for that head's K / V rows
    const int BH = pad8(D.B * D.nH);
    int bh, qt, h, b;
    // ALLQ: the workgroup's four waves are 4 / wpq tile slots of wpq waves each (wpq = waves per query tile, which
    // split the tile's key blocks); slot t is query tile t % qts of the unit's pair t / qts.  With three or four
    // query tiles a unit is one pair and a wave takes a tile; with two tiles (one tile) a unit is up to two (four)
    // pairs (attn_ppu).
    const int n_qt = (D.M + 15) >> 4;
    const int ppu = ALLQ ? attn_ppu(P) : 1, qts = n_qt >= 3 ? 4 : n_qt;
    const int wpq = !ALLQ ? 4 : 4 / (qts * ppu);
    bool live = true;   // ALLQ: the wave's slot has a pair and a query tile
    if (ALLQ) {
        const int t = wave / wpq;
        bh = u * ppu + t / qts;
        qt = t % qts;
        live = bh < D.B * D.nH && qt * 16 < D.M;
        if (!live) { if (wpq == 1) return; bh = 0; qt = 0; }   // (wpq > 1: a workgroup barrier follows, the wave stays)
    }
    else if ((BH & (BH - 1)) == 0) { bh = u & (BH - 1); qt = u >> __builtin_ctz(BH); }   // no division in the usual case
    else { bh = u % BH; qt = u / BH; }
    if (!ALLQ && bh >= D.B * D.nH) return;
    if ((D.nH & (D.nH - 1)) == 0) { h = bh & (D.nH - 1); b = bh >> __builtin_ctz(D.nH); }
    else { h = bh % D.nH; b = bh / D.nH; }
    // everything the unit needs before its first key block is requested at once: row count,
    // committed length, the queries, the mask words (one memory latency instead of three)
    const bool seq_cached = b < ST_SEQ_CACHE;
    const int n_rows = seq_cached ? s_seqRows[b] : ldg(s.n_rows + b);
    const int L = seq_cached ? s_seqL[b] : ldg(s.L + b);
    const int node = min(qt * 16 + c, D.M - 1);
    const bf16_t* ql = (const bf16_t*)s.q + (size_t)layer * s.act_stride;
    const int qrow = b * D.M + node;
    const bf16x8_t Q0 = __builtin_bit_cast(bf16x8_t, ldg4(ql + toff(qrow, h * 64 + 8 * gq, D.d >> 5)));
    const bf16x8_t Q1 = __builtin_bit_cast(bf16x8_t, ldg4(ql + toff(qrow, h * 64 + 32 + 8 * gq, D.d >> 5)));
    // CAUSAL: the rows are a causal pass of the prefill (row n sees rows 0..n): no mask words are
    // read, a pass may have more rows than the mask table has entries.  It is a separate kernel
    // so that the step kernel's attention carries no trace of it.
    uint4 mw = make_uint4(0, 0, 0, 0);
    if constexpr (!CAUSAL) mw = ldg4(s.t_mask[P.table] + (size_t)node * MASK_WORDS);
    const uint32_t mword[4] = {mw.x, mw.y, mw.z, mw.w};
    bf16_t* att = (bf16_t*)s.att + (size_t)layer * s.act_stride;
    if (n_rows == 0) {
        if (ALLQ) {   // (the first wave of the slot stores the zeros; with wpq > 1 the waves go on to the merge's barriers)
            if (live && wave % wpq == 0) {
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
                    if (qt * 16 + c < D.M) stw64(att + toff(b * D.M + qt * 16 + c, h * 64 + dt * 16 + 4 * gq, D.d >> 5), 0ull);
            }
            if (wpq == 1) return;
            live = false;
        } else {
            const int q = tid >> 4, d0 = (tid & 15) * 4, nd = qt * 16 + q;
            if (nd < D.M) stw64(att + toff(b * D.M + nd, h * 64 + d0, D.d >> 5), 0ull);
            return;
        }
    }
    const int T = min(L + D.M, D.maxpos);
    const size_t hb = ((((size_t)layer * D.Bmax + b) * D.nH + h) * kv_cap(D.maxpos)) * 64;
    const bf16_t* Kh = (const bf16_t*)s.Kc + hb;
    const bf16_t* Vh = (const bf16_t*)s.Vc + hb;

    float m_run = -1e30f, l_run = 0.f;
    f32x4_t O[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) O[i] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    const int nblk = live ? (T + 31) >> 5 : 0;   // a wave without a tile to compute takes no key block
    // operands of one 32-key block: K rows of the two 16-key tiles (two k-steps each), V^T tiles
    // (the cache keeps them as the MFMA operands themselves: eight contiguous KiB per block; rows of the last block
    // beyond the sequence's end exist, the cache holds whole blocks, and are masked out below)
    auto load_block = [&](int blk, uint4* kv /*[8]*/) {
        const bf16_t* kb = Kh + (size_t)blk * 2048 + lane * 8;
        const bf16_t* vb = Vh + (size_t)blk * 2048 + lane * 8;
#pragma unroll
        for (int i = 0; i < 4; ++i) { kv[i] = ldg4(kb + i * 512); kv[4 + i] = ldg4(vb + i * 512); }
    };
    // Two blocks in flight behind the one being computed; the loop is unrolled over the NB buffers (no register
    // copies) and loads beyond the last block re-read it (no branch between the loads and the waits the compiler
    // counts for them).  (More blocks in flight were measured for the whole-head units, whose waves walk through
    // ten and more blocks: per layer at batch 64, 24.5 us with NB = 3, 25.5 with 4, 26.3 with 5, 27.9 with 7.)
    constexpr int NB = 3;
    uint4 buf[NB][8];
    const int blk0 = ALLQ ? wave % wpq : wave, bstep = ALLQ ? wpq : 4;   // the waves of a query tile split its key blocks
    if (nblk > 0) {
#pragma unroll
        for (int j = 0; j < NB - 1; ++j) load_block(min(blk0 + j * bstep, nblk - 1), buf[j]);
    }
    auto process = [&](const int blk, const uint4 (&cur)[8]) {
        const int p0 = blk << 5;
        const int v0 = p0 + 8 * gq;
        const uint4 a0 = cur[0], a1 = cur[1], b0 = cur[2], b1 = cur[3];
        uint4 vt[4];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) vt[dt] = cur[4 + dt];
        f32x4_t sa = (f32x4_t){0.f, 0.f, 0.f, 0.f}, sb = sa;
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a0), Q0, sa, 0, 0, 0);
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a1), Q1, sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, b0), Q0, sb, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, b1), Q1, sb, 0, 0, 0);
        // this lane: query c, keys v0 + 0..3 (sa) and v0 + 4..7 (sb)
        // online softmax of the block: scores -> probabilities (bf16 pairs in pk), running max / sum.
        // Instantiated twice: blocks inside the committed cache need no mask tests at all.
        uint32_t pk[4];
        float m_new, corr, psum = 0.f;
        auto softmax_block = [&](const unsigned okm) {
            float sc[8];
            float mx = -1e30f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float sv = (j < 4 ? sa[j] : sb[j - 4]) * 0.125f;
                sc[j] = (okm >> j) & 1u ? sv : -1e30f;
                mx = fmaxf(mx, sc[j]);
            }
            mx = rows_max(mx);
            m_new = fmaxf(m_run, mx);
            corr = __expf(m_run - m_new);
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                const float p0f = (okm >> j) & 1u ? __expf(sc[j] - m_new) : 0.f;
                const float p1f = (okm >> (j + 1)) & 1u ? __expf(sc[j + 1] - m_new) : 0.f;
                psum += p0f + p1f;
                pk[j >> 1] = pack_bf16(p0f, p1f);
            }
        };
        if (p0 + 32 > L) {   // the block reaches into the tree rows (same for the whole wave)
            unsigned okm = 0;   // which of the lane's 8 keys the query may see
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int key = v0 + j;
                bool okj = key < L;
                if (!okj && key < T) {
                    const int mm = key - L;
                    if constexpr (CAUSAL) okj = mm <= node;
                    else okj = (mword[mm >> 5] >> (mm & 31)) & 1u;
                }
                okm |= okj ? (1u << j) : 0u;
            }
            softmax_block(okm);
        } else {
            softmax_block(0xffu);
        }
        l_run = l_run * corr + psum;
        m_run = m_new;
        const bf16x8_t pfrag = __builtin_bit_cast(bf16x8_t, make_uint4(pk[0], pk[1], pk[2], pk[3]));
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            O[dt] *= corr;
            O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vt[dt]), pfrag, O[dt], 0, 0, 0);
        }
    };
    for (int blk = blk0; blk < nblk; blk += NB * bstep) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int bi = blk + i * bstep;
            if (bi < nblk) {
                load_block(min(bi + (NB - 1) * bstep, nblk - 1), buf[(i + NB - 1) % NB]);
                process(bi, buf[i]);
            }
        }
    }
    l_run = rows_sum(l_run);
    if (ALLQ && wpq == 1) {   // this lane: query c, dimensions dt * 16 + 4 gq .. + 3 of every dt
        const float inv = 1.f / l_run;
        const int nd = qt * 16 + c;
        if (nd < D.M) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
                stw64(att + toff(b * D.M + nd, h * 64 + dt * 16 + 4 * gq, D.d >> 5),
                      (uint64_t)pack_bf16(O[dt][0] * inv, O[dt][1] * inv) | ((uint64_t)pack_bf16(O[dt][2] * inv, O[dt][3] * inv) << 32));
        }
        return;
    }
    // merge the four waves: sm_m / sm_l [wave][query], sm_o [wave][dim][query]
    constexpr int SO = 16;   // floats per row of sm_o (rows of 17 as in attn_few, and the 64 x 64 unit's reduction buffer with
                             // folded lane bits, measured slower in this kernel: 1172 -> 1178 / 1174 us per step at batch 16)
    float* sm_o = (float*)smem;
    float* sm_m = sm_o + 4 * 64 * SO;
    float* sm_l = sm_m + 64;
    __syncthreads();
    if (gq == 0) { sm_m[wave * 16 + c] = m_run; sm_l[wave * 16 + c] = l_run; }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i) sm_o[(wave * 64 + dt * 16 + 4 * gq + i) * SO + c] = O[dt][i];
    __syncthreads();
    if constexpr (!ALLQ)
    {
        const int q = tid >> 4, d0 = (tid & 15) * 4, nd = qt * 16 + q;
        float mstar = sm_m[q];
#pragma unroll
        for (int w = 1; w < 4; ++w) mstar = fmaxf(mstar, sm_m[w * 16 + q]);
        float f[4], lsum = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) { f[w] = __expf(sm_m[w * 16 + q] - mstar); lsum += f[w] * sm_l[w * 16 + q]; }
        const float inv = 1.f / lsum;
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) a += f[w] * sm_o[(w * 64 + d0 + j) * SO + q];
            o[j] = a * inv;
        }
        if (nd < D.M)
            stw64(att + toff(b * D.M + nd, h * 64 + d0, D.d >> 5),
                  (uint64_t)pack_bf16(o[0], o[1]) | ((uint64_t)pack_bf16(o[2], o[3]) << 32));
    }
    else {
        // merge the waves of each tile slot (4 / wpq slots; slot t: pair t / qts of the unit, query tile t % qts)
        const int tiles_here = 4 / wpq;
        for (int t = 0; t < tiles_here; ++t) {
            const int q = tid >> 4, d0 = (tid & 15) * 4, w0 = t * wpq;
            const int bh_t = u * ppu + t / qts, nd = (t % qts) * 16 + q;
            if (bh_t >= D.B * D.nH) continue;
            const int h = bh_t % D.nH, b = bh_t / D.nH;   // (shadow the wave's own pair)
            if ((b < ST_SEQ_CACHE ? s_seqRows[b] : ldg(s.n_rows + b)) == 0) continue;   // zeros already stored
            float mstar = sm_m[w0 * 16 + q];
#pragma unroll
            for (int w = 1; w < 4; ++w)
                if (w < wpq) mstar = fmaxf(mstar, sm_m[(w0 + w) * 16 + q]);
            float f[4], lsum = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                f[w] = w < wpq ? __expf(sm_m[(w0 + w) * 16 + q] - mstar) : 0.f;
                if (w < wpq) lsum += f[w] * sm_l[(w0 + w) * 16 + q];
            }
            const float inv = 1.f / lsum;
            float o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float a = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w)
                    if (w < wpq) a += f[w] * sm_o[((w0 + w) * 64 + d0 + j) * SO + q];
                o[j] = a * inv;
            }
            if (nd < D.M)
                stw64(att + toff(b * D.M + nd, h * 64 + d0, D.d >> 5),
                      (uint64_t)pack_bf16(o[0], o[1]) | ((uint64_t)pack_bf16(o[2], o[3]) << 32));
        }
    }
}

// ---------------------------------------------------------------------------
// Attention unit of the few-row kernel (one head, 16 query rows of one sequence; the algorithm, operand layouts and
// merge of attn_unit<false>), in two parts.
//  * attn_prepare works out which (sequence, head, query tile) the unit is, lengths, block count, base addresses (as
//    workgroup-uniform values: they stay in scalar registers) and the lane's offsets and mask words;
//  * attn_few is the unit itself.
// With the descriptor in scalar registers the first key block is requested ~0.7 us into the phase (~2 us before).
// Calling attn_prepare on the other side of the grid barrier that precedes the phase, where the workgroup would
// only wait, was measured 8 us per step SLOWER: the workgroup that arrives last has no wait to hide it in, and it
// is that workgroup which sets the length of the phase.
// ---------------------------------------------------------------------------
struct AttnPrep {
    int ph, u;
    int live;                  // 0: padding unit (nothing to do)
    int layer, b, h, qt, L, T, n_rows, nblk;
    const bf16_t *Kh, *Vh, *ql;
    bf16_t* att;
    uint32_t mword[4];         // per lane: tree-mask words of the lane's query
    int node;                  // per lane: the lane's query row inside the tree
    uint32_t qoff, koff;       // per lane: element offsets of the lane's query piece and of its piece of a key / value tile
};

template <bool CAUSAL>
__device__ __forceinline__ void attn_prepare(int ph_, int u_, AttnPrep& A) {
    const int ph = __builtin_amdgcn_readfirstlane(ph_), u = __builtin_amdgcn_readfirstlane(u_);
    const StepParams& P = sP;
    const Dims& D = P.D;
    const DevState& s = P.s;
    const int lane = threadIdx.x & 63, gq = lane >> 4, c = lane & 15;
    A.ph = ph; A.u = u; A.live = 0;
    A.layer = (ph - 1) / 5;
    // unit = (query tile) * pad8(B * nH) + (sequence, head): the query tiles of one head run on one XCD
    // (workgroup i is on XCD i mod 8) and share its L2 for that head's K / V rows
    const int BH = pad8(D.B * D.nH);
    int bh;
    if ((BH & (BH - 1)) == 0) { bh = u & (BH - 1); A.qt = u >> __builtin_ctz(BH); }
    else { bh = u % BH; A.qt = u / BH; }
    if (bh >= D.B * D.nH) return;
    if ((D.nH & (D.nH - 1)) == 0) { A.h = bh & (D.nH - 1); A.b = bh >> __builtin_ctz(D.nH); }
    else { A.h = bh % D.nH; A.b = bh / D.nH; }
    A.live = 1;
    A.b = __builtin_amdgcn_readfirstlane(A.b); A.h = __builtin_amdgcn_readfirstlane(A.h); A.qt = __builtin_amdgcn_readfirstlane(A.qt);
    const bool seq_cached = A.b < ST_SEQ_CACHE;
    A.n_rows = __builtin_amdgcn_readfirstlane(seq_cached ? s_seqRows[A.b] : ldg(s.n_rows + A.b));
    A.L = __builtin_amdgcn_readfirstlane(seq_cached ? s_seqL[A.b] : ldg(s.L + A.b));
    A.T = __builtin_amdgcn_readfirstlane(min(A.L + D.M, D.maxpos));
    A.nblk = (A.T + 31) >> 5;
    const size_t hb = ((((size_t)A.layer * D.Bmax + A.b) * D.nH + A.h) * kv_cap(D.maxpos)) * 64;
    A.Kh = uniform_ptr((const bf16_t*)s.Kc + hb);
    A.Vh = uniform_ptr((const bf16_t*)s.Vc + hb);
    A.ql = uniform_ptr((const bf16_t*)s.q + (size_t)A.layer * s.act_stride);
    A.att = uniform_ptr((bf16_t*)s.att + (size_t)A.layer * s.act_stride);
    A.node = min(A.qt * 16 + c, D.M - 1);
    A.qoff = (uint32_t)toff(A.b * D.M + A.node, A.h * 64 + 8 * gq, D.d >> 5);
    A.koff = (uint32_t)(lane * 8);
    uint4 mw = make_uint4(0, 0, 0, 0);
    if constexpr (!CAUSAL) mw = ldg4(s.t_mask[P.table] + (size_t)A.node * MASK_WORDS);
    A.mword[0] = mw.x; A.mword[1] = mw.y; A.mword[2] = mw.z; A.mword[3] = mw.w;
}

template <bool CAUSAL>
__device__ __forceinline__ void attn_few(const AttnPrep& A) {
    if (!A.live) return;
    const StepParams& P = sP;
    extern __shared__ uint4 smem[];
    const Dims& D = P.D;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, gq = lane >> 4, c = lane & 15;
    const int b = A.b, h = A.h, qt = A.qt, L = A.L, T = A.T, node = A.node, nblk = A.nblk;
    bf16_t* att = A.att;
    if (A.n_rows == 0) {
        const int q = tid >> 4, d0 = (tid & 15) * 4, nd = qt * 16 + q;
        if (nd < D.M) stw64(att + toff(b * D.M + nd, h * 64 + d0, D.d >> 5), 0ull);
        return;
    }
    tp(A.ph, 5);
    const bf16x8_t Q0 = __builtin_bit_cast(bf16x8_t, ldg4(A.ql + A.qoff));
    const bf16x8_t Q1 = __builtin_bit_cast(bf16x8_t, ldg4(A.ql + A.qoff + 512));   // 32 columns on: the next k-step of the tile (64 lanes x 8 values)
    // operands of one 32-key block: the two 16-key tiles of K (two k-steps each) and the four dimension tiles of V^T,
    // kept in the cache as the MFMA operands themselves: eight contiguous KiB.  Rows of the last block beyond the
    // sequence's end exist (the cache holds whole blocks) and are masked out below.
    auto load_block = [&](int blk, uint4* kv /*[8]*/) {
        const bf16_t* kb = A.Kh + (uint32_t)blk * 2048u + A.koff;
        const bf16_t* vb = A.Vh + (uint32_t)blk * 2048u + A.koff;
#pragma unroll
        for (int i = 0; i < 4; ++i) { kv[i] = ldg4(kb + i * 512); kv[4 + i] = ldg4(vb + i * 512); }
    };
    float m_run = -1e30f, l_run = 0.f;
    f32x4_t O[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) O[i] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    // The waves take the blocks round-robin, two blocks in flight behind the one being computed.  (Measured
    // alternatives on the 64-node workload, attention phase at L ~ 400: this loop 8.0 us; contiguous quarters in
    // groups of three blocks, six blocks in flight and one softmax update per group, 9.4 us: a block costs a wave
    // ~0.4 us of softmax arithmetic and MFMA issue, and the deeper queue only delays the first block's work.)
    uint4 cur[8], nxt[8], nx2[8];
    if (wave < nblk) load_block(wave, cur);
    if (wave + 4 < nblk) load_block(wave + 4, nxt);
    tp(A.ph, 6);
    for (int blk = wave; blk < nblk; blk += 4) {
        if (blk + 8 < nblk) load_block(blk + 8, nx2);
        const int p0 = blk << 5;
        const int v0 = p0 + 8 * gq;
        f32x4_t sa = (f32x4_t){0.f, 0.f, 0.f, 0.f}, sb = sa;
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, cur[0]), Q0, sa, 0, 0, 0);
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, cur[1]), Q1, sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, cur[2]), Q0, sb, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, cur[3]), Q1, sb, 0, 0, 0);
        // this lane: query c, keys v0 + 0..3 (sa) and v0 + 4..7 (sb)
        // online softmax of the block: scores -> probabilities (bf16 pairs in pk), running max / sum.
        // Instantiated twice: blocks inside the committed cache need no mask tests at all.
        uint32_t pk[4];
        float m_new, corr, psum = 0.f;
        auto softmax_block = [&](const unsigned okm) {
            float sc[8];
            float mx = -1e30f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float sv = (j < 4 ? sa[j] : sb[j - 4]) * 0.125f;
                sc[j] = (okm >> j) & 1u ? sv : -1e30f;
                mx = fmaxf(mx, sc[j]);
            }
            mx = rows_max(mx);
            m_new = fmaxf(m_run, mx);
            corr = __expf(m_run - m_new);
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                const float p0f = (okm >> j) & 1u ? __expf(sc[j] - m_new) : 0.f;
                const float p1f = (okm >> (j + 1)) & 1u ? __expf(sc[j + 1] - m_new) : 0.f;
                psum += p0f + p1f;
                pk[j >> 1] = pack_bf16(p0f, p1f);
            }
        };
        if (p0 + 32 > L) {   // the block reaches into the tree rows (same for the whole wave)
            unsigned okm = 0;   // which of the lane's 8 keys the query may see
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int key = v0 + j;
                bool okj = key < L;
                if (!okj && key < T) {
                    const int mm = key - L;
                    if constexpr (CAUSAL) okj = mm <= node;
                    else {
                        const uint32_t mw_ = mm < 32 ? A.mword[0] : mm < 64 ? A.mword[1] : mm < 96 ? A.mword[2] : A.mword[3];   // no indexed access: the words stay in registers
                        okj = (mw_ >> (mm & 31)) & 1u;
                    }
                }
                okm |= okj ? (1u << j) : 0u;
            }
            softmax_block(okm);
        } else {
            softmax_block(0xffu);
        }
        l_run = l_run * corr + psum;
        m_run = m_new;
        const bf16x8_t pfrag = __builtin_bit_cast(bf16x8_t, make_uint4(pk[0], pk[1], pk[2], pk[3]));
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            O[dt] *= corr;
            O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, cur[4 + dt]), pfrag, O[dt], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) { cur[i] = nxt[i]; nxt[i] = nx2[i]; }
    }
    tp(A.ph, 3);
    l_run = rows_sum(l_run);
    // merge the four waves: sm_m / sm_l [wave][query], sm_o [wave][dim][query]
    // (rows of 17 floats: the merge below reads a dimension's 16 queries' worth 64 floats apart, which at 16 floats
    // per row would put a wave's 64 reads into four banks)
    constexpr int SO = 17;
    float* sm_o = (float*)smem;
    float* sm_m = sm_o + 4 * 64 * SO;
    float* sm_l = sm_m + 64;
    __syncthreads();
    tp(A.ph, 7);
    if (gq == 0) { sm_m[wave * 16 + c] = m_run; sm_l[wave * 16 + c] = l_run; }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i) sm_o[(wave * 64 + dt * 16 + 4 * gq + i) * SO + c] = O[dt][i];
    __syncthreads();
    {
        const int q = tid >> 4, d0 = (tid & 15) * 4, nd = qt * 16 + q;
        float mstar = sm_m[q];
#pragma unroll
        for (int w = 1; w < 4; ++w) mstar = fmaxf(mstar, sm_m[w * 16 + q]);
        float f[4], lsum = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) { f[w] = __expf(sm_m[w * 16 + q] - mstar); lsum += f[w] * sm_l[w * 16 + q]; }
        const float inv = 1.f / lsum;
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) a += f[w] * sm_o[(w * 64 + d0 + j) * SO + q];
            o[j] = a * inv;
        }
        if (nd < D.M)
            stw64(att + toff(b * D.M + nd, h * 64 + d0, D.d >> 5),
                  (uint64_t)pack_bf16(o[0], o[1]) | ((uint64_t)pack_bf16(o[2], o[3]) << 32));
    }
}

// Workgroups without a unit in a QKV phase pull the committed part of the key / value cache that the
// coming attention phase will stream into the L2 of the XCD whose attention units read it (Sec. 2.2: the
// committed cache does not depend on the step's rows).  Workgroup i runs on XCD i mod 8 and the attention units of
// (sequence, head) pair p on XCD p mod 8; the idle workgroups of an XCD split that XCD's pairs and each pair's
// blocks among themselves.  Only blocks that lie wholly below the committed length are touched: a block the
// step's rows are written into must not be in any L2 before the barrier (the attention units read it with plain
// loads).  One 4-byte load per 128-byte line; the value is not used.
__device__ __forceinline__ void warm_kv(int ph_, int nu_) {
    const int ph = __builtin_amdgcn_readfirstlane(ph_), nu = __builtin_amdgcn_readfirstlane(nu_);
    const StepParams& P = sP;
    const Dims& D = P.D;
    const DevState& s = P.s;
    const int first = (nu + 7) & ~7;
    const int slot = ((int)blockIdx.x - first) >> 3, nslots = ((int)gridDim.x - first) >> 3;
    if ((int)blockIdx.x < first || (gridDim.x & 7) != 0) return;
    const int per_xcd = pad8(D.B * D.nH) >> 3;
    const int nparts = nslots / per_xcd;
    if (nparts == 0) return;
    const int bh = ((int)blockIdx.x & 7) + 8 * (slot % per_xcd), part = slot / per_xcd;
    if (part >= nparts || bh >= D.B * D.nH) return;
    const int b = bh / D.nH, h = bh - b * D.nH;
    if (b >= ST_SEQ_CACHE || s_seqRows[b] == 0) return;
    const int nfull = __builtin_amdgcn_readfirstlane(min(s_seqL[b], D.maxpos) >> 5);
    const int layer = (ph - 1) / 5;
    const size_t hb = ((((size_t)layer * D.Bmax + b) * D.nH + h) * kv_cap(D.maxpos)) * 64;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;
    // a block is 4 KiB of K and 4 KiB of V^T: lanes 0-31 take the lines of K, lanes 32-63 those of V^T
    const char* base = (const char*)(lane < 32 ? uniform_ptr((const bf16_t*)s.Kc + hb) : uniform_ptr((const bf16_t*)s.Vc + hb)) + (lane & 31) * 128;
    const int stride = nparts * 4;
    uint32_t acc = 0;
    for (int blk = part + nparts * wave; blk < nfull; blk += 4 * stride) {
        const uint32_t v0 = ldg((const uint32_t*)(base + (size_t)blk * 4096));
        const uint32_t v1 = ldg((const uint32_t*)(base + (size_t)min(blk + stride, nfull - 1) * 4096));
        const uint32_t v2 = ldg((const uint32_t*)(base + (size_t)min(blk + 2 * stride, nfull - 1) * 4096));
        const uint32_t v3 = ldg((const uint32_t*)(base + (size_t)min(blk + 3 * stride, nfull - 1) * 4096));
        acc ^= v0 ^ v1 ^ v2 ^ v3;
    }
    keep_alive(acc);
}

// ---------------------------------------------------------------------------
// The units after the decoder layers.  Every kind of unit is a function of its own (not
// inlined into the kernel): each gets its own register allocation, and a change to one does
// not move the code of the others.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void edge_unit(int u_) {
    const int u = __builtin_amdgcn_readfirstlane(u_);
    const StepParams& P = sP;
    const Dims& D = P.D;
    const DevState& s = P.s;
    const int e = u * 4 + (int)(threadIdx.x >> 6);   // one edge per wave: edges 4u .. 4u+3 of the B * M rows
    if (e < D.B * D.M) {
        const int b = e / D.M, n = e - b * D.M;
        const int ok = s.finished[b] ? 0 : dev_edge(D, s, b, n, P.tau);
        if ((threadIdx.x & 63) == 0) stwi(s.edge_ok + e, ok);
    }
}
__device__ __forceinline__ void select_unit(int u_) { const int u = __builtin_amdgcn_readfirstlane(u_); const StepParams& P = sP; dev_select(P.D, P.s, P.seq0 + u, P.ignore_eos); }
__device__ __forceinline__ void final_unit(int u_) {
    const int u = __builtin_amdgcn_readfirstlane(u_);
    const StepParams& P = sP;
    if (P.fuse_select) {
        // Sec. 2.3's choice and the continuation concern one sequence each: one unit does both when a launch runs
        // both (one grid barrier and one phase of a single busy workgroup per sequence less).  The path goes through
        // memory as before (the compaction units read it there): acknowledged before the continuation reads it.
        dev_select(P.D, P.s, P.seq0 + u, P.ignore_eos);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
    dev_finalize<bf16_t>(P.D, P.s, P.seq0 + u, P.prefill_mode, P.ignore_eos, 1);
}
template <bool WIDE>
__device__ __forceinline__ void commit_unit(int u_) {
    const int u = __builtin_amdgcn_readfirstlane(u_);
    const StepParams& P = sP;
    // a unit is four heads of one sequence over commit_layers(P) layers (one in the few-row kernels): one wave (64 head
    // dimensions) per head
    const Dims& D = P.D;
    const int HQ = cdiv(D.nH, 4);
    if constexpr (WIDE) {
        const int LG = commit_layers(P);
        const int head = (u % HQ) * 4 + (int)(threadIdx.x >> 6), b = (u / HQ) % P.nseq, layer0 = u / (HQ * P.nseq) * LG;
        const int nl = D.Ly - layer0 < LG ? D.Ly - layer0 : LG;
        if (head < D.nH) dev_commit_kv_layers<bf16_t>(D, P.s, layer0, nl, P.seq0 + b, head, threadIdx.x & 63);
    } else {
        const int head = (u % HQ) * 4 + (int)(threadIdx.x >> 6), b = (u / HQ) % P.nseq, layer = u / (HQ * P.nseq);
        if (head < D.nH) dev_commit_kv<bf16_t>(D, P.s, layer, P.seq0 + b, head, threadIdx.x & 63);
    }
}
__device__ __forceinline__ void topk_unit(int u_) { const int u = __builtin_amdgcn_readfirstlane(u_); const StepParams& P = sP; dev_topk(P.D, P.s, u / P.D.B, u % P.D.B); }

// ---------------------------------------------------------------------------
// one unit of one phase
// ---------------------------------------------------------------------------
// ---------------------------------------------------------------------------
// one unit of one phase: dispatch to the unit's own function
// ---------------------------------------------------------------------------
template <bool WIDE, bool CAUSAL, bool MID>
__device__ __forceinline__ void run_unit(int ph, int u, const uint32_t* gtab) {
    const StepParams& P = sP;
    const Dims& D = P.D;
    const int H = 1 + 5 * D.Ly;
    // each kind of unit is instantiated once (the kernel's code has to stay small enough for the
    // instruction cache): first decide the kind, then one call site per kind
    enum { K_EMBED, K_ATTN, K_GEMM4, K_GEMM1, K_GEMM22, K_GEMMW, K_EDGE, K_SELECT, K_FINAL, K_COMMIT, K_TOPK };
    int kind;
    if (ph == 0) kind = K_EMBED;
    else if (ph < H) {
        const int k = (ph - 1) % 5;
        kind = k == 1 ? K_ATTN : WIDE ? K_GEMMW : (k == 0 || k == 3) ? (sq_units(P, k == 0 ? 3 * D.d : D.F) ? K_GEMM22 : K_GEMM4) : K_GEMM1;
    } else {
        switch (ph - H) {
        case TP_EDGES: kind = K_EDGE; break;
        case TP_SELECT: kind = K_SELECT; break;
        case TP_FINAL: kind = K_FINAL; break;
        case TP_COMMIT: kind = K_GEMM4; break;
        case TP_TOPK: kind = u < topk_units(P) ? K_TOPK : K_COMMIT; break;
        default: kind = (WIDE && ph == H) ? K_GEMMW : K_GEMM4; break;   // TP_HEAD, TP_DRAFT2
        }
    }
    switch (kind) {
    case K_EMBED: embed_unit<WIDE>(u); break;
    case K_ATTN:
        // (the few-row kernels run their attention units from the kernel's loop: attn_prepare / attn_few)
        if constexpr (WIDE) { if (attn_allq(P)) attn_unit<true, CAUSAL>(ph, u); else attn_unit<false, CAUSAL>(ph, u); }
        break;
    case K_GEMM4: gemm_unit<4>(ph, u, gtab); break;
    case K_GEMM1: if constexpr (!WIDE) { if constexpr (MID) gemm_unit<2>(ph, u, gtab); else gemm_unit<1>(ph, u, gtab); } break;
    case K_GEMM22: if constexpr (!WIDE) { if constexpr (MID) gemm_unit42(ph, u, gtab); else gemm_unit22(ph, u, gtab); } break;
    case K_GEMMW: if constexpr (WIDE) gemm_wide_unit(ph, u); break;
    case K_EDGE: edge_unit(u); break;
    case K_SELECT: select_unit(u); break;
    case K_FINAL: final_unit(u); break;
    case K_COMMIT: commit_unit<WIDE>(u - topk_units(P)); break;
    default: topk_unit(u); break;
    }
}

// Six kernels from one body: the ordinary one (up to 64 rows), the one for 65 to 255 rows (StepParams::mid: QKV and
// FFN1 in 64 x 32 units, the residual maps in 32 x 16 units, so that a 128-row step has one round of units per
// phase) and the one whose layer maps and base head run as 64 x 64 or 128 x 128 units (StepParams::wide), each for
// tree rows and for the causal passes of the prefill; each carries only the unit code it uses.
template <bool WIDE, bool CAUSAL, bool MID>
__global__ __launch_bounds__(256) void k_step(StepParams Parg) {
    {
        const uint32_t* src = (const uint32_t*)&Parg;
        uint32_t* dst = (uint32_t*)&sP;
        for (int i = threadIdx.x; i < (int)(sizeof(StepParams) / 4); i += 256) dst[i] = src[i];
    }
    __syncthreads();
    const StepParams& P = sP;
    uint32_t epoch = P.epoch;
    // unit counts of the five layer phases and of the phases after the layers, once per launch
    __shared__ int s_nu[5 + TP_COUNT];
    const int H = 1 + 5 * P.D.Ly;
    if ((int)threadIdx.x < P.D.B) {   // at most ST_SEQ_CACHE = 256 sequences are cached
        const int b = threadIdx.x;
        s_seqL[b] = ldg(P.s.L + b);
        // tree rows: a finished sequence has none (what the embedding phase is about to store in n_rows)
        s_seqRows[b] = P.prefill_mode ? ldg(P.s.n_rows + b) : (P.s.finished[b] ? 0 : P.D.M);
    }
    if (threadIdx.x < 5 + TP_COUNT) s_nu[threadIdx.x] = phase_units(P, threadIdx.x < 5 ? 1 + (int)threadIdx.x : H + (int)threadIdx.x - 5);
    __syncthreads();
    // the few-row kernel takes the launch-independent part of a layer map's descriptor from the
    // context's table (null: derived per unit)
    const uint32_t* gtab = WIDE ? nullptr : uniform_ptr(P.s.gtab);
    // phases after the layers that have no units (acceptance phases of a prefill pass, the selection phase when the
    // continuation units choose the path) are skipped with their barriers: last_ph = the last phase that runs
    int last_ph = P.ph_hi - 1;
    while (last_ph >= H && last_ph > P.ph_lo && s_nu[5 + last_ph - H] == 0) --last_ph;
    for (int ph = P.ph_lo; ph < P.ph_hi; ++ph) {
        const int nu = ph == 0 ? (WIDE ? cdiv(P.D.B * P.D.M, 4) : P.D.B * P.D.M) : ph < H ? s_nu[(ph - 1) % 5] : s_nu[5 + ph - H];
        if (ph >= H && nu == 0) continue;
        tp(ph, 0);
        const bool few_attn = !WIDE && ph > 0 && ph < H && (ph - 1) % 5 == 1;
        for (int u = blockIdx.x; u < nu; u += gridDim.x) {
            if constexpr (!WIDE) {
                if (few_attn) {
                    AttnPrep ap;
                    attn_prepare<CAUSAL>(ph, u, ap);
                    attn_few<CAUSAL>(ap);
                } else {
                    run_unit<WIDE, CAUSAL, MID>(ph, u, gtab);
                }
            } else {
                run_unit<WIDE, CAUSAL, MID>(ph, u, gtab);
            }
            __syncthreads();
        }
        if constexpr (!WIDE && !CAUSAL) {
            if (ph > 0 && ph < H && (ph - 1) % 5 == 0 && (int)blockIdx.x >= nu && P.persistent) warm_kv(ph, nu);
        }
        tp(ph, 1);
        if (P.persistent && ph < last_ph) {
            ++epoch;
            if (!grid_sync(epoch, ph)) return;
        }
    }
    tp(127, 0);
}

// Writes the descriptor table of a context: one thread runs the per-unit derivation for unit 0 of
// the phases of layers 0 and 1 and stores layer 0's pointers and their advance per layer.
__global__ __launch_bounds__(64) void k_build_gtab(StepParams Parg, uint32_t* tab) {
    {
        const uint32_t* src = (const uint32_t*)&Parg;
        uint32_t* dst = (uint32_t*)&sP;
        for (int i = threadIdx.x; i < (int)(sizeof(StepParams) / 4); i += 64) dst[i] = src[i];
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    for (int k = 0; k < 5; ++k) {
        uint64_t q[16];
        for (int i = 0; i < 16; ++i) q[i] = 0;
        GemmD g0, g1;
        int nt, row0;
        if (describe_gemm<false>(1 + k, 0, g0, nt, row0)) {
            const uint64_t p0[7] = {(uint64_t)g0.X, (uint64_t)g0.Wp, (uint64_t)g0.bias, (uint64_t)g0.colsum,
                                    (uint64_t)g0.stats, (uint64_t)g0.out, (uint64_t)g0.stats_out};
            uint64_t p1[7] = {p0[0], p0[1], p0[2], p0[3], p0[4], p0[5], p0[6]};
            if (sP.D.Ly > 1 && describe_gemm<false>(6 + k, 0, g1, nt, row0)) {
                p1[0] = (uint64_t)g1.X; p1[1] = (uint64_t)g1.Wp; p1[2] = (uint64_t)g1.bias; p1[3] = (uint64_t)g1.colsum;
                p1[4] = (uint64_t)g1.stats; p1[5] = (uint64_t)g1.out; p1[6] = (uint64_t)g1.stats_out;
            }
            for (int i = 0; i < 7; ++i) { q[2 * i] = p0[i]; q[2 * i + 1] = p0[i] ? p1[i] - p0[i] : 0; }
            q[14] = (uint64_t)(uint32_t)g0.K | ((uint64_t)(uint32_t)g0.N << 32);
            q[15] = (uint64_t)(uint32_t)g0.epi;
        }
        for (int i = 0; i < 16; ++i) {
            tab[k * VADUSA_GREC_WORDS + 2 * i] = (uint32_t)q[i];
            tab[k * VADUSA_GREC_WORDS + 2 * i + 1] = (uint32_t)(q[i] >> 32);
        }
    }
}
void launch_build_gtab(const StepParams& p, uint32_t* tab, hipStream_t st) {
    StepParams q = p;
    q.s.gtab = nullptr;   // the derivation itself, not a table
    q.wide = 0;
    hipLaunchKernelGGL(k_build_gtab, dim3(1), dim3(64), 0, st, q, tab);
}

void launch_step(const StepParams& p, int n_cus, hipStream_t st, hipError_t* err) {
    static bool once = false;
    if (!once) {
        (void)hipFuncSetAttribute((const void*)k_step<true, false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, ST_WIDE_LDS_BYTES);
        (void)hipFuncSetAttribute((const void*)k_step<true, true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, ST_WIDE_LDS_BYTES);
        (void)hipFuncSetAttribute((const void*)k_step<false, false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, ST_LDS_BYTES);
        (void)hipFuncSetAttribute((const void*)k_step<false, true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, ST_LDS_BYTES);
        (void)hipFuncSetAttribute((const void*)k_step<false, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, ST_MID_LDS_BYTES);
        (void)hipFuncSetAttribute((const void*)k_step<false, true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, ST_MID_LDS_BYTES);
        once = true;
    }
    *err = hipSuccess;
    const size_t lds = p.wide ? ST_WIDE_LDS_BYTES : p.mid ? ST_MID_LDS_BYTES : ST_LDS_BYTES;
    // six kernels from one body: up to 64 rows, 65 to 255 rows, 256 rows and more; tree (table 0) or causal pass of the prefill (table 1)
    void (*kfn)(StepParams) = p.wide ? (p.table == 1 ? k_step<true, true, false> : k_step<true, false, false>)
                              : p.mid ? (p.table == 1 ? k_step<false, true, true> : k_step<false, false, true>)
                                      : (p.table == 1 ? k_step<false, true, false> : k_step<false, false, false>);
    if (p.persistent) {
        // every workgroup of the grid must fit on the GPU at once
        static int resident = -1;
        if (resident < 0) {
            int nb = 0, nm = 0, nw = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k_step<false, false, false>, 256, ST_LDS_BYTES) != hipSuccess) nb = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nm, k_step<false, true, true>, 256, ST_MID_LDS_BYTES) != hipSuccess) nm = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nw, k_step<true, true, false>, 256, ST_WIDE_LDS_BYTES) != hipSuccess) nw = 0;
            nb = std::min(nb, std::min(nm, nw));
            resident = nb;
        }
        if (resident < 1) { *err = hipErrorCooperativeLaunchTooLarge; return; }
    }
    if (p.persistent) {
        StepParams q = p;
        void* args[] = {&q};
        // The grid barrier needs every workgroup resident.  The grid is one workgroup per compute
        // unit and the kernel's register use allows no second one, so an ordinary launch on an
        // otherwise idle GPU places them all; it costs ~18 us less per step than a cooperative
        // launch.  Should the GPU be shared and a workgroup not get its compute unit, the bounded
        // barrier reports a time-out (VADUSA_EHIP) instead of hanging.  VADUSA_COOPERATIVE_LAUNCH=1
        // selects the cooperative launch, which makes the runtime check residency.
        static const bool coop = getenv("VADUSA_COOPERATIVE_LAUNCH") != nullptr;
        if (!coop) {
            hipLaunchKernelGGL(kfn, dim3(n_cus), dim3(256), lds, st, q);
            *err = hipGetLastError();
        } else {
            *err = hipLaunchCooperativeKernel((const void*)kfn, dim3(n_cus), dim3(256), args, lds, st);
        }
        return;
    }
    for (int ph = p.ph_lo; ph < p.ph_hi; ++ph) {
        StepParams q = p;
        q.ph_lo = ph; q.ph_hi = ph + 1;
        const int nu = phase_units(q, ph);
        if (nu <= 0) continue;
        hipLaunchKernelGGL(kfn, dim3(std::min(nu, 4096)), dim3(256), lds, st, q);
    }
    *err = hipGetLastError();
}

// ---------------------------------------------------------------------------
// weight preparation: fp32 [N][K] row-major -> packed bf16 tiles
// [n-tile][k-step][lane][8]; lane (c, g) of tile (nt, ks) holds
// W[nt*16 + c][ks*32 + 8g .. 8g+7] (times gamma[k] for LN-folded maps).
// Rows >= N are zero.
// ---------------------------------------------------------------------------
__global__ void k_pack_w(const float* __restrict__ src, const float* __restrict__ gamma, uint4* __restrict__ dst,
                         int N, int K) {
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
            if (n < N) {
                lo = src[(size_t)n * K + k0 + 2 * j];
                hi = src[(size_t)n * K + k0 + 2 * j + 1];
                if (gamma) { lo *= gamma[k0 + 2 * j]; hi *= gamma[k0 + 2 * j + 1]; }
            }
            w[j] = (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
        }
        dst[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// colsum[n] = sum_k bf16(gamma[k] W[n][k]),  tvec[n] = sum_k beta[k] W[n][k]; one wave per n
__global__ void k_fold_vectors(const float* __restrict__ src, const float* __restrict__ gamma,
                               const float* __restrict__ beta, float* __restrict__ colsum, float* __restrict__ tvec,
                               int N, int K) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (n >= N) return;
    float cs = 0.f, tv = 0.f;
    for (int k = lane; k < K; k += 64) {
        const float w = src[(size_t)n * K + k];
        cs += bf2f(f2bf(w * gamma[k]));
        tv += beta[k] * w;
    }
    cs = wave_sum(cs);
    tv = wave_sum(tv);
    if (lane == 0) { colsum[n] = cs; tvec[n] = tv; }
}

__global__ void k_add_vec(float* __restrict__ dst, const float* __restrict__ src, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] += src[i];
}

void launch_pack_w(const float* src, void* dst, int N, int K, hipStream_t st) {
    const size_t total = (size_t)((N + 15) / 16) * (K >> 5) * 64;
    const int blocks = (int)std::min<size_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(k_pack_w, dim3(blocks), dim3(256), 0, st, src, (const float*)nullptr, (uint4*)dst, N, K);
}

void launch_pack_w_ln(const float* src, const float* gamma, const float* beta, void* dst, float* colsum,
                      float* tvec, int N, int K, hipStream_t st) {
    const size_t total = (size_t)((N + 15) / 16) * (K >> 5) * 64;
    const int blocks = (int)std::min<size_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(k_pack_w, dim3(blocks), dim3(256), 0, st, src, gamma, (uint4*)dst, N, K);
    hipLaunchKernelGGL(k_fold_vectors, dim3((N + 3) / 4), dim3(256), 0, st, src, gamma, beta, colsum, tvec, N, K);
}

void launch_add_vec(float* dst, const float* src, int n, hipStream_t st) {
    hipLaunchKernelGGL(k_add_vec, dim3((n + 255) / 256), dim3(256), 0, st, dst, src, n);
}
