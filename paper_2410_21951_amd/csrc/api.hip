// C ABI of libvadusa: argument checks, arena layout, weight loading and the
// order in which the kernels of a prefill / verification / compaction run.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "common.h"

// ---------------------------------------------------------------------------
// small host helpers
// ---------------------------------------------------------------------------
static void set_msg(char* msg, size_t n, const char* fmt, ...) {
    if (!msg || !n) return;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(msg, n, fmt, ap);
    va_end(ap);
}

static int fail(vadusa_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    return code;
}

#define HIP_TRY(c, call)                                                                   \
    do {                                                                                   \
        hipError_t e_ = (call);                                                            \
        if (e_ != hipSuccess)                                                              \
            return fail((c), VADUSA_EHIP, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
// rows of one sequence in one pass of the prefill, and the most rows one sequence ever has in a forward
static int prefill_rows(const vadusa_config& c) { return c.prefill_chunk > 0 ? c.prefill_chunk : c.max_tree_nodes; }
static int seq_rows_cap(const vadusa_config& c) { return std::max(c.max_tree_nodes, prefill_rows(c)); }
static int pad16(int n) { return (n + 15) / 16 * 16; }

extern "C" int vadusa_config_check(const vadusa_config* c, char* msg, size_t n) {
    if (!c) { set_msg(msg, n, "config is null"); return VADUSA_EINVAL; }
#define BAD(code, ...) do { set_msg(msg, n, __VA_ARGS__); return code; } while (0)
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_ffn < 1 || c->speech_vocab < 1 ||
        c->text_vocab < 1 || c->max_positions < 2 || c->max_batch < 1 || c->max_tree_nodes < 1)
        BAD(VADUSA_EINVAL, "sizes must be positive");
    if (c->prefill_chunk < 0) BAD(VADUSA_EINVAL, "prefill_chunk must be >= 0");
    if (c->prefill_chunk > VADUSA_MAX_PREFILL_CHUNK) BAD(VADUSA_ESHAPE, "prefill_chunk must be <= %d", VADUSA_MAX_PREFILL_CHUNK);
    if (c->dtype != 0 && c->dtype != 1) BAD(VADUSA_EINVAL, "dtype must be 0 (fp32) or 1 (bf16)");
    if (c->ignore_eos != 0 && c->ignore_eos != 1) BAD(VADUSA_EINVAL, "ignore_eos must be 0 or 1");
    if (c->head_dim != 64) BAD(VADUSA_ESHAPE, "head_dim must be 64 (got %d)", c->head_dim);
    if (c->d_model != c->n_heads * c->head_dim) BAD(VADUSA_ESHAPE, "d_model must equal n_heads * head_dim");
    if (c->d_ffn % 64) BAD(VADUSA_ESHAPE, "d_ffn must be a multiple of 64");
    if (c->n_draft_heads < 1 || c->n_draft_heads > VADUSA_MAX_DRAFT_HEADS)
        BAD(VADUSA_ESHAPE, "n_draft_heads must be 1..%d", VADUSA_MAX_DRAFT_HEADS);
    if (c->max_tree_nodes > VADUSA_MAX_TREE_NODES)
        BAD(VADUSA_ESHAPE, "max_tree_nodes must be <= %d", VADUSA_MAX_TREE_NODES);
    if (c->max_positions <= c->max_tree_nodes)
        BAD(VADUSA_ESHAPE, "max_positions must exceed max_tree_nodes");
    if (c->max_positions % 8) BAD(VADUSA_ESHAPE, "max_positions must be a multiple of 8");
    if (c->d_model % 64) BAD(VADUSA_ESHAPE, "d_model must be a multiple of 64");
    if ((int64_t)c->max_batch * std::max(c->max_tree_nodes, c->prefill_chunk) > (1 << 20))
        BAD(VADUSA_ESHAPE, "max_batch * max(max_tree_nodes, prefill_chunk) too large");
#undef BAD
    return VADUSA_OK;
}

// Depth of every node, or an error.  Checks the ordering rules of vadusa.h.
static int tree_depths(const vadusa_config* c, const vadusa_tree_spec* t, std::vector<int32_t>* depth,
                       char* msg, size_t n) {
#define BAD(...) do { set_msg(msg, n, __VA_ARGS__); return VADUSA_EINVAL; } while (0)
    if (!t || !t->parent || !t->rank) BAD("tree or its arrays are null");
    const int M = t->n_nodes;
    if (M < 1 || M > c->max_tree_nodes) BAD("n_nodes %d outside 1..max_tree_nodes (%d)", M, c->max_tree_nodes);
    if (t->parent[0] != -1) BAD("parent[0] must be -1");
    depth->assign(M, 0);
    std::vector<std::vector<int32_t>> path(M);
    for (int i = 1; i < M; ++i) {
        const int p = t->parent[i];
        if (p < 0 || p >= i) BAD("parent[%d] = %d must be in [0, %d)", i, p, i);
        (*depth)[i] = (*depth)[p] + 1;
        if ((*depth)[i] > c->n_draft_heads) BAD("node %d is deeper than the number of draft heads", i);
        if (t->rank[i] < 0 || t->rank[i] >= VADUSA_MAX_TOPK) BAD("rank[%d] = %d outside [0, %d)", i, t->rank[i], VADUSA_MAX_TOPK);
        path[i] = path[p];
        path[i].push_back(t->rank[i]);
        // canonical order: (depth, rank path) strictly increasing; also rules out equal siblings
        const bool deeper = (*depth)[i] > (*depth)[i - 1];
        if (!deeper && !((*depth)[i] == (*depth)[i - 1] && path[i - 1] < path[i]))
            BAD("node %d breaks the canonical (depth, rank path) order", i);
    }
#undef BAD
    return VADUSA_OK;
}

// Sec. 2.4's greedy construction: best-first expansion of the full top-k tree by path
// probability.  A child's probability never exceeds its parent's, so the set taken is
// ancestor-closed, and taking the largest probabilities maximises their sum, the expected
// number of accepted draft tokens.
extern "C" int vadusa_build_tree(int32_t n_heads, int32_t width, const float* acc, int32_t n_nodes,
                                 int32_t* parent, int32_t* rank, int32_t* n_out) {
    if (!acc || !parent || !rank || !n_out) return VADUSA_EINVAL;
    if (n_heads < 1 || n_heads > VADUSA_MAX_DRAFT_HEADS || width < 1 || width > VADUSA_MAX_TOPK ||
        n_nodes < 1 || n_nodes > VADUSA_MAX_TREE_NODES)
        return VADUSA_EINVAL;
    for (int i = 0; i < n_heads * width; ++i)
        if (!(acc[i] >= 0.f && acc[i] <= 1.f)) return VADUSA_EINVAL;
    struct Cand { double p; std::vector<int32_t> path; };
    // "a goes before b": larger probability, then shallower, then smaller rank path
    auto before = [](const Cand& a, const Cand& b) {
        if (a.p != b.p) return a.p > b.p;
        if (a.path.size() != b.path.size()) return a.path.size() < b.path.size();
        return a.path < b.path;
    };
    std::vector<Cand> open{Cand{1.0, {}}}, chosen;
    while (!open.empty() && (int)chosen.size() < n_nodes) {
        size_t best = 0;
        for (size_t i = 1; i < open.size(); ++i)
            if (before(open[i], open[best])) best = i;
        Cand c = open[best];
        open.erase(open.begin() + (long)best);
        if ((int)c.path.size() < n_heads)
            for (int r = 0; r < width; ++r) {
                Cand ch{c.p * (double)acc[c.path.size() * (size_t)width + r], c.path};
                ch.path.push_back(r);
                open.push_back(ch);
            }
        chosen.push_back(c);
    }
    // canonical order: depth, then rank path
    std::sort(chosen.begin(), chosen.end(), [](const Cand& a, const Cand& b) {
        if (a.path.size() != b.path.size()) return a.path.size() < b.path.size();
        return a.path < b.path;
    });
    for (size_t i = 0; i < chosen.size(); ++i) {
        const auto& p = chosen[i].path;
        rank[i] = p.empty() ? 0 : p.back();
        parent[i] = -1;
        if (!p.empty()) {
            const std::vector<int32_t> pp(p.begin(), p.end() - 1);
            for (size_t j = 0; j < i; ++j)
                if (chosen[j].path == pp) { parent[i] = (int32_t)j; break; }
        }
    }
    *n_out = (int32_t)chosen.size();
    return VADUSA_OK;
}

extern "C" int vadusa_tree_check(const vadusa_config* c, const vadusa_tree_spec* t, char* msg, size_t n) {
    int rc = vadusa_config_check(c, msg, n);
    if (rc) return rc;
    std::vector<int32_t> depth;
    return tree_depths(c, t, &depth, msg, n);
}

// ---------------------------------------------------------------------------
// Arena layout.  With base == nullptr only the total size is computed.
// ---------------------------------------------------------------------------
struct Carver {
    char* base;
    size_t off = 0;
    void* take(size_t bytes) {
        off = align_up(off, 256);
        void* p = base ? base + off : nullptr;
        off += bytes;
        return p;
    }
};

// blob order; kind 0 vector, 1 table, 2 linear map.  For LayerNorm-folded maps of the bf16 model:
// gamma/beta of the LayerNorm in front, the map's own bias (or null) and where colsum / t go.
struct WeightSlot {
    void* dev; size_t rows, cols; int kind;
    const float *gamma, *beta, *bias; float *colsum, *tvec;
};

static size_t layout(const vadusa_config& c, char* base, DevState* s, std::vector<LayerW>* layers,
                     std::vector<DraftW>* draft, std::vector<WeightSlot>* slots, size_t* staging_floats,
                     float** uniforms = nullptr, float** scores = nullptr) {
    Carver cv{base};
    const size_t e = c.dtype ? 2 : 4;
    const size_t d = c.d_model, F = c.d_ffn, V1 = c.speech_vocab + 1, Hh = c.n_draft_heads;
    const size_t R = (size_t)c.max_batch * seq_rows_cap(c), B = c.max_batch, P = c.max_positions;
    DevState st{};
    std::vector<LayerW> lw(c.n_layers);
    std::vector<DraftW> dw(Hh);
    std::vector<WeightSlot> sl;
    size_t biggest = std::max(R * std::max(d, V1), P * d);
    auto mat = [&](const void** dst, size_t rows, size_t cols, int kind = 2) {
        *dst = cv.take((size_t)pad16((int)rows) * cols * e);
        sl.push_back({(void*)*dst, rows, cols, kind, nullptr, nullptr, nullptr, nullptr, nullptr});
        biggest = std::max(biggest, rows * cols);
    };
    auto vec = [&](const float** dst, size_t n) {
        *dst = (const float*)cv.take(n * 4);
        sl.push_back({(void*)*dst, 1, n, 0, nullptr, nullptr, nullptr, nullptr, nullptr});
    };
    mat(&st.E_text, c.text_vocab, d, 1);
    mat(&st.E_speech, V1, d, 1);
    mat(&st.P, P, d, 1);
    auto fold = [&](const float* g, const float* b, float** cs, float** t, size_t n) {
        // call right after mat(): remembers the LayerNorm to fold into that map
        *cs = (float*)cv.take((size_t)pad16((int)n) * 4);   // read as whole 16-column tiles
        *t = (float*)cv.take((size_t)pad16((int)n) * 4);
        WeightSlot& w = sl.back();
        w.gamma = g; w.beta = b; w.colsum = *cs; w.tvec = *t;
    };
    for (int l = 0; l < c.n_layers; ++l) {
        LayerW& w = lw[l];
        vec(&w.ln1_g, d); vec(&w.ln1_b, d);
        mat(&w.Wqkv, 3 * d, d);
        if (c.dtype) fold(w.ln1_g, w.ln1_b, &w.cs_qkv, &w.t_qkv, 3 * d);
        const size_t iq = sl.size() - 1;
        vec(&w.bqkv, 3 * d);
        sl[iq].bias = w.bqkv;
        mat(&w.Wo, d, d); vec(&w.bo, d);
        vec(&w.ln2_g, d); vec(&w.ln2_b, d);
        mat(&w.W1, F, d);
        if (c.dtype) fold(w.ln2_g, w.ln2_b, &w.cs_w1, &w.t_w1, F);
        const size_t i1 = sl.size() - 1;
        vec(&w.b1, F);
        sl[i1].bias = w.b1;
        mat(&w.W2, d, F); vec(&w.b2, d);
    }
    vec(&st.lnf_g, d); vec(&st.lnf_b, d);
    mat(&st.W_out, V1, d);
    if (c.dtype) fold(st.lnf_g, st.lnf_b, &st.cs_out, &st.t_out, V1);
    for (size_t i = 0; i < Hh; ++i) {
        mat(&dw[i].W1, d, d); vec(&dw[i].b1, d); mat(&dw[i].W2, V1, d);
    }
    const size_t kv = (size_t)c.n_layers * B * c.n_heads * kv_cap((int)P) * 64 * e;
    st.Kc = cv.take(kv);
    st.Vc = cv.take(kv);
    st.x = (float*)cv.take(R * d * 4);
    const size_t nslots = c.dtype ? 2 * (size_t)c.n_layers + 1 : 0, per_layer = c.dtype ? c.n_layers : 1;
    const size_t Rp = (R + 15) / 16 * 16, Bp = (B + 15) / 16 * 16;   // tiled activation buffers hold whole row tiles
    st.act_stride = Rp * d; st.stats_stride = (d / 16) * R * 2; st.hid_stride = Rp * F; st.draft_stride = Bp * d;
    st.xb = (bf16_t*)cv.take(nslots * Rp * d * 2);
    st.stats = (float*)cv.take(nslots * st.stats_stride * 4);
    st.bar = (uint32_t*)cv.take((size_t)VADUSA_BAR_WORDS * 4);
    st.tprof = (long long*)cv.take(1024 * 8);
    st.gtab = (const uint32_t*)cv.take((size_t)5 * VADUSA_GREC_WORDS * 4);
    st.layers_dev = (const LayerW*)cv.take(sizeof(LayerW) * c.n_layers);
    st.draft_dev = (const DraftW*)cv.take(sizeof(DraftW) * Hh);
    st.xn = cv.take(R * d * e);
    st.q = cv.take(per_layer * Rp * d * e);
    st.att = cv.take(per_layer * Rp * d * e);
    st.hid = cv.take(per_layer * Rp * F * e);
    st.hn = cv.take(R * d * e);
    st.logits = (float*)cv.take(R * V1 * 4);
    st.hbest = cv.take(Bp * d * e);
    st.rdraft = cv.take(Hh * Bp * d * e);
    st.zdraft = (float*)cv.take(Hh * B * V1 * 4);
    auto ints = [&](size_t n) { return (int32_t*)cv.take(n * 4); };
    // What a step hands back to the host sits in one block, so that one copy fetches it: the error word (4 words),
    // accepted lengths, committed lengths, accepted tokens (result_block_words)
    int32_t* res = ints(4 + 2 * B + B * (VADUSA_MAX_DRAFT_HEADS + 1));
    st.kerr = res; st.acc_len = res + 4; st.L = res + 4 + B; st.acc_tok = res + 4 + 2 * B;
    st.root = ints(B); st.finished = ints(B);
    st.draft_topk = ints(B * Hh * VADUSA_MAX_TOPK);
    st.tok = ints(R); st.n_rows = ints(B); st.edge_ok = ints(R);
    st.path = ints(B * (VADUSA_MAX_DRAFT_HEADS + 2));
    st.out_tok = ints(B * P); st.n_out = ints(B);
    st.chunk_tok = ints(R);
    st.override_topk = ints(B * Hh * VADUSA_MAX_TOPK);
    for (int t = 0; t < 2; ++t) {
        st.t_parent[t] = ints(VADUSA_MAX_TREE_NODES);
        st.t_depth[t] = ints(VADUSA_MAX_TREE_NODES);
        st.t_rank[t] = ints(VADUSA_MAX_TREE_NODES);
        st.t_mask[t] = (uint32_t*)cv.take(VADUSA_MAX_TREE_NODES * MASK_WORDS * 4);
    }
    st.staging = (float*)cv.take(biggest * 4);
    float* un = (float*)cv.take(R * V1 * 4);
    float* sc = (float*)cv.take(R * V1 * 4);
    if (uniforms) *uniforms = un;
    if (scores) *scores = sc;
    if (s) *s = st;
    if (layers) *layers = lw;
    if (draft) *draft = dw;
    if (slots) *slots = sl;
    if (staging_floats) *staging_floats = biggest;
    return align_up(cv.off, 256);
}

extern "C" size_t vadusa_arena_bytes(const vadusa_config* c) {
    if (vadusa_config_check(c, nullptr, 0)) return 0;
    return layout(*c, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
}

extern "C" size_t vadusa_blob_floats(const vadusa_config* c) {
    if (vadusa_config_check(c, nullptr, 0)) return 0;
    std::vector<WeightSlot> sl;
    layout(*c, nullptr, nullptr, nullptr, nullptr, &sl, nullptr);
    size_t n = 0;
    for (auto& w : sl) n += w.rows * w.cols;
    return n;
}

// ---------------------------------------------------------------------------
// life cycle
// ---------------------------------------------------------------------------
static Dims make_dims(const vadusa_ctx* c, int B, int M) {
    Dims D;
    D.Ly = c->cfg.n_layers; D.d = c->cfg.d_model; D.nH = c->cfg.n_heads; D.F = c->cfg.d_ffn;
    D.V1 = c->cfg.speech_vocab + 1; D.Hh = c->cfg.n_draft_heads; D.maxpos = c->cfg.max_positions;
    D.Bmax = c->cfg.max_batch; D.Mmax = c->cfg.max_tree_nodes; D.B = B; D.M = M;
    return D;
}

// The launch-independent part of the step kernel's parameters.
static StepParams base_params(const vadusa_ctx* c, const Dims& D) {
    StepParams P{};
    P.D = D; P.s = c->s; P.big_min = c->big_min; P.allq_min = c->allq_min;
    P.lw0 = c->layers[0]; P.dw0 = c->draft[0];
    P.lw_stride = c->layers.size() > 1 ? (size_t)((const char*)c->layers[1].Wqkv - (const char*)c->layers[0].Wqkv) : 0;
    P.dw_stride = c->draft.size() > 1 ? (size_t)((const char*)c->draft[1].W1 - (const char*)c->draft[0].W1) : 0;
    return P;
}


extern "C" int vadusa_create(const vadusa_config* cfg, void* arena, size_t arena_bytes, void* hip_stream,
                             vadusa_ctx** out) {
    if (!out) return VADUSA_EINVAL;
    *out = nullptr;
    char msg[256];
    int rc = vadusa_config_check(cfg, msg, sizeof msg);
    if (rc) return rc;
    const size_t need = vadusa_arena_bytes(cfg);
    if (!arena || arena_bytes < need || ((uintptr_t)arena & 255)) return VADUSA_EINVAL;
    vadusa_ctx* c = new (std::nothrow) vadusa_ctx();
    if (!c) return VADUSA_EINVAL;
    c->cfg = *cfg;
    c->stream = (hipStream_t)hip_stream;
    c->arena = (char*)arena;
    c->arena_bytes = arena_bytes;
    c->elem = cfg->dtype ? 2 : 4;
    c->state = 0;
    c->batch = 0;
    c->M = 0;
    layout(*cfg, c->arena, &c->s, &c->layers, &c->draft, nullptr, &c->staging_floats, &c->uniforms, &c->scores);
    c->sampled = 0;
    if (cfg->dtype) {
        // the step kernel addresses layer l as layer 0 + l * stride: the layout must be that regular
        auto off = [](const void* a, const void* b) { return (const char*)a - (const char*)b; };
        bool ok = true;
        for (size_t l = 1; l < c->layers.size() && ok; ++l) {
            const LayerW &a = c->layers[0], &b = c->layers[l];
            const ptrdiff_t st = off(c->layers[1].Wqkv, a.Wqkv) * (ptrdiff_t)l;
            ok = off(b.Wqkv, a.Wqkv) == st && off(b.Wo, a.Wo) == st && off(b.W1, a.W1) == st && off(b.W2, a.W2) == st &&
                 off(b.bo, a.bo) == st && off(b.b2, a.b2) == st && off(b.t_qkv, a.t_qkv) == st &&
                 off(b.cs_qkv, a.cs_qkv) == st && off(b.t_w1, a.t_w1) == st && off(b.cs_w1, a.cs_w1) == st;
        }
        for (size_t i = 1; i < c->draft.size() && ok; ++i) {
            const DraftW &a = c->draft[0], &b = c->draft[i];
            const ptrdiff_t st = off(c->draft[1].W1, a.W1) * (ptrdiff_t)i;
            ok = off(b.W1, a.W1) == st && off(b.b1, a.b1) == st && off(b.W2, a.W2) == st;
        }
        if (!ok) { delete c; return VADUSA_ESHAPE; }
    }
    c->L_ub.assign(cfg->max_batch, 0);
    c->pending.assign(cfg->max_batch, 0);
    c->epoch = 0;
    c->errored = 0;
    c->persistent = getenv("VADUSA_PHASE_LAUNCHES") ? 0 : 1;
    c->profile = getenv("VADUSA_PHASE_CLOCK") ? std::max(1, atoi(getenv("VADUSA_PHASE_CLOCK"))) : 0;   // n: workgroup n - 1 records
    // 128 x 128 units from 129 of them on (more than half of the 256 compute units busy for one round: with fewer, the
    // four times as many 64 x 64 units take two rounds of less than half the time each); whole-head attention units
    // once there is one per compute unit
    c->big_min = getenv("VADUSA_BIG_MIN_UNITS") ? std::max(1, atoi(getenv("VADUSA_BIG_MIN_UNITS"))) : 129;
    c->allq_min = getenv("VADUSA_BIG_MIN_UNITS") ? c->big_min : 256;
    {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) { delete c; return VADUSA_EHIP; }
        c->n_cus = std::min(prop.multiProcessorCount, 1024);
        // barrier flags and the error flag start at zero; an unwritten KV row must never hold NaN bits
        const size_t kv = (size_t)cfg->n_layers * cfg->max_batch * cfg->n_heads * cfg->max_positions * 64 * c->elem;
        hipError_t e0 = hipMemset(c->s.bar, 0, (size_t)VADUSA_BAR_WORDS * 4);
        if (e0 == hipSuccess) e0 = hipMemset(c->s.tprof, 0, 1024 * 8);
        if (e0 == hipSuccess) e0 = hipMemset(c->s.kerr, 0, 16);
        if (e0 == hipSuccess) e0 = hipMemset(c->s.Kc, 0, kv);
        if (e0 == hipSuccess) e0 = hipMemset(c->s.Vc, 0, kv);
        if (e0 != hipSuccess) { delete c; return VADUSA_EHIP; }
    }
    // causal table for prefill chunks: row n sees rows 0..n; positions are consecutive
    const int Mm = VADUSA_MAX_TREE_NODES;
    std::vector<int32_t> par(Mm), dep(Mm), rk(Mm, 0);
    std::vector<uint32_t> mask((size_t)Mm * MASK_WORDS, 0);
    for (int n = 0; n < Mm; ++n) {
        par[n] = n - 1; dep[n] = n;
        for (int m = 0; m <= n; ++m) mask[(size_t)n * MASK_WORDS + (m >> 5)] |= 1u << (m & 31);
    }
    hipError_t e = hipMemcpy(c->s.t_parent[1], par.data(), Mm * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->s.t_depth[1], dep.data(), Mm * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->s.t_rank[1], rk.data(), Mm * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->s.t_mask[1], mask.data(), mask.size() * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) { delete c; return VADUSA_EHIP; }
    *out = c;
    return VADUSA_OK;
}

// Frees host memory only and makes no HIP call: it may run while the process is shutting down (a binding's
// finaliser, an exit handler), when the HIP runtime or a profiler's library has already been torn down; a stream
// synchronisation at that point ended one profiled run with a segmentation fault inside the exit handlers.
// The caller drains its stream before it frees the arena.
extern "C" void vadusa_destroy(vadusa_ctx* c) {
    if (!c) return;
    delete c;
}

// Test aid: raises the error word as a kernel that gave up at a grid barrier would (the next synchronising call
// reports VADUSA_EHIP and the context refuses work until vadusa_prefill has reset it).
extern "C" int vadusa_debug_raise_error(vadusa_ctx* c) {
    if (!c) return VADUSA_EINVAL;
    if (!c->cfg.dtype) return fail(c, VADUSA_ESTATE, "the fp32 path has no persistent kernel and no error word");
    const int32_t one = 1;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(c->s.kerr, &one, 4, hipMemcpyHostToDevice));
    return VADUSA_OK;
}

extern "C" const char* vadusa_last_error(const vadusa_ctx* c) { return c ? c->err.c_str() : "null context"; }

extern "C" int vadusa_load_weights(vadusa_ctx* c, const float* blob, size_t n_floats, int on_device) {
    if (!c) return VADUSA_EINVAL;
    if (!blob) return fail(c, VADUSA_EINVAL, "blob is null");
    if (n_floats != vadusa_blob_floats(&c->cfg))
        return fail(c, VADUSA_EINVAL, "blob has %zu floats, expected %zu", n_floats, vadusa_blob_floats(&c->cfg));
    std::vector<WeightSlot> sl;
    layout(c->cfg, c->arena, nullptr, nullptr, nullptr, &sl, nullptr);
    size_t off = 0;
    for (auto& w : sl) {
        const size_t n = w.rows * w.cols;
        void* dst = w.dev;
        const float* src = blob + off;
        const bool is_matrix = w.kind != 0;
        if (!on_device) {
            if (is_matrix) {
                HIP_TRY(c, hipMemcpyAsync(c->s.staging, src, n * 4, hipMemcpyHostToDevice, c->stream));
                src = c->s.staging;
            } else {
                HIP_TRY(c, hipMemcpyAsync(dst, src, n * 4, hipMemcpyHostToDevice, c->stream));
            }
        } else if (!is_matrix) {
            HIP_TRY(c, hipMemcpyAsync(dst, src, n * 4, hipMemcpyDeviceToDevice, c->stream));
        }
        if (is_matrix) {
            if (w.kind == 2 && c->cfg.dtype) {
                // linear maps of the bf16 model are stored in the MFMA-tiled layout, with the
                // LayerNorm in front of them (if any) folded in
                if (w.gamma) launch_pack_w_ln(src, w.gamma, w.beta, dst, w.colsum, w.tvec, (int)w.rows, (int)w.cols, c->stream);
                else launch_pack_w(src, dst, (int)w.rows, (int)w.cols, c->stream);
            } else {
                const size_t padded = (size_t)pad16((int)w.rows) * w.cols;
                if (padded > n)
                    HIP_TRY(c, hipMemsetAsync((char*)dst + n * c->elem, 0, (padded - n) * c->elem, c->stream));
                launch_convert(src, dst, n, c->cfg.dtype, c->stream);
            }
        }
        off += n;
    }
    if (c->cfg.dtype) {
        for (auto& w : sl)   // t = beta W^T + bias, once every bias has arrived
            if (w.gamma && w.bias) launch_add_vec(w.tvec, w.bias, (int)w.rows, c->stream);
        HIP_TRY(c, hipMemcpyAsync((void*)c->s.layers_dev, c->layers.data(), sizeof(LayerW) * c->layers.size(),
                                  hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync((void*)c->s.draft_dev, c->draft.data(), sizeof(DraftW) * c->draft.size(),
                                  hipMemcpyHostToDevice, c->stream));
    }
    if (c->cfg.dtype) {
        const StepParams P = base_params(c, make_dims(c, 1, 1));
        launch_build_gtab(P, (uint32_t*)c->s.gtab, c->stream);
    }
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipGetLastError());
    c->gtab_ready = c->cfg.dtype != 0;
    c->state = 1;
    return VADUSA_OK;
}

// ---------------------------------------------------------------------------
// forward of B x M rows through the decoder (Sec. 2.1 tree attention; the
// prefill uses the same path with a causal chunk as the "tree")
// ---------------------------------------------------------------------------
static void gemm(vadusa_ctx* c, const GemmArgs& a) { launch_gemm_simple(a, 0, c->stream); }

// bf16 model: run phases [lo, hi) of the step kernel (see k_step.hip)
static int run_phases(vadusa_ctx* c, const Dims& D, int table, int prefill_mode, int tau, int lo, int hi,
                      int seq0, int nseq, float* rank_rows = nullptr) {
    // Rows of more than 4096 logits: the draft lists come from the stand-alone top-k kernel (it
    // handles such rows slice by slice; the step kernel's own top-k phase would re-scan the row
    // once per list entry)
    const bool topk_apart = D.V1 > 4096 && hi == 1 + 5 * D.Ly + TP_COUNT;
    StepParams P = base_params(c, D);
    if (rank_rows) P.s.logits = rank_rows;   // acceptance and continuation rank these rows instead of the logits
    P.table = table; P.prefill_mode = prefill_mode; P.tau = tau;
    P.ignore_eos = c->cfg.ignore_eos; P.ph_lo = lo; P.ph_hi = hi; P.persistent = c->persistent; P.profile = c->profile; P.wide = D.B * D.M >= 256; P.mid = !P.wide && D.B * D.M > 64;
    P.epoch = c->epoch; P.seq0 = seq0; P.nseq = nseq; P.topk_apart = topk_apart;
    {
        const int Hp = 1 + 5 * D.Ly;
        P.fuse_select = c->persistent && !prefill_mode && lo <= Hp + TP_SELECT && hi > Hp + TP_FINAL;
    }
    if (!c->gtab_ready) P.s.gtab = nullptr;
    hipError_t e;
    launch_step(P, c->n_cus, c->stream, &e);
    if (e != hipSuccess) return fail(c, VADUSA_EHIP, "step kernel launch failed: %s", hipGetErrorString(e));
    if (c->persistent) { const int live = step_live_phases(P); c->epoch += (uint32_t)(live > 0 ? live - 1 : 0); }
    if (topk_apart) launch_topk(D, c->s, seq0, nseq, c->stream);
    return VADUSA_OK;
}

// After a synchronisation: did a kernel give up at a grid barrier?
static int kerr_seen(vadusa_ctx* c, int32_t k) {
    if (k) {
        // The launch that gave up left the barrier counters and the decoding state half-way: nothing the context
        // holds can be trusted until vadusa_prefill has reset it (see recover()).
        c->errored = 1;
        return fail(c, VADUSA_EHIP, "the step kernel timed out at a grid barrier; vadusa_prefill resets the context");
    }
    return VADUSA_OK;
}
static int check_kerr(vadusa_ctx* c) {
    if (!c->cfg.dtype) return VADUSA_OK;
    int32_t k = 0;
    HIP_TRY(c, hipMemcpy(&k, c->s.kerr, 4, hipMemcpyDeviceToHost));
    return kerr_seen(c, k);
}

// Every call except vadusa_prefill, vadusa_load_weights and vadusa_destroy refuses a context whose kernel gave up.
static int refuse_errored(vadusa_ctx* c) {
    if (c->errored) return fail(c, VADUSA_ESTATE, "a step kernel gave up at a grid barrier earlier; vadusa_prefill resets the context");
    return VADUSA_OK;
}

// Back to a clean start after a kernel gave up: nothing is running (the stream is drained), the barrier counters,
// the error word and the host's epoch start again from zero.  The decoding state is rebuilt by the prefill that follows.
static int recover(vadusa_ctx* c) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemset(c->s.bar, 0, (size_t)VADUSA_BAR_WORDS * 4));
    HIP_TRY(c, hipMemset(c->s.kerr, 0, 16));
    c->epoch = 0;
    c->errored = 0;
    std::fill(c->pending.begin(), c->pending.end(), 0);
    if (c->state > 1) c->state = 1;
    return VADUSA_OK;
}

static void forward(vadusa_ctx* c, const Dims& D, int table, int prefill_mode, bool want_logits) {
    const int dt = c->cfg.dtype;
    const DevState& s = c->s;
    hipStream_t st = c->stream;
    const int R = D.B * D.M;
    const size_t kv_layer = (size_t)D.Bmax * D.nH * kv_cap(D.maxpos) * 64 * c->elem;
    launch_embed(D, s, dt, prefill_mode, table, st);
    for (int l = 0; l < D.Ly; ++l) {
        const LayerW& w = c->layers[l];
        launch_layernorm(s.x, w.ln1_g, w.ln1_b, s.xn, R, D.d, dt, st);
        GemmArgs a{};
        a.X = s.xn; a.W = w.Wqkv; a.bias = w.bqkv; a.R = R; a.K = D.d; a.N = 3 * D.d; a.epi = EPI_QKV;
        a.out = s.q; a.Kc = (char*)s.Kc + l * kv_layer; a.Vc = (char*)s.Vc + l * kv_layer;
        a.L = s.L; a.M = D.M; a.nH = D.nH; a.maxpos = D.maxpos; a.d = D.d;
        gemm(c, a);
        launch_attn_simple(D, s, l, table, dt, st);
        GemmArgs o{};
        o.X = s.att; o.W = w.Wo; o.bias = w.bo; o.R = R; o.K = D.d; o.N = D.d; o.epi = EPI_RESID; o.outf = s.x;
        gemm(c, o);
        launch_layernorm(s.x, w.ln2_g, w.ln2_b, s.xn, R, D.d, dt, st);
        GemmArgs f1{};
        f1.X = s.xn; f1.W = w.W1; f1.bias = w.b1; f1.R = R; f1.K = D.d; f1.N = D.F; f1.epi = EPI_GELU; f1.out = s.hid;
        gemm(c, f1);
        GemmArgs f2{};
        f2.X = s.hid; f2.W = w.W2; f2.bias = w.b2; f2.R = R; f2.K = D.F; f2.N = D.d; f2.epi = EPI_RESID; f2.outf = s.x;
        gemm(c, f2);
    }
    if (want_logits) {
        launch_layernorm(s.x, s.lnf_g, s.lnf_b, s.hn, R, D.d, dt, st);
        GemmArgs h{};
        h.X = s.hn; h.W = s.W_out; h.bias = nullptr; h.R = R; h.K = D.d; h.N = D.V1; h.epi = EPI_F32; h.outf = s.logits;
        gemm(c, h);
    }
}

// Draft heads on the hidden state of the last accepted node (Sec. 2.1,
// Sec. 3.1.1): z_i = W2_i (h + SiLU(W1_i h + b1_i)), then the top-k lists.
static void draft_heads(vadusa_ctx* c, const Dims& D, int seq0, int nseq) {
    const DevState& s = c->s;
    for (int i = 0; i < D.Hh; ++i) {
        char* r = (char*)s.rdraft + ((size_t)i * D.Bmax + seq0) * D.d * c->elem;
        GemmArgs a{};
        a.X = (char*)s.hbest + (size_t)seq0 * D.d * c->elem; a.W = c->draft[i].W1; a.bias = c->draft[i].b1;
        a.R = nseq; a.K = D.d; a.N = D.d; a.epi = EPI_SILU_RESID; a.out = r;
        gemm(c, a);
        GemmArgs z{};
        z.X = r; z.W = c->draft[i].W2; z.bias = nullptr; z.R = nseq; z.K = D.d; z.N = D.V1; z.epi = EPI_F32;
        z.outf = s.zdraft + ((size_t)i * D.Bmax + seq0) * D.V1;
        gemm(c, z);
    }
    launch_topk(D, s, seq0, nseq, c->stream);
}

// ---------------------------------------------------------------------------
// prefill
// ---------------------------------------------------------------------------
extern "C" int vadusa_prefill(vadusa_ctx* c, int32_t batch, const int32_t* text_tok, const int32_t* text_len,
                              const int32_t* prompt_tok, const int32_t* prompt_len, int32_t* first_root) {
    if (!c) return VADUSA_EINVAL;
    if (c->state < 1) return fail(c, VADUSA_ESTATE, "weights not loaded");
    if (batch < 1 || batch > c->cfg.max_batch) return fail(c, VADUSA_EINVAL, "batch %d outside 1..%d", batch, c->cfg.max_batch);
    if (!text_len || !prompt_len) return fail(c, VADUSA_EINVAL, "length arrays are null");
    if (c->errored) { int rc = recover(c); if (rc) return rc; }
    int Mc = prefill_rows(c->cfg);
    {   // no pass needs more rows per sequence than the longest sequence has (whole 16-row tiles)
        int longest = 1;
        for (int b = 0; b < batch; ++b) longest = std::max(longest, text_len[b] + prompt_len[b]);
        Mc = std::min(Mc, std::max((longest + 15) / 16 * 16, std::min(c->cfg.max_tree_nodes, Mc)));
    }
    std::vector<std::vector<int32_t>> seqs(batch);
    size_t to = 0, po = 0;
    int max_chunks = 0;
    for (int b = 0; b < batch; ++b) {
        const int tl = text_len[b], pl = prompt_len[b];
        if (tl < 0 || pl < 0 || tl + pl < 1) return fail(c, VADUSA_EINVAL, "sequence %d is empty or has a negative length", b);
        if ((tl && !text_tok) || (pl && !prompt_tok)) return fail(c, VADUSA_EINVAL, "token array is null");
        if (tl + pl + c->cfg.max_tree_nodes > c->cfg.max_positions)
            return fail(c, VADUSA_EKVFULL, "sequence %d: %d tokens + %d tree rows exceed max_positions %d", b, tl + pl,
                        c->cfg.max_tree_nodes, c->cfg.max_positions);
        for (int i = 0; i < tl; ++i) {
            const int t = text_tok[to + i];
            if (t < 0 || t >= c->cfg.text_vocab) return fail(c, VADUSA_EINVAL, "text token %d out of range", t);
            seqs[b].push_back(-t - 1);
        }
        for (int i = 0; i < pl; ++i) {
            const int t = prompt_tok[po + i];
            if (t < 0 || t > c->cfg.speech_vocab) return fail(c, VADUSA_EINVAL, "speech token %d out of range", t);
            seqs[b].push_back(t);
        }
        to += tl; po += pl;
        max_chunks = std::max(max_chunks, (tl + pl + Mc - 1) / Mc);
    }
    const DevState& s = c->s;
    const size_t B = batch;
    // reset the decoding state
    HIP_TRY(c, hipMemsetAsync(s.L, 0, B * 4, c->stream));
    HIP_TRY(c, hipMemsetAsync(s.finished, 0, B * 4, c->stream));
    HIP_TRY(c, hipMemsetAsync(s.n_out, 0, B * 4, c->stream));
    HIP_TRY(c, hipMemsetAsync(s.path, 0, B * (VADUSA_MAX_DRAFT_HEADS + 2) * 4, c->stream));
    const Dims D = make_dims(c, batch, Mc);
    // chunks are right-aligned so that every sequence ends in the last chunk
    std::vector<std::vector<int32_t>> keep;   // host buffers stay alive until the final sync
    for (int ch = 0; ch < max_chunks; ++ch) {
        keep.emplace_back((size_t)batch * Mc, 0);
        keep.emplace_back(batch, 0);
        std::vector<int32_t>& ctok = keep[keep.size() - 2];
        std::vector<int32_t>& rows = keep[keep.size() - 1];
        for (int b = 0; b < batch; ++b) {
            const int total = (int)seqs[b].size();
            const int nch = (total + Mc - 1) / Mc;
            const int first = total - (nch - 1) * Mc;       // size of the sequence's first chunk
            const int k = ch - (max_chunks - nch);           // chunk index within the sequence
            if (k < 0) continue;
            const int begin = k == 0 ? 0 : first + (k - 1) * Mc;
            const int cnt = k == 0 ? first : Mc;
            rows[b] = cnt;
            for (int i = 0; i < cnt; ++i) ctok[(size_t)b * Mc + i] = seqs[b][begin + i];
        }
        HIP_TRY(c, hipMemcpyAsync(s.chunk_tok, ctok.data(), ctok.size() * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(s.n_rows, rows.data(), rows.size() * 4, hipMemcpyHostToDevice, c->stream));
        const bool last = ch == max_chunks - 1;
        if (c->cfg.dtype) {
            // bf16 model: the chunk is a causal "tree" for the step kernel; the last chunk also runs
            // the base head, the continuation and the draft heads (acceptance has no units here)
            const int H = 1 + 5 * D.Ly;
            int rc = run_phases(c, D, 1, 1, 1, 0, last ? H + TP_COUNT : H, 0, batch);
            if (rc) return rc;
        } else {
            forward(c, D, 1, 1, last);
        }
        if (!last) launch_advance(s, batch, c->stream);
    }
    if (!c->cfg.dtype) {
        launch_finalize(D, s, 0, batch, 1, c->cfg.ignore_eos, c->cfg.dtype, c->stream);
        draft_heads(c, D, 0, batch);
    }
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipGetLastError());
    { int rc = check_kerr(c); if (rc) return rc; }
    if (first_root) HIP_TRY(c, hipMemcpy(first_root, s.root, B * 4, hipMemcpyDeviceToHost));
    c->batch = batch;
    c->state = 2;
    for (int b = 0; b < batch; ++b) { c->L_ub[b] = (int)seqs[b].size(); c->pending[b] = 0; }
    return VADUSA_OK;
}

// ---------------------------------------------------------------------------
// verification
// ---------------------------------------------------------------------------
static int upload_tree(vadusa_ctx* c, const vadusa_tree_spec* t, const std::vector<int32_t>& depth) {
    const int M = t->n_nodes;
    const bool same = (int)c->tree_parent.size() == M &&
                      !memcmp(c->tree_parent.data(), t->parent, M * 4) &&
                      !memcmp(c->tree_rank.data() + 1, t->rank + 1, (M - 1) * 4);
    if (same) return VADUSA_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));   // earlier uploads from these vectors are done
    c->tree_parent.assign(t->parent, t->parent + M);
    c->tree_rank.assign(t->rank, t->rank + M);
    c->tree_rank[0] = 0;
    c->tree_depth = depth;
    std::vector<uint32_t> mask((size_t)M * MASK_WORDS, 0);
    for (int n = 0; n < M; ++n)
        for (int m = n; m >= 0; m = t->parent[m]) mask[(size_t)n * MASK_WORDS + (m >> 5)] |= 1u << (m & 31);
    const DevState& s = c->s;
    HIP_TRY(c, hipMemcpy(s.t_parent[0], c->tree_parent.data(), M * 4, hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(s.t_depth[0], c->tree_depth.data(), M * 4, hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(s.t_rank[0], c->tree_rank.data(), M * 4, hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(s.t_mask[0], mask.data(), mask.size() * 4, hipMemcpyHostToDevice));
    return VADUSA_OK;
}

static void mark_compacted(vadusa_ctx* c, int seq0, int nseq, int n_forced) {
    bool any = false;
    for (int b = 0; b < c->batch; ++b) {
        if (b >= seq0 && b < seq0 + nseq && c->pending[b]) {
            c->pending[b] = 0;
            c->L_ub[b] += (n_forced ? n_forced : std::min(c->cfg.n_draft_heads + 1, c->M));
        }
        any |= c->pending[b] != 0;
    }
    if (!any) c->state = 2;
}

// Verification; with fuse_compact the compaction of every sequence's chosen path and the
// draft heads follow in the same launch (bf16 model) or right behind (fp32 model).
static int verify_impl(vadusa_ctx* c, const vadusa_tree_spec* tree, int32_t tau, const int32_t* draft_override,
                       bool fuse_compact, const vadusa_sampling* sp = nullptr) {
    if (!c) return VADUSA_EINVAL;
    { int rc = refuse_errored(c); if (rc) return rc; }
    if (c->state != 2) return fail(c, VADUSA_ESTATE, c->state == 3 ? "a verification is still waiting for vadusa_kv_compact" : "prefill first");
    if (tau < 1) return fail(c, VADUSA_EINVAL, "tau must be >= 1 (got %d)", tau);
    if (sp) {
        if (!(sp->temperature > 0.f) || !std::isfinite(sp->temperature))
            return fail(c, VADUSA_EINVAL, "temperature must be positive and finite");
        if (!(sp->top_p > 0.f)) return fail(c, VADUSA_EINVAL, "top_p must be positive");
        if (!sp->uniforms) return fail(c, VADUSA_EINVAL, "uniforms is null");
        if ((size_t)(c->cfg.speech_vocab + 1) * sizeof(float) > 65536)
            return fail(c, VADUSA_ESHAPE, "stochastic verification keeps one row of V+1 floats in 64 KiB of LDS: vocabulary too large");
    }
    char msg[256];
    std::vector<int32_t> depth;
    int rc = tree_depths(&c->cfg, tree, &depth, msg, sizeof msg);
    if (rc) return fail(c, rc, "%s", msg);
    const int M = tree->n_nodes, B = c->batch;
    const DevState& s = c->s;
    // capacity: rows L .. L+M-1 are written by this forward
    bool maybe_full = false;
    for (int b = 0; b < B; ++b) maybe_full |= c->L_ub[b] + M > c->cfg.max_positions;
    if (maybe_full) {
        std::vector<int32_t> L(B), fin(B);
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        HIP_TRY(c, hipMemcpy(L.data(), s.L, B * 4, hipMemcpyDeviceToHost));
        HIP_TRY(c, hipMemcpy(fin.data(), s.finished, B * 4, hipMemcpyDeviceToHost));
        for (int b = 0; b < B; ++b) {
            c->L_ub[b] = L[b];
            if (!fin[b] && L[b] + M > c->cfg.max_positions)
                return fail(c, VADUSA_EKVFULL, "sequence %d: L = %d plus %d tree rows exceeds max_positions %d", b, L[b], M, c->cfg.max_positions);
        }
    }
    rc = upload_tree(c, tree, depth);
    if (rc) return rc;
    if (draft_override) {
        for (size_t i = 0; i < (size_t)B * c->cfg.n_draft_heads * VADUSA_MAX_TOPK; ++i)
            if (draft_override[i] < 0 || draft_override[i] > c->cfg.speech_vocab)
                return fail(c, VADUSA_EINVAL, "draft_override holds a token outside the vocabulary");
        HIP_TRY(c, hipMemcpyAsync(s.draft_topk, draft_override, (size_t)B * c->cfg.n_draft_heads * VADUSA_MAX_TOPK * 4,
                                  hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));   // the caller's buffer is not kept
    }
    const Dims D = make_dims(c, B, M);
    c->M = M;
    c->sampled = sp != nullptr;
    if (sp) {
        const size_t bytes = (size_t)B * M * D.V1 * sizeof(float);
        HIP_TRY(c, hipMemcpyAsync(c->uniforms, sp->uniforms, bytes,
                                  sp->uniforms_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, c->stream));
        if (!sp->uniforms_on_device) HIP_TRY(c, hipStreamSynchronize(c->stream));   // the caller's buffer is not kept
    }
    // Stochastic rule: the forward stops after the base head, the logits become perturbed scores,
    // and acceptance, choice and continuation rank the scores in place of the logits.
    DevState sr = s;
    if (sp) sr.logits = c->scores;
    if (c->cfg.dtype) {
        const int H = 1 + 5 * D.Ly;
        const int end = fuse_compact ? H + TP_COUNT : H + TP_FINAL;
        if (sp) {
            rc = run_phases(c, D, 0, 0, tau, 0, H + TP_EDGES, 0, B);
            if (rc) return rc;
            launch_perturb(s.logits, c->uniforms, c->scores, B * M, D.V1, sp->temperature, sp->top_p, tau, c->stream);
            rc = run_phases(c, D, 0, 0, tau, H + TP_EDGES, end, 0, B, c->scores);
        } else {
            rc = run_phases(c, D, 0, 0, tau, 0, end, 0, B);
        }
        if (rc) return rc;
    } else {
        forward(c, D, 0, 0, true);
        if (sp) launch_perturb(s.logits, c->uniforms, c->scores, B * M, D.V1, sp->temperature, sp->top_p, tau, c->stream);
        launch_accept(D, sr, tau, c->cfg.ignore_eos, c->stream);
        if (fuse_compact) {
            launch_finalize(D, sr, 0, B, 0, c->cfg.ignore_eos, 0, c->stream);
            launch_commit_kv(D, s, 0, B, 0, c->stream);
            draft_heads(c, D, 0, B);
        }
        HIP_TRY(c, hipGetLastError());
    }
    c->state = 3;
    for (int b = 0; b < B; ++b) c->pending[b] = 1;
    if (fuse_compact) mark_compacted(c, 0, B, 0);
    return VADUSA_OK;
}

extern "C" int vadusa_verify(vadusa_ctx* c, const vadusa_tree_spec* tree, int32_t tau, const int32_t* draft_override) {
    return verify_impl(c, tree, tau, draft_override, false);
}

extern "C" int vadusa_verify_sampled(vadusa_ctx* c, const vadusa_tree_spec* tree, int32_t tau,
                                     const vadusa_sampling* sampling, const int32_t* draft_override) {
    if (!c) return VADUSA_EINVAL;
    if (!sampling) return fail(c, VADUSA_EINVAL, "sampling is null");
    return verify_impl(c, tree, tau, draft_override, false, sampling);
}

extern "C" int vadusa_kv_compact(vadusa_ctx* c, int32_t seq, const int32_t* path_nodes, int32_t n) {
    if (!c) return VADUSA_EINVAL;
    { int rc = refuse_errored(c); if (rc) return rc; }
    if (c->state != 3) return fail(c, VADUSA_ESTATE, "no verification is pending");
    const int B = c->batch;
    if (seq < -1 || seq >= B) return fail(c, VADUSA_EINVAL, "seq %d outside -1..%d", seq, B - 1);
    if (seq == -1 && (path_nodes || n)) return fail(c, VADUSA_EINVAL, "seq = -1 takes no explicit path");
    if ((path_nodes == nullptr) != (n == 0)) return fail(c, VADUSA_EINVAL, "path_nodes and n must both be given or both be empty");
    const DevState& s = c->s;
    const Dims D = make_dims(c, B, c->M);
    int seq0 = 0, nseq = B;
    if (seq >= 0) {
        if (!c->pending[seq]) return fail(c, VADUSA_ESTATE, "sequence %d has no pending verification", seq);
        seq0 = seq; nseq = 1;
        if (path_nodes) {
            if (n < 1 || n > c->cfg.n_draft_heads + 1) return fail(c, VADUSA_EINVAL, "path length %d outside 1..%d", n, c->cfg.n_draft_heads + 1);
            if (path_nodes[0] != 0) return fail(c, VADUSA_EINVAL, "a path starts at node 0");
            for (int j = 1; j < n; ++j)
                if (path_nodes[j] < 1 || path_nodes[j] >= c->M || c->tree_parent[path_nodes[j]] != path_nodes[j - 1])
                    return fail(c, VADUSA_EINVAL, "path_nodes[%d] is not a child of path_nodes[%d]", j, j - 1);
            int32_t buf[VADUSA_MAX_DRAFT_HEADS + 2] = {0};
            buf[0] = n;
            memcpy(buf + 1, path_nodes, n * 4);
            HIP_TRY(c, hipMemcpyAsync(s.path + (size_t)seq * (VADUSA_MAX_DRAFT_HEADS + 2), buf, sizeof buf,
                                      hipMemcpyHostToDevice, c->stream));
            HIP_TRY(c, hipStreamSynchronize(c->stream));
        }
    }
    if (c->cfg.dtype) {
        const int H = 1 + 5 * D.Ly;
        int rc = run_phases(c, D, 0, 0, 1, H + TP_FINAL, H + TP_COUNT, seq0, nseq, c->sampled ? c->scores : nullptr);
        if (rc) return rc;
    } else {
        DevState sr = s;
        if (c->sampled) sr.logits = c->scores;   // the next root is the first draw at the last committed node
        launch_finalize(D, sr, seq0, nseq, 0, c->cfg.ignore_eos, 0, c->stream);
        launch_commit_kv(D, s, seq0, nseq, 0, c->stream);
        draft_heads(c, D, seq0, nseq);
        HIP_TRY(c, hipGetLastError());
    }
    mark_compacted(c, seq0, nseq, path_nodes ? n : 0);
    return VADUSA_OK;
}

static int step_impl(vadusa_ctx* c, const vadusa_tree_spec* tree, int32_t tau, const vadusa_sampling* sp,
                     const int32_t* draft_override, int32_t* accepted_tok, int32_t* accepted_len) {
    if ((accepted_tok == nullptr) != (accepted_len == nullptr))
        return fail(c, VADUSA_EINVAL, "accepted_tok and accepted_len must both be given or both be null");
    int rc = verify_impl(c, tree, tau, draft_override, true, sp);
    if (rc) return rc;
    if (accepted_tok) {
        const int B = c->batch, W = VADUSA_MAX_DRAFT_HEADS + 1, Hh1 = c->cfg.n_draft_heads + 1;
        // one copy for everything the host reads after a step (every separate copy is a trip of tens of microseconds)
        std::vector<int32_t> blk(4 + 2 * (size_t)c->cfg.max_batch + (size_t)c->cfg.max_batch * W);
        HIP_TRY(c, hipMemcpyAsync(blk.data(), c->s.kerr, blk.size() * 4, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        rc = kerr_seen(c, c->cfg.dtype ? blk[0] : 0);
        if (rc) return rc;
        const int32_t* len = blk.data() + 4;
        const int32_t* L = len + c->cfg.max_batch;
        const int32_t* tok = L + c->cfg.max_batch;
        for (int b = 0; b < B; ++b) {
            accepted_len[b] = len[b];
            for (int j = 0; j < Hh1; ++j) accepted_tok[(size_t)b * Hh1 + j] = j < len[b] ? tok[(size_t)b * W + j] : -1;
            c->L_ub[b] = L[b];
        }
    }
    return VADUSA_OK;
}

extern "C" int vadusa_step(vadusa_ctx* c, const vadusa_tree_spec* tree, int32_t tau, const int32_t* draft_override,
                           int32_t* accepted_tok, int32_t* accepted_len) {
    if (!c) return VADUSA_EINVAL;
    return step_impl(c, tree, tau, nullptr, draft_override, accepted_tok, accepted_len);
}

extern "C" int vadusa_step_sampled(vadusa_ctx* c, const vadusa_tree_spec* tree, int32_t tau,
                                   const vadusa_sampling* sampling, const int32_t* draft_override,
                                   int32_t* accepted_tok, int32_t* accepted_len) {
    if (!c) return VADUSA_EINVAL;
    if (!sampling) return fail(c, VADUSA_EINVAL, "sampling is null");
    return step_impl(c, tree, tau, sampling, draft_override, accepted_tok, accepted_len);
}

extern "C" int vadusa_read_output(vadusa_ctx* c, int32_t seq, int32_t* tok, int32_t capacity, int32_t* n_out) {
    if (!c) return VADUSA_EINVAL;
    { int rc = refuse_errored(c); if (rc) return rc; }
    if (c->state < 2) return fail(c, VADUSA_ESTATE, "prefill first");
    if (seq < 0 || seq >= c->batch || !n_out) return fail(c, VADUSA_EINVAL, "bad seq or null n_out");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    { int rc = check_kerr(c); if (rc) return rc; }
    int32_t n = 0;
    HIP_TRY(c, hipMemcpy(&n, c->s.n_out + seq, 4, hipMemcpyDeviceToHost));
    *n_out = n;
    if (tok) {
        const int m = std::min(n, capacity);
        if (m > 0) HIP_TRY(c, hipMemcpy(tok, c->s.out_tok + (size_t)seq * c->cfg.max_positions, (size_t)m * 4, hipMemcpyDeviceToHost));
    }
    return VADUSA_OK;
}

// ---------------------------------------------------------------------------
// inspection
// ---------------------------------------------------------------------------
extern "C" int vadusa_debug_read(vadusa_ctx* c, int32_t what, void* host, size_t bytes) {
    if (!c || !host) return VADUSA_EINVAL;
    { int rc = refuse_errored(c); if (rc) return rc; }
    if (c->state < 2) return fail(c, VADUSA_ESTATE, "prefill first");
    const DevState& s = c->s;
    const size_t B = c->batch, M = c->M, d = c->cfg.d_model, V1 = c->cfg.speech_vocab + 1, Hh = c->cfg.n_draft_heads;
    const size_t Bmax = c->cfg.max_batch;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (what != VADUSA_DBG_PHASE_CLOCK) { int rc = check_kerr(c); if (rc) return rc; }   // data of a launch that gave up is never handed out
    const void* src = nullptr;
    size_t need = 0;
    switch (what) {
    case VADUSA_DBG_LOGITS: src = s.logits; need = B * M * V1 * 4; break;
    case VADUSA_DBG_SCORES:
        if (!c->sampled) return fail(c, VADUSA_ESTATE, "the last verification was not a stochastic one");
        src = c->scores; need = B * M * V1 * 4; break;
    case VADUSA_DBG_TREE_TOK: src = s.tok; need = B * M * 4; break;
    case VADUSA_DBG_DRAFT_TOPK: src = s.draft_topk; need = B * Hh * VADUSA_MAX_TOPK * 4; break;
    case VADUSA_DBG_KV_LEN: src = s.L; need = B * 4; break;
    case VADUSA_DBG_ROOT: src = s.root; need = B * 4; break;
    case VADUSA_DBG_EDGE_OK: src = s.edge_ok; need = B * M * 4; break;
    case VADUSA_DBG_FINISHED: src = s.finished; need = B * 4; break;
    case VADUSA_DBG_PHASE_CLOCK:
#ifndef VADUSA_CLOCK_BUILD
        return fail(c, VADUSA_ESTATE, "this library was built without timing points: use libvadusa_clock.so");
#endif
        src = s.tprof; need = 1024 * 8; break;
    case VADUSA_DBG_H_NODES: {
        need = B * M * d * 4;
        if (bytes != need) return fail(c, VADUSA_EINVAL, "expected %zu bytes", need);
        if (c->cfg.dtype)   // the step kernel keeps no node states: recompute them from the residual stream
            launch_layernorm(s.x, s.lnf_g, s.lnf_b, s.hn, (int)(B * M), (int)d, 1, c->stream);
        launch_to_float(s.hn, s.staging, B * M * d, c->cfg.dtype, c->stream);
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        HIP_TRY(c, hipMemcpy(host, s.staging, need, hipMemcpyDeviceToHost));
        return VADUSA_OK;
    }
    case VADUSA_DBG_PATH: {
        need = B * (Hh + 2) * 4;
        if (bytes != need) return fail(c, VADUSA_EINVAL, "expected %zu bytes", need);
        std::vector<int32_t> tmp(B * (VADUSA_MAX_DRAFT_HEADS + 2));
        HIP_TRY(c, hipMemcpy(tmp.data(), s.path, tmp.size() * 4, hipMemcpyDeviceToHost));
        int32_t* o = (int32_t*)host;
        for (size_t b = 0; b < B; ++b)
            for (size_t j = 0; j < Hh + 2; ++j) o[b * (Hh + 2) + j] = tmp[b * (VADUSA_MAX_DRAFT_HEADS + 2) + j];
        return VADUSA_OK;
    }
    case VADUSA_DBG_DRAFT_LOGITS: {
        need = B * Hh * V1 * 4;
        if (bytes != need) return fail(c, VADUSA_EINVAL, "expected %zu bytes", need);
        float* o = (float*)host;
        for (size_t b = 0; b < B; ++b)
            for (size_t i = 0; i < Hh; ++i)
                HIP_TRY(c, hipMemcpy(o + (b * Hh + i) * V1, s.zdraft + (i * Bmax + b) * V1, V1 * 4, hipMemcpyDeviceToHost));
        return VADUSA_OK;
    }
    default: return fail(c, VADUSA_EINVAL, "unknown item %d", what);
    }
    if (bytes != need) return fail(c, VADUSA_EINVAL, "expected %zu bytes, got %zu", need, bytes);
    if (need) HIP_TRY(c, hipMemcpy(host, src, need, hipMemcpyDeviceToHost));
    return VADUSA_OK;
}

extern "C" int vadusa_debug_read_kv(vadusa_ctx* c, int32_t layer, int32_t seq, int32_t which, int32_t pos0,
                                    int32_t npos, float* host) {
    if (!c || !host) return VADUSA_EINVAL;
    { int rc = refuse_errored(c); if (rc) return rc; }
    if (c->state < 2) return fail(c, VADUSA_ESTATE, "prefill first");
    if (layer < 0 || layer >= c->cfg.n_layers || seq < 0 || seq >= c->cfg.max_batch || (which != 0 && which != 1) ||
        pos0 < 0 || npos < 1 || pos0 + npos > c->cfg.max_positions)
        return fail(c, VADUSA_EINVAL, "bad layer / seq / range");
    const Dims D = make_dims(c, c->batch, c->M);
    const size_t kv_layer = (size_t)D.Bmax * D.nH * kv_cap(D.maxpos) * 64 * c->elem;
    const char* base = (const char*)(which ? c->s.Vc : c->s.Kc) + layer * kv_layer;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    { int rc = check_kerr(c); if (rc) return rc; }
    launch_read_kv(D, base, seq, which, pos0, npos, c->s.staging, c->cfg.dtype, c->stream);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(host, c->s.staging, (size_t)npos * D.d * 4, hipMemcpyDeviceToHost));
    return VADUSA_OK;
}

// ---------------------------------------------------------------------------
// vadusa_debug_read_kv for callers that may not allocate: the float staging rows live in a file-scope device
// array instead of the arena's staging area.  Every GPU the library runs on holds its own copy of the array (1 MiB)
// until the process ends; its device address is looked up once per device, with that device current, and only
// that pointer is ever handed to a kernel or a copy (the array's name is a host-side stand-in, not an address).
// ---------------------------------------------------------------------------
#define VADUSA_STATIC_KV_FLOATS (256 * 1024)
static __device__ __align__(256) float scratch[VADUSA_STATIC_KV_FLOATS];
#define VADUSA_MAX_DEVICES 64
static float* g_scratch_ptr[VADUSA_MAX_DEVICES];   // device address of `scratch` on each device, null until looked up

static int static_scratch(vadusa_ctx* c, float** out) {
    int dev = -1;
    HIP_TRY(c, hipGetDevice(&dev));
    if (dev < 0 || dev >= VADUSA_MAX_DEVICES) return fail(c, VADUSA_EINVAL, "device %d outside 0..%d", dev, VADUSA_MAX_DEVICES - 1);
    float* p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        HIP_TRY(c, hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(c, VADUSA_EHIP, "hipGetSymbolAddress returned a null address");
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);   // two threads may both look it up: same value
    }
    *out = p;
    return VADUSA_OK;
}

extern "C" int vadusa_debug_read_kv_static(vadusa_ctx* c, int32_t layer, int32_t seq, int32_t which, int32_t pos0,
                                           int32_t npos, float* host) {
    if (!c || !host) return VADUSA_EINVAL;
    { int rc = refuse_errored(c); if (rc) return rc; }
    if (c->state < 2) return fail(c, VADUSA_ESTATE, "prefill first");
    if (layer < 0 || layer >= c->cfg.n_layers || seq < 0 || seq >= c->cfg.max_batch || (which != 0 && which != 1) ||
        pos0 < 0 || npos < 1 || pos0 + npos > c->cfg.max_positions)
        return fail(c, VADUSA_EINVAL, "bad layer / seq / range");
    const Dims D = make_dims(c, c->batch, c->M);
    if ((size_t)npos * D.d > (size_t)VADUSA_STATIC_KV_FLOATS)
        return fail(c, VADUSA_ESHAPE, "%d rows of %d floats exceed the static staging array of %d floats (at most %d rows per call)",
                    npos, D.d, VADUSA_STATIC_KV_FLOATS, VADUSA_STATIC_KV_FLOATS / D.d);
    float* stage = nullptr;
    { int rc = static_scratch(c, &stage); if (rc) return rc; }
    const size_t kv_layer = (size_t)D.Bmax * D.nH * kv_cap(D.maxpos) * 64 * c->elem;
    const char* base = (const char*)(which ? c->s.Vc : c->s.Kc) + layer * kv_layer;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    { int rc = check_kerr(c); if (rc) return rc; }
    // every float of rows 0..npos-1 is overwritten by the kernel: nothing of the previous call's contents is read
    launch_read_kv(D, base, seq, which, pos0, npos, stage, c->cfg.dtype, c->stream);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(host, stage, (size_t)npos * D.d * 4, hipMemcpyDeviceToHost));
    return VADUSA_OK;
}
