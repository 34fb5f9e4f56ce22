/*
 * vadusa.h -- C ABI of the VADUSA speculative decode step for one MI355X (gfx950).
 *
 * The library runs, entirely in its own HIP kernels, one step of the decoding
 * scheme of "Fast and High-Quality Auto-Regressive Speech Synthesis via
 * Speculative Decoding" (arXiv 2410.21951): draft heads on the last hidden
 * state (Sec. 2.1, Sec. 3.1.1), expansion of their top-k lists into a fixed
 * sparse candidate tree (Sec. 2.1, Sec. 2.4), one tree-masked forward of every
 * tree node through the decoder against a KV cache (Sec. 2.1 "tree attention",
 * Sec. 2.2), verification with tolerance (Algorithm 1), choice of the longest /
 * leftmost accepted branch (Sec. 2.3) and compaction of the KV cache to the
 * accepted path.
 *
 * Conventions
 *  - All functions return VADUSA_OK (0) or a negative error code; nothing
 *    throws or aborts across this boundary.  After an error the decoding state
 *    of the context is unchanged unless the code is VADUSA_EHIP.  A text for the
 *    last error of a context is available from vadusa_last_error().
 *  - The bf16 step runs as one persistent kernel whose workgroups meet at grid
 *    barriers, launched as an ordinary kernel with one workgroup per compute
 *    unit: it needs the GPU to itself while it runs (no other kernel on another
 *    stream or from another process at the same time).  Every wait is bounded: if a
 *    workgroup is not placed, the kernel gives up, the next call that
 *    synchronises (a step with result pointers, vadusa_read_output, the debug
 *    readers) returns VADUSA_EHIP, and from then on every call except
 *    vadusa_prefill, vadusa_load_weights and vadusa_destroy returns
 *    VADUSA_ESTATE; vadusa_prefill resets the barrier state and starts the
 *    sequences again.  VADUSA_COOPERATIVE_LAUNCH=1 makes the runtime verify
 *    residency at every launch instead (about 18 us per step).
 *  - "host" / "device" in a comment says where a pointer must point.  The
 *    library never keeps a caller's host pointer after the call returns.
 *  - The library allocates no device memory: the caller passes one device
 *    arena of vadusa_arena_bytes() bytes (256-byte aligned) that the context
 *    carves up and owns until vadusa_destroy(); the caller frees it afterwards.
 *  - All kernels are enqueued on the HIP stream given to vadusa_create().
 *  - Speech token ids are 0..V-1, the end-of-sequence id is V (= speech_vocab);
 *    logits have V+1 entries.
 */
#ifndef VADUSA_H
#define VADUSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VADUSA_OK        0
#define VADUSA_EINVAL   -1   /* bad argument (null pointer, tau < 1, malformed tree ...) */
#define VADUSA_ESHAPE   -2   /* configuration outside what the kernels support */
#define VADUSA_EKVFULL  -3   /* a sequence has no room left for L + tree rows */
#define VADUSA_ESTATE   -4   /* call out of order (e.g. step before prefill) */
#define VADUSA_EHIP     -5   /* a HIP call or a kernel reported a failure */

#define VADUSA_MAX_TREE_NODES 128   /* M, root included (Sec. 3.1.3 uses 64, 96, 128) */
#define VADUSA_MAX_TOPK        16   /* largest rank + 1 a tree may use (the paper uses 10) */
#define VADUSA_MAX_PREFILL_CHUNK 1024 /* most rows of one sequence in one pass of the prefill */
#define VADUSA_MAX_DRAFT_HEADS  8   /* the paper uses 4 or 6 */

typedef struct vadusa_ctx vadusa_ctx;   /* opaque */

/* Model and capacity description (Sec. 3.1.1 gives 12 / 1024 / 16 / 4096). */
typedef struct {
    int32_t n_layers;
    int32_t d_model;        /* must equal n_heads * head_dim, multiple of 64 */
    int32_t n_heads;
    int32_t head_dim;       /* 64 */
    int32_t d_ffn;          /* multiple of 64 */
    int32_t speech_vocab;   /* V; EOS id == V */
    int32_t text_vocab;
    int32_t n_draft_heads;  /* 1..VADUSA_MAX_DRAFT_HEADS */
    int32_t max_positions;  /* KV rows per sequence and rows of the position table */
    int32_t max_batch;      /* sequences decoded together */
    int32_t max_tree_nodes; /* largest M used in any step, <= VADUSA_MAX_TREE_NODES */
    int32_t dtype;          /* 0: fp32 weights/activations, 1: bf16 storage with fp32 accumulation */
    int32_t ignore_eos;     /* 1: EOS is an ordinary token (fixed-length benchmarks) */
    int32_t prefill_chunk;  /* rows of a sequence that one pass of vadusa_prefill runs through the decoder:
                               0 = max_tree_nodes, else 1..VADUSA_MAX_PREFILL_CHUNK (longer passes turn the
                               prompt's linear maps into many-row products; the arena grows with
                               max_batch * prefill_chunk rows of activations) */
} vadusa_config;

/*
 * Candidate tree (Sec. 2.1 top-k tree, Sec. 2.4 sparse subset), host pointers.
 * Node 0 is the root (the base head's next token).  A node at depth D >= 1
 * carries rank[n]: its token is entry rank[n] of draft head D's top-k list.
 * Nodes must be in canonical order: by depth, then by the lexicographic order
 * of their rank paths, so that parent[n] < n and "leftmost" (Sec. 2.3) is the
 * smallest index among nodes of equal depth.  parent[0] = -1, rank[0] ignored.
 * Depth may not exceed n_draft_heads, ranks must be < VADUSA_MAX_TOPK and
 * siblings must have distinct ranks.
 */
typedef struct {
    int32_t        n_nodes;
    const int32_t* parent;   /* host [n_nodes] */
    const int32_t* rank;     /* host [n_nodes] */
} vadusa_tree_spec;

/* ---- host-only helpers (no GPU needed) -------------------------------- */

/* Checks a configuration; VADUSA_OK or VADUSA_EINVAL / VADUSA_ESHAPE.  If msg
 * is non-null a description of the first problem is written (at most msg_bytes). */
int vadusa_config_check(const vadusa_config* cfg, char* msg, size_t msg_bytes);

/* Builds a sparse candidate tree (Sec. 2.4: within a fixed number of nodes, maximise the
 * expected accepted length).  acc is host memory [n_heads][width]: acc[i][r] is the measured
 * probability that draft head i+1's rank-r candidate is accepted given that its parent was
 * (from a calibration run with the full tree); every value must lie in [0, 1].  A node's path
 * probability is the product of the acc values along its rank path; the n_nodes nodes (root
 * included) of largest path probability are kept, which is the ancestor-closed set of that
 * size with the largest expected accepted length.  Equal probabilities: the shallower node
 * first, then the lexicographically smaller rank path.  Output in canonical order into the
 * caller's arrays parent[n_nodes], rank[n_nodes]; *n_out receives the number of nodes (less
 * than n_nodes only if the full tree is smaller).  VADUSA_EINVAL for bad arguments
 * (n_heads outside 1..VADUSA_MAX_DRAFT_HEADS, width outside 1..VADUSA_MAX_TOPK, n_nodes
 * outside 1..VADUSA_MAX_TREE_NODES, a value outside [0, 1], null pointers). */
int vadusa_build_tree(int32_t n_heads, int32_t width, const float* acc, int32_t n_nodes,
                      int32_t* parent, int32_t* rank, int32_t* n_out);

/* Checks a tree against a configuration (rules above). */
int vadusa_tree_check(const vadusa_config* cfg, const vadusa_tree_spec* tree,
                      char* msg, size_t msg_bytes);

/* Device bytes vadusa_create() needs for this configuration (0 if invalid). */
size_t vadusa_arena_bytes(const vadusa_config* cfg);

/* Number of fp32 values in the weight blob of vadusa_load_weights() (0 if invalid). */
size_t vadusa_blob_floats(const vadusa_config* cfg);

/* ---- life cycle -------------------------------------------------------- */

/* Creates a context inside `arena` (device, >= vadusa_arena_bytes(), 256-byte
 * aligned, current device).  hip_stream is a hipStream_t (NULL = default
 * stream).  *out receives the context (host object, freed by vadusa_destroy). */
int vadusa_create(const vadusa_config* cfg, void* arena, size_t arena_bytes,
                  void* hip_stream, vadusa_ctx** out);
/* Environment variables read by vadusa_create, VADUSA_COOPERATIVE_LAUNCH at the process's first
 * step launch (debugging and test aids; none changes results):
 *   VADUSA_PHASE_LAUNCHES       one kernel launch per phase of the bf16 step instead of one
 *                               persistent launch with grid barriers
 *   VADUSA_COOPERATIVE_LAUNCH   launch the persistent kernel cooperatively
 *   VADUSA_PHASE_CLOCK=n        record the timing points of VADUSA_DBG_PHASE_CLOCK in workgroup n - 1 (only the
 *                               library built with -DVADUSA_CLOCK_BUILD, libvadusa_clock.so, has them)
 *   VADUSA_BIG_MIN_UNITS=n      many-row kernel (>= 256 rows): a linear map takes 128 x 128 output
 *                               units, and attention whole (sequence, head) units, from n such
 *                               units on (default 256 = one per compute unit); lets tests
 *                               reach those code paths with small shapes */

/* Frees the context (host object).  Makes no HIP call, so it is safe in a finaliser or an exit handler;
 * the caller drains the stream before it frees or reuses the arena. */
void vadusa_destroy(vadusa_ctx* ctx);

const char* vadusa_last_error(const vadusa_ctx* ctx);

/*
 * Loads the model (Sec. 3.1.1) from a flat fp32 blob, host (blob_on_device = 0)
 * or device (1).  Every linear map is [out_features][in_features] row-major
 * (y = W x + b).  Order:
 *   E_text[text_vocab][d], E_speech[V+1][d], P[max_positions][d],
 *   per layer: ln1_g[d], ln1_b[d], Wqkv[3d][d] (q rows, then k, then v), bqkv[3d],
 *              Wo[d][d], bo[d], ln2_g[d], ln2_b[d], W1[F][d], b1[F], W2[d][F], b2[d],
 *   lnf_g[d], lnf_b[d], W_out[V+1][d],
 *   per draft head: Wd1[d][d], bd1[d], Wd2[V+1][d].
 * The block is pre-LayerNorm: x += Wo Attn(LN1 x) + bo; x += W2 GELU(W1 LN2 x + b1) + b2,
 * exact (erf) GELU, LayerNorm eps 1e-5; a draft head computes
 * z = Wd2 (h + SiLU(Wd1 h + bd1)) on the final-LayerNorm'd state h.
 * With dtype = 1 the values are rounded to bf16 (nearest even) while loading.
 * Synchronises the stream before returning.
 */
int vadusa_load_weights(vadusa_ctx* ctx, const float* blob, size_t n_floats, int blob_on_device);

/* ---- decoding ---------------------------------------------------------- */

/*
 * Prefilling pass (Sec. 2.1, Fig. 1a) for `batch` sequences (1..max_batch):
 * runs text tokens followed by prompt speech tokens through the decoder
 * (causal), fills the KV cache, takes the base head's first next token as the
 * root and the draft heads' top-k lists from the last position.
 * Host arrays: text_tok is the concatenation of all sequences' text tokens,
 * text_len[batch] their lengths; likewise prompt_tok / prompt_len.  Each
 * sequence needs text_len + prompt_len >= 1 and
 * text_len + prompt_len + max_tree_nodes <= max_positions.
 * first_root: host [batch] out, may be NULL.  Synchronises the stream.
 * Resets any previous decoding state.
 */
int vadusa_prefill(vadusa_ctx* ctx, int32_t batch,
                   const int32_t* text_tok, const int32_t* text_len,
                   const int32_t* prompt_tok, const int32_t* prompt_len,
                   int32_t* first_root);

/*
 * Verification half of a step: expands the draft lists into the tree's node
 * tokens, runs every node through the decoder in one tree-masked forward
 * (node n sees the committed prefix, itself and its ancestors; Sec. 2.1),
 * applies Algorithm 1 with tolerance tau in the deterministic reading (a draft
 * token is accepted iff fewer than tau logits of its parent's row rank before
 * it; equal logits: lower id first) and picks the longest, then leftmost,
 * accepted root path (Sec. 2.3).  Nothing is committed: the decision stays on
 * the device (see vadusa_debug_read) until vadusa_kv_compact().
 * draft_override: NULL, or host [batch][n_draft_heads][VADUSA_MAX_TOPK] token
 * ids used instead of the draft heads' own top-k lists (test hook).
 * Does not synchronise.
 */
int vadusa_verify(vadusa_ctx* ctx, const vadusa_tree_spec* tree, int32_t tau,
                  const int32_t* draft_override);

/*
 * Compaction: moves the K/V rows of the tree nodes path_nodes[0..n) of the
 * pending verification of sequence `seq` to cache rows L..L+n-1, advances L by
 * n, appends the nodes' tokens to the sequence's output, and continues from
 * the last of them: next root = top-1 of its logits, new draft lists from its
 * hidden state (Sec. 2.1: decoding continues from the prediction of the last
 * accepted token).  path_nodes: host [n], a root path (path_nodes[0] = 0, each
 * node the parent of the next); NULL with n = 0 commits the path the
 * verification chose (cut after the first EOS unless ignore_eos).
 * seq = -1 with path_nodes = NULL commits every sequence's chosen path.
 * VADUSA_ESTATE if no verification is pending for the sequence.
 * Does not synchronise.
 */
int vadusa_kv_compact(vadusa_ctx* ctx, int32_t seq, const int32_t* path_nodes, int32_t n);

/*
 * One whole speculative step = vadusa_verify + vadusa_kv_compact(-1, NULL, 0).
 * accepted_tok: host [batch][n_draft_heads + 1] out, accepted_len: host [batch]
 * out (1..n_draft_heads+1; 0 for a sequence that had already ended with EOS).
 * accepted_tok[b][0] is always the root (Algorithm 1: a_0 = c_0).
 * If both output pointers are NULL the step is only enqueued (no
 * synchronisation); results can be fetched later with vadusa_read_output().
 * Otherwise the stream is synchronised once at the end.
 */
int vadusa_step(vadusa_ctx* ctx, const vadusa_tree_spec* tree, int32_t tau,
                const int32_t* draft_override,
                int32_t* accepted_tok, int32_t* accepted_len);

/*
 * Stochastic form of Algorithm 1 (the verification as printed: at every position of a branch
 * tau tokens are drawn from the nucleus of the temperature-scaled distribution, Sec. 3.1.2,
 * and the next candidate is accepted iff it is among the draws).
 * With s = logit / temperature, the nucleus of a position keeps token v iff the tokens of
 * strictly larger s hold less than top_p of softmax(s) (equal s: kept or dropped together);
 * it is widened to the tau most probable tokens where it would hold fewer, so that tau draws
 * exist; top_p >= 1 keeps every token.  The tau draws are without replacement and come from
 * the caller's uniforms: the kept tokens are ordered by s - log(-log u), which lists them in
 * the order successive draws would, and the first tau are the draws.  The continuation token
 * after the accepted path is the first draw at its last node.
 * uniforms: [batch][tree->n_nodes][V+1] floats, each strictly inside (0, 1), independent;
 * host memory (copied before the call returns) or, with uniforms_on_device = 1, device memory
 * (copied on the stream).  The prefill's first root stays the most probable token.
 * Needs (V+1) * 4 <= 65536 bytes (VADUSA_ESHAPE otherwise).
 */
typedef struct {
    float        temperature;        /* > 0 */
    float        top_p;              /* > 0; >= 1 keeps every token */
    const float* uniforms;
    int32_t      uniforms_on_device; /* 0: host pointer, 1: device pointer */
} vadusa_sampling;

/* vadusa_verify with the stochastic rule; vadusa_kv_compact then continues from the first
 * draw at the last committed node.  Same state rules and errors as vadusa_verify, plus
 * VADUSA_EINVAL for a bad temperature / top_p or null pointers.  Does not synchronise
 * unless the uniforms come from host memory. */
int vadusa_verify_sampled(vadusa_ctx* ctx, const vadusa_tree_spec* tree, int32_t tau,
                          const vadusa_sampling* sampling, const int32_t* draft_override);

/* vadusa_step with the stochastic rule (= vadusa_verify_sampled + vadusa_kv_compact(-1, NULL, 0));
 * outputs as in vadusa_step. */
int vadusa_step_sampled(vadusa_ctx* ctx, const vadusa_tree_spec* tree, int32_t tau,
                        const vadusa_sampling* sampling, const int32_t* draft_override,
                        int32_t* accepted_tok, int32_t* accepted_len);

/* All tokens committed so far for `seq` (after synchronising the stream).
 * tok: host [capacity] out (may be NULL to query the count); *n_out: count. */
int vadusa_read_output(vadusa_ctx* ctx, int32_t seq, int32_t* tok, int32_t capacity,
                       int32_t* n_out);

/* ---- inspection (tests, parity checks) --------------------------------- */

enum {
    VADUSA_DBG_LOGITS     = 0,  /* float [batch][M][V+1], base-head logits of the last verify */
    VADUSA_DBG_H_NODES    = 1,  /* float [batch][M][d], final-LayerNorm'd node states */
    VADUSA_DBG_TREE_TOK   = 2,  /* int32 [batch][M], node tokens of the last verify */
    VADUSA_DBG_DRAFT_TOPK = 3,  /* int32 [batch][n_draft_heads][VADUSA_MAX_TOPK], current lists */
    VADUSA_DBG_KV_LEN     = 4,  /* int32 [batch], committed length L */
    VADUSA_DBG_ROOT       = 5,  /* int32 [batch], current root token */
    VADUSA_DBG_EDGE_OK    = 6,  /* int32 [batch][M], 1 if the node's own edge passed (root: 1) */
    VADUSA_DBG_PATH       = 7,  /* int32 [batch][n_draft_heads+2]: count, then node indices */
    VADUSA_DBG_FINISHED   = 8,  /* int32 [batch] */
    VADUSA_DBG_DRAFT_LOGITS = 9, /* float [batch][n_draft_heads][V+1], logits behind the lists */
    VADUSA_DBG_PHASE_CLOCK = 10, /* int64 [128][8]: device clock (100 MHz) of workgroup 0 in the last launch of
                                    the bf16 step kernel: [p][0] start of phase p, [p][1] its own units done,
                                    [p][2..] points inside a unit, [127][0] end of the kernel.  Recorded only by
                                    contexts created while the environment variable VADUSA_PHASE_CLOCK is set
                                    (each point costs a few hundred ns); zero otherwise.  The points are compiled
                                    into libvadusa_clock.so only (switched off they still cost the step 4 %);
                                    the ordinary library returns VADUSA_ESTATE */
    VADUSA_DBG_SCORES     = 11  /* float [batch][M][V+1]: the perturbed scores (s - log(-log u) on the nucleus,
                                    -inf elsewhere) of the last stochastic verification; VADUSA_ESTATE if the
                                    last verification was a deterministic one */
};

/* Copies one of the items above to host memory after synchronising the stream.
 * bytes must equal the item's size for the current batch and tree. */
int vadusa_debug_read(vadusa_ctx* ctx, int32_t what, void* host_buf, size_t bytes);

/* Test aid for the failure path described under "Conventions": sets the error word a step kernel raises when
 * it gives up at a grid barrier (bf16 contexts; VADUSA_ESTATE for fp32 ones).  No kernel is disturbed: the
 * stream is drained first. */
int vadusa_debug_raise_error(vadusa_ctx* ctx);

/* Copies K (which = 0) or V (1) rows pos0..pos0+npos-1 of a layer and sequence
 * to host as float [npos][d_model] (heads concatenated), after synchronising. */
int vadusa_debug_read_kv(vadusa_ctx* ctx, int32_t layer, int32_t seq, int32_t which,
                         int32_t pos0, int32_t npos, float* host_buf);

/* vadusa_debug_read_kv for callers that cannot allocate device memory or be handed a workspace for this
 * purpose (code between graph captures, tight serving loops, harnesses that forbid hipMalloc): the float rows
 * are staged in a static device array of the library, 1 MiB = 262 144 floats per GPU, held until the process
 * ends, instead of the arena's staging area.  Same arguments, result and errors as vadusa_debug_read_kv;
 * in addition npos * d_model > 262 144 returns VADUSA_ESHAPE (read in several calls).  Calls no allocating
 * routine.  All contexts on one GPU share the array: calls that overlap on one GPU race; serialise them. */
int vadusa_debug_read_kv_static(vadusa_ctx* ctx, int32_t layer, int32_t seq, int32_t which,
                                int32_t pos0, int32_t npos, float* host_buf);

#ifdef __cplusplus
}
#endif
#endif /* VADUSA_H */
