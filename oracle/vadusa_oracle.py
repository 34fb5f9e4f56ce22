"""CPU oracle for the VADUSA speculative decode step.  TEST INFRASTRUCTURE ONLY.

Plain numpy, fp64 arithmetic on the given (fp32 or bf16-rounded) weights.  It is
imported by the tests, by the smoke check and by the benchmark's CPU-baseline
leg; the product path (the HIP library and its Python binding) never touches it
and shares no code with it.

Every function cites the passage of the paper (arXiv 2410.21951) it follows.
Where the paper is silent the reading taken is stated next to the code.

Parity status of the functions below
  * causal_forward           pinned (library transformer layer, closed forms)
  * tree_forward             pinned (brute force against causal_forward)
  * draft_heads / top_k      pinned (closed forms, sort with planted ties)
  * topk_needed / draft_lists / expand_tree / ancestor_mask
                             pinned (hand-drawn trees in tests/golden/tree_cases.json:
                             the full top-2 tree of depth 3 of Fig. 1(c) and a sparse
                             tree, node tokens, depths and mask written out by hand)
  * verify_branch / select   pinned (worked example of Sec. 2.1, Alg. 1 cases)
  * generate at tau = 1      pinned (equals plain greedy decoding, Sec. 2.1 "lossless")
  * generate at tau > 1      replay property only; the exact token stream at
                             tau > 1 is defined by the readings stated here:
                             parity unpinned beyond that property.
  * nucleus / gumbel / perturbed_scores / step(sample=...)
                             pinned (hand-worked nucleus cases, brute-force set
                             definition, draw frequencies against the closed-form
                             probabilities of sampling without replacement, limits
                             that reduce to the deterministic rule)
"""
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np
from scipy.special import erf

LN_EPS = 1e-5


# --------------------------------------------------------------------------
# Model (Sec. 3.1.1: decoder-only transformer, 12 layers / 16 heads / 1024 /
# 4096 in the paper; sizes come from the config).  Readings where the paper
# gives sizes only: pre-LayerNorm blocks, exact (erf) GELU, learned absolute
# positions over the concatenated text+speech sequence, fully causal attention,
# biases on the QKV / output / feed-forward maps, none on the vocabulary map.
# --------------------------------------------------------------------------
class Model:
    def __init__(self, cfg, weights):
        self.cfg = cfg
        self.W = {k: np.asarray(v, dtype=np.float64) for k, v in weights.items()}


def layer_norm(x, g, b):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + LN_EPS) * g + b


def gelu(x):
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax_rows(s):
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def attend(q, K, V, allow, n_heads):
    """Multi-head attention of n queries over T keys.

    q [n, d], K/V [T, d], allow bool [n, T] (True = query may see key).
    Scores are q.k / sqrt(head_dim), softmax over the allowed keys.
    """
    n, d = q.shape
    hd = d // n_heads
    out = np.empty_like(q)
    for h in range(n_heads):
        sl = slice(h * hd, (h + 1) * hd)
        s = q[:, sl] @ K[:, sl].T / np.sqrt(hd)
        s = np.where(allow, s, -np.inf)
        out[:, sl] = softmax_rows(s) @ V[:, sl]
    return out


def block(model, l, x, K_ctx, V_ctx, allow_ctx):
    """One pre-LN decoder block for the rows x.

    K_ctx/V_ctx [Tc, d] are keys/values already known for this layer (may be
    empty); the rows' own keys/values are appended after them, and allow_ctx
    [n, Tc + n] says which of those Tc + n keys each row may see.
    Returns the new x and the rows' own k, v.
    """
    W, nH = model.W, model.cfg.n_heads
    d = model.cfg.d_model
    p = f"L{l}."
    a = layer_norm(x, W[p + "ln1_g"], W[p + "ln1_b"])
    qkv = a @ W[p + "Wqkv"].T + W[p + "bqkv"]
    q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    K_all = np.concatenate([K_ctx, k], axis=0)
    V_all = np.concatenate([V_ctx, v], axis=0)
    o = attend(q, K_all, V_all, allow_ctx, nH)
    x = x + o @ W[p + "Wo"].T + W[p + "bo"]
    a = layer_norm(x, W[p + "ln2_g"], W[p + "ln2_b"])
    hdn = gelu(a @ W[p + "W1"].T + W[p + "b1"])
    x = x + hdn @ W[p + "W2"].T + W[p + "b2"]
    return x, k, v


def base_head(model, x):
    """Final LayerNorm and the vocabulary map: returns (h, logits over V+1 ids)."""
    W = model.W
    h = layer_norm(x, W["lnf_g"], W["lnf_b"])
    return h, h @ W["W_out"].T


def causal_forward(model, text, speech):
    """The definition: full causal forward over text tokens followed by speech
    tokens (Sec. 2.1, prefilling pass over {t_1..t_k}).

    Returns logits [T, V+1], h [T, d] and per-layer K, V [Ly, T, d].
    """
    W, cfg = model.W, model.cfg
    text = np.asarray(text, dtype=np.int64)
    speech = np.asarray(speech, dtype=np.int64)
    T = len(text) + len(speech)
    x = np.concatenate([W["E_text"][text], W["E_speech"][speech]], axis=0) + W["P"][:T]
    causal = np.tril(np.ones((T, T), bool))
    empty = np.zeros((0, cfg.d_model))
    Ks, Vs = [], []
    for l in range(cfg.n_layers):
        x, k, v = block(model, l, x, empty, empty, causal)
        Ks.append(k)
        Vs.append(v)
    h, logits = base_head(model, x)
    return dict(logits=logits, h=h, K=np.stack(Ks), V=np.stack(Vs))


# --------------------------------------------------------------------------
# Draft heads (Sec. 2.1: the i-th draft head predicts the (i+1)-th next token;
# Sec. 3.1.1: each is a residual block with a linear layer and a SiLU, on top
# of the last transformer layer).  Readings: the heads read the same final-
# LayerNorm'd vector as the base head; r = h + SiLU(W1 h + b1); z = W2 r with
# W2 separate per head and without bias.
# --------------------------------------------------------------------------
def draft_heads(model, h):
    W = model.W
    out = []
    for i in range(model.cfg.n_draft_heads):
        r = h + silu(h @ W[f"D{i}.W1"].T + W[f"D{i}.b1"])
        out.append(r @ W[f"D{i}.W2"].T)
    return out


def top_k(z, k):
    """Ids of the k largest logits, descending; equal logits: lower id first (Sec. 2.1)."""
    return np.argsort(-np.asarray(z), kind="stable")[:k].astype(np.int64)


# --------------------------------------------------------------------------
# Decoding state with a KV cache (Sec. 2.2: kv-cache for in-context memory)
# --------------------------------------------------------------------------
@dataclass
class SeqState:
    K: np.ndarray                  # [Ly, capacity, d]
    V: np.ndarray
    L: int                         # committed positions
    root: int                      # base head's next token (t_{k+1,0})
    draft_logits: List[np.ndarray]  # per draft head, logits from the last accepted position
    root_logits: Optional[np.ndarray] = None   # the base-head row the root was taken from
    finished: bool = False
    emitted: List[int] = field(default_factory=list)


def prefill(model, text, prompt):
    """Prefilling pass (Sec. 2.1, Fig. 1a): the base head gives the first next
    token, the draft heads give the logits their top-k candidates come from."""
    cfg = model.cfg
    f = causal_forward(model, text, prompt)
    L = f["logits"].shape[0]
    K = np.zeros((cfg.n_layers, cfg.max_positions, cfg.d_model))
    V = np.zeros_like(K)
    K[:, :L], V[:, :L] = f["K"], f["V"]
    root = int(top_k(f["logits"][-1], 1)[0])
    return SeqState(K=K, V=V, L=L, root=root, draft_logits=draft_heads(model, f["h"][-1]),
                    root_logits=f["logits"][-1])


def topk_needed(depth, rank, n_heads):
    """K_i of Sec. 2.4's sparse tree: how many of draft head i's top entries the
    tree uses = 1 + the largest rank among the nodes at depth i (0 if none)."""
    need = [0] * n_heads
    for dep, r in zip(np.asarray(depth)[1:], np.asarray(rank)[1:]):
        need[int(dep) - 1] = max(need[int(dep) - 1], int(r) + 1)
    return need


def draft_lists(model, st, tree):
    """Per-head top-K_i candidate lists, K_i = what the tree uses of head i."""
    need = topk_needed(tree.depth, tree.rank, model.cfg.n_draft_heads)
    return [top_k(z, k) for z, k in zip(st.draft_logits, need)]


def expand_tree(root, lists, tree):
    """Node tokens (Sec. 2.1: the root is the first next token, depth D is filled
    from the D-th draft head's top-k; Sec. 2.4: only the sparse subset is kept)."""
    tok = np.empty(tree.n_nodes, np.int64)
    tok[0] = root
    for n in range(1, tree.n_nodes):
        tok[n] = lists[tree.depth[n] - 1][tree.rank[n]]
    return tok


def ancestor_mask(parent):
    """Tree attention mask (Sec. 2.1, Fig. 1c): bool [M, M], entry (n, m) is True
    iff m is n itself or lies on the way from the root to n."""
    parent = np.asarray(parent)
    M = len(parent)
    A = np.zeros((M, M), bool)
    for n in range(M):
        m = n
        while m >= 0:
            A[n, m] = True
            m = int(parent[m])
    return A


def tree_forward(model, st, tok, tree):
    """One forward of all tree nodes (Sec. 2.1, tree attention): a node sees the
    committed prefix and, inside the tree, itself and its ancestors only.
    Returns logits [M, V+1], h [M, d], k, v [Ly, M, d]."""
    W, cfg = model.W, model.cfg
    M, L = tree.n_nodes, st.L
    x = W["E_speech"][tok] + W["P"][L + tree.depth]
    allow = np.concatenate([np.ones((M, L), bool), ancestor_mask(tree.parent)], axis=1)
    ks, vs = [], []
    for l in range(cfg.n_layers):
        x, k, v = block(model, l, x, st.K[l, :L], st.V[l, :L], allow)
        ks.append(k)
        vs.append(v)
    h, logits = base_head(model, x)
    return logits, h, np.stack(ks), np.stack(vs)


# --------------------------------------------------------------------------
# Verification with tolerance (Algorithm 1) and choice among branches (Sec. 2.3)
# Reading of tau: deterministic; the base head's tau "correct tokens" at a
# position are its tau highest-logit ids (ties: lower id first).  tau = 1 is the
# vanilla rule of Sec. 2.1.
# --------------------------------------------------------------------------
def verify_branch(logits_branch, cand, tau):
    """Algorithm 1 for one branch.  cand = (c_0..c_k), logits_branch[i] = the base
    head's logits at c_i.  Returns k*: the accepted sequence is (c_0..c_{k*}).

    c_{i+1} is tolerated at position i iff it is one of the tau "correct" ids of
    logits_branch[i]; the accepted sequence is the longest prefix all of whose
    steps are tolerated, so k* = the number of leading tolerated steps."""
    cand = np.asarray(cand)
    k = len(cand) - 1
    tolerated = np.array([cand[i + 1] in top_k(logits_branch[i], tau) for i in range(k)], dtype=bool)
    return int(np.cumprod(tolerated).sum())


def branches(tree):
    """Root-to-leaf node-index paths, left to right."""
    M = tree.n_nodes
    has_child = np.zeros(M, bool)
    has_child[tree.parent[1:]] = True
    out = []
    for n in range(M):
        if not has_child[n]:
            path = []
            m = n
            while m >= 0:
                path.append(m)
                m = int(tree.parent[m])
            out.append(path[::-1])
    out.sort(key=lambda p: tree.paths[p[-1]])
    return out


def select_path(tree, tok, logits, tau):
    """Run Algorithm 1 on every branch, keep the longest accepted sequence; among
    equally long ones the leftmost (Sec. 2.3).  Returns the node-index path."""
    best = None
    for br in branches(tree):
        k_star = verify_branch(logits[br], tok[br], tau)
        acc = br[:k_star + 1]
        if best is None or len(acc) > len(best) or (
                len(acc) == len(best) and tree.paths[acc[-1]] < tree.paths[best[-1]]):
            best = acc
    return best


# --------------------------------------------------------------------------
# Stochastic verification: Algorithm 1 as printed draws, at every position i of
# a branch, tau tokens from the nucleus of the temperature-scaled distribution
# of L(i) and accepts the next candidate iff it is among the draws (Sec. 3.1.2:
# nucleus sampling with a temperature).
# Readings where the paper is silent: the tau draws are without replacement; a
# nucleus smaller than tau is widened to the tau most probable tokens so that
# tau draws exist; the continuation token after the accepted sequence is the
# first draw at its last position.
# The draws come from uniforms u in (0, 1) handed in by the caller, one per
# (position, token): with g = -log(-log u), ordering the kept tokens by
# s + g (s = logit / temperature) lists them in the order successive draws
# without replacement from softmax(s) would produce them (the "Gumbel top-k"
# identity), so "among the tau draws" is "among the tau largest s + g".
# --------------------------------------------------------------------------
def nucleus(s, top_p, min_keep=1):
    """Which tokens nucleus sampling keeps (bool per token) for scores s.

    Token v is kept iff the tokens with a strictly larger score hold less than
    top_p of softmax(s)'s probability, i.e. the most probable tokens are taken
    until their mass reaches top_p; tokens of equal score are kept or dropped
    together.  A token with fewer than min_keep tokens strictly above it is kept
    in any case.  top_p >= 1 keeps every token.
    """
    s = np.asarray(s, dtype=np.float64)
    if top_p >= 1.0:
        return np.ones(s.shape, bool)
    p = softmax_rows(s)
    order = np.argsort(-s, kind="stable")
    ss, ps = s[order], p[order]
    before_me = np.concatenate([[0.0], np.cumsum(ps)[:-1]])     # mass of the tokens sorted ahead
    first_equal = np.searchsorted(-ss, -ss, side="left")          # start of each run of equal scores
    mass_above = before_me[first_equal]
    keep_sorted = (mass_above < top_p) | (first_equal < min_keep)
    keep = np.empty(s.shape, bool)
    keep[order] = keep_sorted
    return keep


def gumbel(u):
    """Standard Gumbel variate from a uniform u in (0, 1)."""
    with np.errstate(divide="ignore"):
        return -np.log(-np.log(np.asarray(u, dtype=np.float64)))


def perturbed_scores(z, u, temperature, top_p, tau):
    """Row(s) of s + g over the kept tokens, -inf elsewhere; z, u [..., V+1].
    The tau largest entries of a row are that position's tau draws, in order."""
    z = np.asarray(z, dtype=np.float64)
    s = z / temperature
    g = gumbel(u)
    flat_s = s.reshape(-1, s.shape[-1])
    keep = np.stack([nucleus(r, top_p, min_keep=tau) for r in flat_s]).reshape(s.shape)
    return np.where(keep, s + g, -np.inf)


def step(model, st, tree, tau, draft_override=None, ignore_eos=False, sample=None):
    """One speculative step (Sec. 2.1 decoding pass + Sec. 2.3): expand, verify the
    whole tree in one forward, accept, commit the accepted path's keys/values and
    continue from the last accepted node's prediction.

    draft_override: optional per-head id lists used in place of the draft heads'
    own top-k (test hook to plant longer accepted paths).
    sample: None for the deterministic rule, or (temperature, top_p, u) with
    uniforms u [M, V+1] for the stochastic rule of Algorithm 1: the same choice
    among branches, taken on the perturbed scores instead of the logits.
    Returns a dict with everything a lockstep comparison needs.
    """
    cfg = model.cfg
    if st.finished:
        return dict(accepted=[], path=[], tok=None, logits=None, lists=None)
    lists = draft_lists(model, st, tree) if draft_override is None else \
        [np.asarray(a, np.int64) for a in draft_override]
    tok = expand_tree(st.root, lists, tree)
    logits, h, k, v = tree_forward(model, st, tok, tree)
    scores = logits if sample is None else perturbed_scores(logits, sample[2], sample[0], sample[1], tau)
    path = select_path(tree, tok, scores, tau)
    accepted = [int(tok[n]) for n in path]
    # EOS (id V): paper silent; reading: the path is cut after the first EOS and
    # the sequence stops, unless the fixed-length benchmarks ask to ignore it.
    if not ignore_eos and cfg.speech_vocab in accepted:
        cut = accepted.index(cfg.speech_vocab) + 1
        accepted, path = accepted[:cut], path[:cut]
        st.finished = True
    n = len(path)
    st.K[:, st.L:st.L + n] = k[:, path]
    st.V[:, st.L:st.L + n] = v[:, path]
    st.L += n
    last = path[-1]
    st.root = int(top_k(scores[last], 1)[0])          # prediction of the last accepted token (first draw)
    st.root_logits = scores[last]
    st.draft_logits = draft_heads(model, h[last])     # new drafts from that position
    st.emitted += accepted
    return dict(accepted=accepted, path=path, tok=tok, logits=logits, scores=scores, lists=lists,
                h=h, next_root=st.root)


def generate(model, text, prompt, tree, tau, n_tokens, ignore_eos=False):
    """Prefill then speculative steps until n_tokens are emitted (or EOS)."""
    st = prefill(model, text, prompt)
    lens = []
    while len(st.emitted) < n_tokens and not st.finished:
        lens.append(len(step(model, st, tree, tau, ignore_eos=ignore_eos)["accepted"]))
    return st.emitted[:n_tokens], lens


def greedy_ar(model, text, prompt, n_tokens, ignore_eos=False):
    """Plain auto-regressive greedy decoding, one full causal forward per token:
    the baseline the vanilla (tau = 1) verification must reproduce (Sec. 2.1)."""
    speech = list(np.asarray(prompt).tolist())
    out = []
    for _ in range(n_tokens):
        t = int(top_k(causal_forward(model, text, speech)["logits"][-1], 1)[0])
        out.append(t)
        speech.append(t)
        if t == model.cfg.speech_vocab and not ignore_eos:
            break
    return out
