"""Pins for the oracle's transformer forward, KV cache, tree attention and draft heads.

None of these compares the oracle with itself through the same code path: the
base forward is pinned to torch's library transformer layer and to closed forms,
the cached / tree forward to brute-force causal forwards.
"""
import numpy as np
import pytest
import torch

from oracle import vadusa_oracle as O
from synth import make_tree, chain_tree, full_tree, make_weights
from helpers import SMALL, small_model

RTOL = 1e-9


def rel(a, b):
    return np.linalg.norm(np.asarray(a) - np.asarray(b)) / max(np.linalg.norm(b), 1e-300)


def _torch_stack(model):
    """The same network assembled from torch.nn library modules (fp64)."""
    cfg, W = model.cfg, model.W
    layers = []
    for l in range(cfg.n_layers):
        lay = torch.nn.TransformerEncoderLayer(
            d_model=cfg.d_model, nhead=cfg.n_heads, dim_feedforward=cfg.d_ffn, dropout=0.0,
            activation="gelu", batch_first=True, norm_first=True, layer_norm_eps=1e-5).double()
        p = f"L{l}."
        sd = {
            "self_attn.in_proj_weight": W[p + "Wqkv"], "self_attn.in_proj_bias": W[p + "bqkv"],
            "self_attn.out_proj.weight": W[p + "Wo"], "self_attn.out_proj.bias": W[p + "bo"],
            "linear1.weight": W[p + "W1"], "linear1.bias": W[p + "b1"],
            "linear2.weight": W[p + "W2"], "linear2.bias": W[p + "b2"],
            "norm1.weight": W[p + "ln1_g"], "norm1.bias": W[p + "ln1_b"],
            "norm2.weight": W[p + "ln2_g"], "norm2.bias": W[p + "ln2_b"],
        }
        lay.load_state_dict({k: torch.from_numpy(np.array(v)) for k, v in sd.items()})
        lay.train()   # dropout is 0; train mode keeps torch on its composed (not fused) path
        layers.append(lay)
    return layers


def test_causal_forward_matches_torch_library_layers():
    model = small_model()
    cfg, W = model.cfg, model.W
    rng = np.random.default_rng(0)
    text = rng.integers(0, cfg.text_vocab, 9)
    speech = rng.integers(0, cfg.speech_vocab + 1, 14)
    got = O.causal_forward(model, text, speech)
    T = 23
    x = torch.from_numpy(np.concatenate([W["E_text"][text], W["E_speech"][speech]]) + W["P"][:T])[None]
    mask = torch.triu(torch.full((T, T), float("-inf"), dtype=torch.float64), diagonal=1)
    with torch.no_grad():
        for lay in _torch_stack(model):
            x = lay(x, src_mask=mask)
        h = torch.nn.functional.layer_norm(x, (cfg.d_model,), torch.from_numpy(W["lnf_g"]),
                                           torch.from_numpy(W["lnf_b"]), 1e-5)
        logits = torch.nn.functional.linear(h, torch.from_numpy(W["W_out"]))
    assert rel(got["h"], h[0].numpy()) < RTOL
    assert rel(got["logits"], logits[0].numpy()) < RTOL


def test_zero_layers_closed_form():
    """All block weights zero => blocks are identities => logits = W_out LN(E[tok] + P[pos])."""
    model = small_model()
    for k in model.W:
        if k.startswith("L") and not k.endswith(("_g",)):
            model.W[k] = np.zeros_like(model.W[k])
    W = model.W
    text, speech = np.array([1, 2, 3]), np.array([5, 6, 40])
    got = O.causal_forward(model, text, speech)["logits"]
    x = np.concatenate([W["E_text"][text], W["E_speech"][speech]]) + W["P"][:6]
    mu = x.mean(1, keepdims=True)
    sd = np.sqrt(x.var(1, keepdims=True) + 1e-5)
    want = ((x - mu) / sd * W["lnf_g"] + W["lnf_b"]) @ W["W_out"].T
    assert rel(got, want) < 1e-12


def test_position_and_table_choice_matter():
    """A dropped position term or a swapped embedding table must change the result."""
    model = small_model()
    a = O.causal_forward(model, [1, 2], [3, 4])["logits"]
    b = O.causal_forward(model, [2, 1], [3, 4])["logits"]
    c = O.causal_forward(model, [1], [2, 3, 4])["logits"]
    assert rel(a[-1], b[-1]) > 1e-3 and rel(a[-1], c[-1]) > 1e-3
    # causality: changing a later token leaves earlier rows untouched
    d = O.causal_forward(model, [1, 2], [3, 9])["logits"]
    assert np.array_equal(a[:3], d[:3]) and rel(a[3], d[3]) > 1e-3


def test_kv_cached_token_by_token_equals_full_causal():
    model = small_model()
    cfg = model.cfg
    rng = np.random.default_rng(1)
    text = rng.integers(0, cfg.text_vocab, 7)
    speech = rng.integers(0, cfg.speech_vocab, 20)
    full = O.causal_forward(model, text, speech)
    st = O.prefill(model, text, speech[:5])
    one = chain_tree(1)
    for j in range(5, 20):
        logits, h, k, v = O.tree_forward(model, st, np.array([speech[j]]), one)
        assert rel(logits[0], full["logits"][7 + j]) < RTOL
        st.K[:, st.L], st.V[:, st.L] = k[:, 0], v[:, 0]
        st.L += 1
    assert rel(st.K[:, :27], full["K"]) < RTOL and rel(st.V[:, :27], full["V"]) < RTOL


@pytest.mark.parametrize("tree", [make_tree(16, (4, 2, 2)), full_tree((2, 2, 2)), chain_tree(4),
                                  make_tree(24, (5, 5, 5))])
def test_tree_forward_equals_brute_force_per_path(tree):
    """Tree attention verifies the whole tree in one pass (Sec. 2.1): every node's
    logits equal a separate causal forward over prefix + root-to-node path."""
    model = small_model()
    cfg = model.cfg
    rng = np.random.default_rng(2)
    text = rng.integers(0, cfg.text_vocab, 6)
    prompt = rng.integers(0, cfg.speech_vocab, 11)
    st = O.prefill(model, text, prompt)
    tok = rng.integers(0, cfg.speech_vocab + 1, tree.n_nodes)
    logits, h, k, v = O.tree_forward(model, st, tok, tree)
    for n in range(tree.n_nodes):
        path, m = [], n
        while m >= 0:
            path.append(m)
            m = int(tree.parent[m])
        path = path[::-1]
        ref = O.causal_forward(model, text, np.concatenate([prompt, tok[path]]))
        assert rel(logits[n], ref["logits"][-1]) < RTOL
        assert rel(k[:, n], ref["K"][:, -1]) < RTOL and rel(v[:, n], ref["V"][:, -1]) < RTOL


@pytest.mark.parametrize("tree", [make_tree(16, (4, 2, 2)), make_tree(64, (10,) * 4),
                                  make_tree(128, (10,) * 5), full_tree((3, 2))])
def test_tree_mask_invariants(tree):
    A = O.ancestor_mask(tree.parent)
    M = tree.n_nodes
    assert A.diagonal().all() and A[:, 0].all()
    assert not np.triu(A, 1).any()                      # lower triangular in canonical order
    for n in range(1, M):
        p = tree.parent[n]
        assert p < n and tree.depth[n] == tree.depth[p] + 1
        assert np.array_equal(A[n] & ~np.eye(M, dtype=bool)[n], A[p])   # ancestor-closed
        assert A[n].sum() == tree.depth[n] + 1
    order = [(len(p), p) for p in tree.paths]
    assert order == sorted(order)


def test_draft_head_closed_forms():
    model = small_model()
    cfg, W = model.cfg, model.W
    h = np.random.default_rng(3).standard_normal(cfg.d_model)
    # W1 = 0, b1 = 0 => SiLU(0) = 0 => z = W2 h
    W["D0.W1"] = np.zeros_like(W["D0.W1"])
    W["D0.b1"] = np.zeros_like(W["D0.b1"])
    # head 1: additionally W2 = W_out => reproduces the base head's logits
    W["D1.W1"] = np.zeros_like(W["D1.W1"])
    W["D1.b1"] = np.zeros_like(W["D1.b1"])
    W["D1.W2"] = W["W_out"].copy()
    z = O.draft_heads(model, h)
    assert rel(z[0], W["D0.W2"] @ h) < 1e-12
    assert rel(z[1], W["W_out"] @ h) < 1e-12
    # head 2 against the formula written with scalar loops
    a = W["D2.W1"] @ h + W["D2.b1"]
    r = np.array([h[j] + a[j] / (1.0 + np.exp(-a[j])) for j in range(cfg.d_model)])
    want = np.array([sum(W["D2.W2"][v, j] * r[j] for j in range(cfg.d_model))
                     for v in range(cfg.n_logits)])
    assert rel(z[2], want) < 1e-12


def test_top_k_against_full_sort_with_planted_ties():
    rng = np.random.default_rng(4)
    for _ in range(50):
        z = rng.integers(0, 6, 30).astype(float)      # many ties
        k = int(rng.integers(1, 12))
        want = sorted(range(30), key=lambda v: (-z[v], v))[:k]
        assert O.top_k(z, k).tolist() == want
    assert O.top_k(np.array([1.0, 3.0, 3.0, 2.0]), 3).tolist() == [1, 2, 3]


def test_gelu_silu_values():
    # textbook values: GELU(x) = x Phi(x), SiLU(x) = x sigmoid(x)
    assert abs(O.gelu(np.array(1.0)) - 0.8413447460685429) < 1e-12
    assert abs(O.gelu(np.array(-2.0)) - (-2.0 * 0.022750131948179195)) < 1e-12
    assert abs(O.silu(np.array(1.0)) - 0.7310585786300049) < 1e-12
    assert abs(O.silu(np.array(-3.0)) - (-3.0 * 0.04742587317756678)) < 1e-12
