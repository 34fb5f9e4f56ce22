"""GPU parity: the HIP library against the CPU oracle, through the C ABI.

Tolerances: logits relative L2 <= 1e-4 (fp32 model) / 1e-2 (bf16 model); token
decisions exact wherever the oracle's deciding margin exceeds 1e-2 (see
tests/parity.py for the protocol).
"""
import dataclasses

import numpy as np
import pytest

from oracle import vadusa_oracle as O
from synth import (ModelConfig, PRESETS, make_weights, make_tokens, make_tree, chain_tree,
                   full_tree)
from helpers import planted_lists

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _lock(*a, **k):
    from parity import Lockstep
    return Lockstep(*a, **k)


# Weight scale of the small models.  The 1e-2 decision margin is an absolute logit
# gap stated for the workload's logit scale (std ~0.64 = 0.02 * sqrt(1024)); the small
# bf16 models are scaled to the same logit std (0.05 * sqrt(128) ~ 0.57) so that the
# same absolute margin means the same thing.
STD = {"fp32": 0.08, "bf16": 0.05}


def small_cfg(dtype, layers=2, d=128, heads=3, V=300, maxpos=256):
    return ModelConfig(n_layers=layers, d_model=d, n_heads=d // 64, head_dim=64, d_ffn=4 * d,
                       speech_vocab=V, text_vocab=50, n_draft_heads=heads, max_positions=maxpos,
                       dtype=dtype)


def rand_tokens(cfg, rng, B, tl, pl):
    text = [rng.integers(0, cfg.text_vocab, int(rng.integers(tl[0], tl[1] + 1))).astype(np.int32) for _ in range(B)]
    prompt = [rng.integers(0, cfg.speech_vocab, int(rng.integers(pl[0], pl[1] + 1))).astype(np.int32) for _ in range(B)]
    return text, prompt


@pytest.mark.parametrize("tau", [1, 3])
def test_tiny_fp32_full_generation(tau):
    """Configuration 1 end to end: 32 text + 75 prompt tokens, 150 generated, 16-node tree."""
    wl = PRESETS["tiny"]
    _say(f"tiny fp32 tau={tau}")
    W = make_weights(wl.model, wl.seed)
    text, prompt = make_tokens(wl)
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    ls = _lock(wl.model, W, text, prompt, wl.tree_nodes)
    while len(ls.sts[0].emitted) < wl.n_generate:
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"  steps {s.steps} compared {s.compared} ties root/list/edge {s.tie_root}/{s.tie_list}/{s.tie_edge} "
         f"logit err {s.max_logit_err:.2e} kv err {s.max_kv_err:.2e}")
    assert s.compared >= 0.8 * s.steps
    assert s.tie_edge + s.tie_root <= 0.05 * s.steps, "more than 5 % of the steps lost to decisions inside the margin"
    assert s.max_logit_err < 1e-4


@pytest.mark.parametrize("dtype,tau", [("fp32", 1), ("fp32", 2), ("bf16", 1), ("bf16", 3)])
def test_planted_drafts_long_paths(dtype, tau):
    """Acceptance dial: the true continuation planted among the candidates gives
    accepted paths of every length, exercising acceptance, compaction and the
    continuation from the last accepted node."""
    cfg = small_cfg(dtype)
    _say(f"planted drafts {dtype} tau={tau}")
    W = make_weights(cfg, 5, std=STD[dtype], ln_jitter=0.1)
    rng = np.random.default_rng(21)
    text, prompt = rand_tokens(cfg, rng, 1, (9, 9), (21, 21))
    tree = make_tree(24, (3, 3, 2), alpha0=0.9, decay=1.0)
    assert tree.max_depth == 3
    model = O.Model(cfg, W)
    greedy = O.generate(model, text[0], prompt[0], chain_tree(1), 1, 70, ignore_eos=True)[0]
    ls = _lock(cfg, W, text, prompt, 24)
    while len(ls.sts[0].emitted) < 48:
        st = ls.sts[0]
        n = len(st.emitted)
        on = st.emitted == greedy[:n] and st.root == greedy[n]
        fut = greedy[n + 1:n + 1 + cfg.n_draft_heads] if on else []
        lists = planted_lists(fut, tree, cfg.n_draft_heads, cfg.n_logits, rng, p_hit=0.8)
        ls.step(tree, tau, override=[lists])
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"  accepted lengths {np.bincount(s.accepted_hist).tolist()} ties {s.tie_root}/{s.tie_list}/{s.tie_edge} "
         f"logit err {s.max_logit_err:.2e}")
    assert max(s.accepted_hist) == cfg.n_draft_heads + 1 and min(s.accepted_hist) == 1


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_ragged_batch_multi_chunk_prefill(dtype):
    """Three sequences of different lengths; prompts longer than one prefill chunk
    (ragged first chunk), different trees from step to step."""
    cfg = small_cfg(dtype, maxpos=320)
    _say(f"ragged batch {dtype}")
    W = make_weights(cfg, 6, std=STD[dtype], ln_jitter=0.1)
    rng = np.random.default_rng(22)
    text, prompt = rand_tokens(cfg, rng, 3, (3, 30), (17, 120))
    ls = _lock(cfg, W, text, prompt, 32)
    trees = [make_tree(32, (6, 4, 3)), chain_tree(4), full_tree((3, 2)), make_tree(17, (4, 2, 2)), chain_tree(1)]
    for i in range(15):
        ls.step(trees[i % len(trees)], 1 + i % 3)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} ties {s.tie_root}/{s.tie_list}/{s.tie_edge} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 10


def test_eos_cuts_path_and_finishes():
    cfg = small_cfg("fp32")
    W = make_weights(cfg, 8, std=0.08)
    rng = np.random.default_rng(23)
    text, prompt = rand_tokens(cfg, rng, 2, (5, 5), (12, 12))
    tree = chain_tree(4)
    ls = _lock(cfg, W, text, prompt, 8, ignore_eos=False)
    eos = cfg.speech_vocab
    # tau = V+1 accepts every edge; sequence 0 gets EOS as its second draft
    lists = [[[7], [eos], [9]], [[1], [2], [3]]]
    r = ls.step(tree, cfg.n_logits, override=lists)
    assert r[0]["accepted"][-1] == eos and len(r[0]["accepted"]) == 3 and len(r[1]["accepted"]) == 4
    assert ls.sts[0].finished and not ls.sts[1].finished
    r = ls.step(tree, cfg.n_logits, override=lists)
    assert r[0]["accepted"] == []
    out = ls.dev.step(__import__("paper_2410_21951_amd").TreeArrays(tree.parent, tree.rank), 1)
    assert out[0] == [] and len(out[1]) >= 1


@pytest.fixture(scope="module")
def valle():
    wl = PRESETS["valle_b1"]
    _say("generating 12-layer d=1024 weights")
    return wl, make_weights(wl.model, wl.seed)


@pytest.mark.parametrize("extra", [0, 500])
def test_valle_b1_sampled_steps(valle, extra):
    """Configuration 2 at full size (12 layers, d=1024, bf16, 64-node tree): steps at
    the start of generation (L = 289) and deep into it (L = 789)."""
    wl, W = valle
    text, prompt = make_tokens(wl)
    rng = np.random.default_rng(24)
    prompt = [np.concatenate([prompt[0], rng.integers(0, wl.model.speech_vocab, extra).astype(np.int32)])]
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    _say(f"valle_b1 L0={len(text[0]) + len(prompt[0])}")
    ls = _lock(wl.model, W, text, prompt, wl.tree_nodes)
    for i, tau in enumerate((1, 2, 4, 8)):
        ls.step(tree, tau)
        _say(f"  step {i} tau {tau} logit err {ls.stats.max_logit_err:.3e}")
    ls.check_kv(layers=[0, 5, 11])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} ties {s.tie_root}/{s.tie_list}/{s.tie_edge} "
         f"logit err {s.max_logit_err:.2e} h err {s.max_h_err:.2e} kv err {s.max_kv_err:.2e}")
    assert s.compared >= 3


def test_longform_shape_128_nodes_5_heads():
    """Configuration 4's shape (5 draft heads, 128-node tree) on a 3-layer d=1024 model
    with a prompt spanning several prefill chunks."""
    m = PRESETS["longform_b1"].model
    cfg = dataclasses.replace(m, n_layers=3, max_positions=1024)
    W = make_weights(cfg, 9)
    rng = np.random.default_rng(25)
    text, prompt = rand_tokens(cfg, rng, 1, (64, 64), (400, 400))
    tree = make_tree(128, (10,) * 5)
    ls = _lock(cfg, W, text, prompt, 128)
    for tau in (1, 4, 4):
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 2])
    s = ls.stats
    _say(f"longform shape: compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 2


def test_throughput_shape_batch():
    """Configuration 5's shape (many sequences, 32-node trees) reduced to 8 sequences
    and 2 layers of the d=1024 model."""
    m = PRESETS["throughput_b64"].model
    cfg = dataclasses.replace(m, n_layers=2, max_positions=400)
    W = make_weights(cfg, 10)
    rng = np.random.default_rng(126)
    text, prompt = rand_tokens(cfg, rng, 8, (64, 64), (225, 225))
    tree = make_tree(32, (10,) * 4)
    ls = _lock(cfg, W, text, prompt, 32)
    for tau in (1, 8):
        ls.step(tree, tau)
    s = ls.stats
    _say(f"throughput shape: compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 1


def test_longform_b1_full_size():
    """Configuration 4 at full size (12 layers, 5 draft heads, 128-node tree), at the start of
    generation (L = 814) in lockstep and deep into it (L = 2914, cache past 3000 rows)
    on one verification."""
    from parity import sampled_check
    wl = PRESETS["longform_b1"]
    _say("generating longform_b1 weights")
    W = make_weights(wl.model, wl.seed)
    text, prompt = make_tokens(wl)
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    ls = _lock(wl.model, W, text, prompt, wl.tree_nodes)
    for tau in (1, 4):
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 11])
    s = ls.stats
    _say(f"longform_b1 L0={len(text[0]) + len(prompt[0])}: compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 1
    ls.dev.close()
    rng = np.random.default_rng(27)
    deep = [np.concatenate([prompt[0], rng.integers(0, wl.model.speech_vocab, 2100).astype(np.int32)])]
    n, skipped, err = sampled_check(wl.model, W, text, deep, tree, 4, [0], kv_layers=(0, 11))
    _say(f"longform_b1 L0={len(text[0]) + len(deep[0])}: compared {n} skipped {skipped} logit err {err:.2e}")
    assert n + skipped == 1


def test_hubert_b16_full_size():
    """Configuration 3 at full size: 16 ragged sequences, vocabulary 2049, tau = 3; the oracle
    follows four of them."""
    from parity import sampled_check
    wl = PRESETS["hubert_b16"]
    _say("generating hubert_b16 weights")
    W = make_weights(wl.model, wl.seed)
    text, prompt = make_tokens(wl)
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    n, skipped, err = sampled_check(wl.model, W, text, prompt, tree, 3, [0, 5, 10, 15], kv_layers=(0, 11))
    _say(f"hubert_b16: compared {n} skipped {skipped} logit err {err:.2e}")
    assert n >= 3


def test_throughput_b64_full_size():
    """Configuration 5 at full size: 64 sequences, 32-node trees, cache for 1200 positions per
    sequence; the oracle follows four of them."""
    from parity import sampled_check
    wl = PRESETS["throughput_b64"]
    _say("generating throughput_b64 weights")
    W = make_weights(wl.model, wl.seed)
    text, prompt = make_tokens(wl)
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    n, skipped, err = sampled_check(wl.model, W, text, prompt, tree, 8, [0, 21, 42, 63], kv_layers=(0, 11))
    _say(f"throughput_b64: compared {n} skipped {skipped} logit err {err:.2e}")
    assert n >= 3


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_single_node_tree_is_plain_ar(dtype):
    """A tree of the root alone: every step commits exactly one token, and the stream equals
    the oracle's plain greedy auto-regressive decoding (the baseline of the paper's speedup)."""
    cfg = small_cfg(dtype)
    W = make_weights(cfg, 31, std=STD[dtype])
    rng = np.random.default_rng(32)
    text, prompt = rand_tokens(cfg, rng, 2, (4, 9), (17, 30))
    tree = chain_tree(1)
    ls = _lock(cfg, W, text, prompt, 8)
    for _ in range(12):
        r = ls.step(tree, 1)
        if r is not None:
            assert all(len(x["accepted"]) == 1 for x in r)
    s = ls.stats
    _say(f"single-node tree {dtype}: compared {s.compared}/{s.steps} ties {s.tie_root} logit err {s.max_logit_err:.2e}")
    if s.tie_root == 0:
        model = O.Model(cfg, W)
        for b in range(2):
            assert ls.sts[b].emitted == O.greedy_ar(model, text[b], prompt[b], len(ls.sts[b].emitted), ignore_eos=True)
    assert s.compared >= 8


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_degenerate_lengths(dtype):
    """Sequences at the edge of what the boundary accepts: no text at all with a one-token
    prompt, text only (the first root is predicted from a text position), next to an ordinary
    one; a sequence with neither text nor prompt is refused."""
    from paper_2410_21951_amd import VadusaError
    cfg = small_cfg(dtype)
    W = make_weights(cfg, 51, std=STD[dtype])
    rng = np.random.default_rng(52)
    text = [np.zeros(0, np.int32), rng.integers(0, cfg.text_vocab, 3).astype(np.int32),
            rng.integers(0, cfg.text_vocab, 5).astype(np.int32)]
    prompt = [rng.integers(0, cfg.speech_vocab, 1).astype(np.int32), np.zeros(0, np.int32),
              rng.integers(0, cfg.speech_vocab, 17).astype(np.int32)]
    tree = make_tree(16, (4, 2, 2))
    ls = _lock(cfg, W, text, prompt, 16)
    for tau in (1, 3, 2):
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"degenerate lengths {dtype}: compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 2
    with pytest.raises(VadusaError) as e:
        ls.dev.prefill([np.zeros(0, np.int32)] * 3, [np.zeros(0, np.int32)] * 3)
    assert e.value.code == -1


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_maximum_heads_ranks_and_path_length(dtype):
    """The limits of the boundary at once: 8 draft heads, candidates of rank 15 (the last entry
    of a 16-wide list), and tau above the vocabulary size, which accepts every edge, so every
    step commits the deepest leftmost path of 9 nodes and compacts 9 cache rows."""
    from synth.trees import tree_from_paths
    cfg = small_cfg(dtype, heads=8)
    W = make_weights(cfg, 61, std=STD[dtype])
    rng = np.random.default_rng(62)
    text, prompt = rand_tokens(cfg, rng, 2, (3, 6), (20, 33))
    paths = [tuple([0] * d) for d in range(9)] + [(15,), (0, 15), (15, 0), (15, 15), (7,), (0, 0, 15)]
    paths = sorted(set(paths), key=lambda p: (len(p), p))
    tree = tree_from_paths(paths)
    ls = _lock(cfg, W, text, prompt, len(paths))
    for _ in range(3):
        r = ls.step(tree, cfg.n_logits + 1)
        if r is not None:
            assert all(len(x["accepted"]) == 9 for x in r)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"max heads/ranks {dtype}: compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 2


def test_smallest_width_bf16():
    """d = 64 (one head): a linear map has two k-steps, so two of the four waves of a workgroup
    have none and only merge the LayerNorm statistics of their rows."""
    cfg = ModelConfig(n_layers=2, d_model=64, n_heads=1, head_dim=64, d_ffn=128, speech_vocab=70, text_vocab=20,
                      n_draft_heads=2, max_positions=64, dtype="bf16")
    W = make_weights(cfg, 71, std=0.08)
    rng = np.random.default_rng(72)
    text, prompt = rand_tokens(cfg, rng, 2, (2, 4), (5, 12))
    tree = make_tree(8, (3, 2))
    ls = _lock(cfg, W, text, prompt, 8)
    for tau in (1, 3, 2):
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"d=64 bf16: compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 2


SAMPLING_MIX = ((1, 1.0, 1.0), (4, 0.9, 0.9), (32, 1.0, 0.6), (100, 0.9, 1.0), (8, 0.5, 0.05), (2, 1.0, 0.95))


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_stochastic_rule_small_models(dtype):
    """Algorithm 1 with sampling (temperature, nucleus, tau draws from the caller's uniforms):
    every temperature / top_p / tau regime, batch of two, paths of several lengths."""
    from synth import make_uniforms
    cfg = small_cfg(dtype)
    _say(f"stochastic rule {dtype}")
    W = make_weights(cfg, 15, std=STD[dtype], ln_jitter=0.1)
    rng = np.random.default_rng(41)
    text, prompt = rand_tokens(cfg, rng, 2, (5, 9), (17, 30))
    tree = make_tree(24, (3, 3, 2), alpha0=0.9, decay=1.0)
    ls = _lock(cfg, W, text, prompt, 24)
    for i in range(12):
        tau, T, top_p = SAMPLING_MIX[i % len(SAMPLING_MIX)]
        ls.step(tree, tau, sample=(T, top_p, make_uniforms(77, i, 2, tree.n_nodes, cfg.n_logits)))
    ls.step(tree, 2)                      # a deterministic step after stochastic ones
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} accepted lengths {np.bincount(s.accepted_hist).tolist()} "
         f"ties {s.tie_root}/{s.tie_list}/{s.tie_edge} logit err {s.max_logit_err:.2e} score err {s.max_score_err:.2e} "
         f"mean kept {[round(x) for x in s.nucleus_sizes[:12:2]]}")
    assert s.compared >= 10
    assert max(s.accepted_hist) >= 3 and min(s.accepted_hist) == 1
    assert min(s.nucleus_sizes) < 16 and max(s.nucleus_sizes) == cfg.n_logits


def test_valle_b1_stochastic_steps(valle):
    """The stochastic rule at configuration 2's full size, in the launch shape the benchmark times."""
    from synth import make_uniforms
    wl, W = valle
    text, prompt = make_tokens(wl)
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    _say("valle_b1 stochastic")
    ls = _lock(wl.model, W, text, prompt, wl.tree_nodes)
    for i, (tau, T, top_p) in enumerate(((1, 0.9, 0.9), (8, 1.0, 1.0), (64, 0.9, 0.95))):
        ls.step(tree, tau, sample=(T, top_p, make_uniforms(78, i, 1, tree.n_nodes, wl.model.n_logits)))
        _say(f"  step {i} tau {tau} T {T} top_p {top_p}: kept {ls.stats.nucleus_sizes[-1]:.0f} score err {ls.stats.max_score_err:.2e}")
    ls.check_kv(layers=[0, 11])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} accepted lengths {np.bincount(s.accepted_hist).tolist()} "
         f"ties {s.tie_root}/{s.tie_list}/{s.tie_edge}")
    assert s.compared >= 2


def test_large_vocabulary_16k():
    """A 16 000-entry speech vocabulary (16 001 logits per row: the draft lists come from the
    re-scanning top-k, the stochastic rule holds a whole row in LDS) on a 3-layer d = 1024 model."""
    from synth import make_uniforms
    m = PRESETS["vocab16k_b1"].model
    cfg = dataclasses.replace(m, n_layers=3, max_positions=512)
    _say("vocabulary 16k")
    W = make_weights(cfg, 19)
    rng = np.random.default_rng(45)
    text, prompt = rand_tokens(cfg, rng, 1, (32, 32), (100, 100))
    tree = make_tree(64, (10,) * 4)
    ls = _lock(cfg, W, text, prompt, 64)
    for i, tau in enumerate((1, 4, 64)):
        ls.step(tree, tau)
    ls.step(tree, 16, sample=(0.9, 0.9, make_uniforms(79, 0, 1, 64, cfg.n_logits)))
    ls.step(tree, 2, sample=(1.0, 1.0, make_uniforms(79, 1, 1, 64, cfg.n_logits)))
    ls.check_kv(layers=[0, 2])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} ties {s.tie_root}/{s.tie_list}/{s.tie_edge} logit err {s.max_logit_err:.2e} "
         f"score err {s.max_score_err:.2e} kept {[round(x) for x in s.nucleus_sizes]}")
    assert s.compared >= 4


def test_many_row_unit_kinds_on_ragged_shapes(monkeypatch):
    """The many-row kernel's 128 x 128 linear-map units and whole-head attention units, which the
    library only picks for maps and batches that fill the GPU, forced on for a small batch with
    ragged shapes (280 rows: a partial 128-row block; 56-node tree: a partial query tile;
    vocabulary 301: a partial column group)."""
    monkeypatch.setenv("VADUSA_BIG_MIN_UNITS", "1")     # read when the context is created
    cfg = small_cfg("bf16", layers=2, d=128, heads=3, V=300, maxpos=256)
    _say("many-row unit kinds, ragged shapes")
    W = make_weights(cfg, 17, std=STD["bf16"], ln_jitter=0.1)
    rng = np.random.default_rng(47)
    text, prompt = rand_tokens(cfg, rng, 5, (3, 9), (40, 75))
    tree = make_tree(56, (10, 10, 10))
    ls = _lock(cfg, W, text, prompt, 56)
    for tau in (1, 3, 8):
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} ties {s.tie_root}/{s.tie_list}/{s.tie_edge} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 2


@pytest.mark.parametrize("nodes,caps,batch", [(32, (6, 6, 6), 9), (12, (4, 3, 2), 24)])
def test_many_row_attention_units_of_several_pairs(monkeypatch, nodes, caps, batch):
    """Whole-head attention units of the many-row kernel for trees of one or two query tiles: a unit takes four or
    two (sequence, head) pairs, a wave per query tile.  Forced on for a small batch whose pair count (27, 72 with
    three attention heads) leaves the last unit short of pairs (27 = 13 x 2 + 1) or not (72 = 18 x 4)."""
    monkeypatch.setenv("VADUSA_BIG_MIN_UNITS", "1")
    cfg = small_cfg("bf16", layers=2, d=192, heads=3, V=300, maxpos=160)
    _say(f"many-row attention units of several pairs, {nodes}-node tree, batch {batch}")
    W = make_weights(cfg, 19, std=STD["bf16"], ln_jitter=0.1)
    rng = np.random.default_rng(59)
    text, prompt = rand_tokens(cfg, rng, batch, (3, 9), (20, 75))
    tree = make_tree(nodes, caps)
    ls = _lock(cfg, W, text, prompt, nodes)
    for tau in (1, 3):
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} ties {s.tie_root}/{s.tie_list}/{s.tie_edge} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 1


@pytest.mark.parametrize("dtype,chunk", [("fp32", 160), ("bf16", 160), ("bf16", 512)])
def test_prefill_in_long_passes(dtype, chunk):
    """vadusa_config.prefill_chunk: the prompt runs through the decoder in passes of up to that many
    rows per sequence (more than the 128 rows a tree can have; from 256 rows on in the many-row
    kernel), ragged batch, then ordinary steps."""
    cfg = small_cfg(dtype, maxpos=512)
    _say(f"prefill passes of {chunk} rows, {dtype}")
    W = make_weights(cfg, 23, std=STD[dtype], ln_jitter=0.1)
    rng = np.random.default_rng(51)
    text, prompt = rand_tokens(cfg, rng, 2, (5, 40), (150, 330))
    tree = make_tree(24, (3, 3, 2))
    ls = _lock(cfg, W, text, prompt, 24, prefill_chunk=chunk)      # the constructor checks the prefill against the oracle
    for tau in (1, 3):
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"  lengths {[len(t) + len(p) for t, p in zip(text, prompt)]} compared {s.compared}/{s.steps} "
         f"logit err {s.max_logit_err:.2e} kv err {s.max_kv_err:.2e}")
    assert s.compared >= 1


def test_valle_b1_prefill_in_one_pass(valle):
    """Configuration 2 at full size with prefill_chunk = 512: the 289-token prompt is one pass of the
    many-row kernel; then steps as usual."""
    wl, W = valle
    text, prompt = make_tokens(wl)
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    _say("valle_b1, prefill in one pass")
    ls = _lock(wl.model, W, text, prompt, wl.tree_nodes, prefill_chunk=512)
    for tau in (1, 4):
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 6, 11])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e} kv err {s.max_kv_err:.2e}")
    assert s.compared >= 1


def test_many_row_kernel_with_128_node_tree(monkeypatch):
    """A 128-node tree has eight query tiles per head: the whole-head attention unit (four waves, one
    query tile each) must not be picked for it even where every other condition holds."""
    monkeypatch.setenv("VADUSA_BIG_MIN_UNITS", "1")
    cfg = small_cfg("bf16", layers=2, d=128, heads=4, V=300, maxpos=384)
    _say("many-row kernel, 128-node tree")
    W = make_weights(cfg, 29, std=STD["bf16"])
    rng = np.random.default_rng(53)
    text, prompt = rand_tokens(cfg, rng, 2, (3, 9), (40, 75))
    tree = make_tree(128, (10, 10, 10, 10))
    ls = _lock(cfg, W, text, prompt, 128)
    for tau in (1, 4):
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 1


def test_valle_b1_planted_drafts_fused_step(valle):
    """Configuration 2 at full size through the one-call step the benchmark times (vadusa_step), with the true
    continuation planted among the candidates: accepted paths of every length 1..5, so the compaction units
    of all 12 layers and 16 heads move several rows, the continuation starts from deep nodes, and the cache
    is compared with the oracle's on every layer."""
    wl, W = valle
    cfg = wl.model
    text, prompt = make_tokens(wl)
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    model = O.Model(cfg, W)
    _say("valle_b1 planted drafts, fused step: greedy continuation on the oracle")
    greedy = O.generate(model, text[0], prompt[0], chain_tree(1), 1, 90, ignore_eos=True)[0]
    rng = np.random.default_rng(31)
    ls = _lock(cfg, W, text, prompt, wl.tree_nodes)
    steps = 0
    while steps < 26 and len(ls.sts[0].emitted) < 84:
        st = ls.sts[0]
        n = len(st.emitted)
        on = st.emitted == greedy[:n] and st.root == greedy[n]
        fut = greedy[n + 1:n + 1 + cfg.n_draft_heads] if on else []
        lists = planted_lists(fut, tree, cfg.n_draft_heads, cfg.n_logits, rng, p_hit=0.9, p_first=0.8)
        ls.step(tree, 1 + steps % 2, override=[lists], fused=True)
        steps += 1
    ls.check_kv(layers=list(range(cfg.n_layers)))
    s = ls.stats
    _say(f"  steps {s.steps} compared {s.compared} accepted lengths {np.bincount(s.accepted_hist).tolist()} "
         f"ties {s.tie_root}/{s.tie_list}/{s.tie_edge} logit err {s.max_logit_err:.2e} kv err {s.max_kv_err:.2e}")
    assert s.steps >= 20 and s.compared >= 16
    assert set(s.accepted_hist) >= {1, 2, 3, 4, 5}


@pytest.mark.parametrize("heads,nodes", [(4, 96), (6, 64), (6, 128)])
def test_ablation_trees_full_size(heads, nodes):
    """The ablation shapes of Sec. 3.1.3 (four or six draft heads, 64 / 96 / 128 candidates) on the 12-layer
    d = 1024 model: 96 nodes are six query tiles, six heads give paths of up to seven rows."""
    cfg = dataclasses.replace(PRESETS["valle_b1"].model, n_draft_heads=heads, max_positions=640)
    _say(f"ablation shape: {heads} heads, {nodes} nodes")
    W = make_weights(cfg, 20241021 + heads)
    rng = np.random.default_rng(61 + nodes)
    text, prompt = rand_tokens(cfg, rng, 1, (64, 64), (225, 225))
    tree = make_tree(nodes, (10,) * heads)
    assert tree.n_nodes == nodes
    ls = _lock(cfg, W, text, prompt, nodes)
    ls.step(tree, 1)
    ls.step(tree, 3, fused=True)
    ls.check_kv(layers=[0, 11])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} ties {s.tie_root}/{s.tie_list}/{s.tie_edge} logit err {s.max_logit_err:.2e}")
    assert s.compared >= 1


def test_large_vocabulary_16k_full_depth():
    """The 16 001-logit vocabulary on all 12 layers: one step."""
    wl = PRESETS["vocab16k_b1"]
    cfg = dataclasses.replace(wl.model, max_positions=512)
    _say("vocabulary 16k, 12 layers")
    W = make_weights(cfg, wl.seed)
    rng = np.random.default_rng(46)
    text, prompt = rand_tokens(cfg, rng, 1, (32, 32), (100, 100))
    tree = make_tree(64, (10,) * 4)
    ls = _lock(cfg, W, text, prompt, 64)
    ls.step(tree, 4, fused=True)
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} ties {s.tie_root}/{s.tie_list}/{s.tie_edge} logit err {s.max_logit_err:.2e}")
    assert s.compared + s.tie_root + s.tie_edge >= 1


def _extended(prompt, vocab, extra, seed):
    rng = np.random.default_rng(seed)
    return [np.concatenate([p, rng.integers(0, vocab, extra).astype(np.int32)]) for p in prompt]


def test_hubert_b16_consecutive_steps_and_end_of_generation():
    """Configuration 3 at full size beyond one verification: three consecutive steps from the start of
    generation, and one verification at the committed lengths of its end (620..780), the oracle following
    sampled sequences."""
    from parity import sampled_check
    wl = PRESETS["hubert_b16"]
    _say("hubert_b16: three consecutive steps")
    W = make_weights(wl.model, wl.seed)
    text, prompt = make_tokens(wl)
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    n, skipped, err = sampled_check(wl.model, W, text, prompt, tree, 3, [2, 13], kv_layers=(0, 6, 11), steps=3)
    _say(f"  compared {n} skipped {skipped} logit err {err:.2e}")
    assert n >= 4
    deep = _extended(prompt, wl.model.speech_vocab, wl.n_generate, 71)
    _say(f"hubert_b16 at the end of generation: L = {min(len(t) + len(p) for t, p in zip(text, deep))}.."
         f"{max(len(t) + len(p) for t, p in zip(text, deep))}")
    n, skipped, err = sampled_check(wl.model, W, text, deep, tree, 3, [7, 15], kv_layers=(11,))
    _say(f"  compared {n} skipped {skipped} logit err {err:.2e}")
    assert n >= 1


def test_throughput_b64_consecutive_steps_and_end_of_generation():
    """Configuration 5 at full size beyond one verification at tau = 8: three consecutive steps at tau = 1, 8, 1
    and one verification at L = 1039 (the end of generation; the cache holds 1200 rows per sequence)."""
    from parity import sampled_check
    wl = PRESETS["throughput_b64"]
    _say("throughput_b64: three consecutive steps, tau 1 / 8 / 1")
    W = make_weights(wl.model, wl.seed)
    text, prompt = make_tokens(wl)
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    n, skipped, err = sampled_check(wl.model, W, text, prompt, tree, [1, 8, 1], [9, 50], kv_layers=(0, 11), steps=3)
    _say(f"  compared {n} skipped {skipped} logit err {err:.2e}")
    assert n >= 4
    deep = _extended(prompt, wl.model.speech_vocab, wl.n_generate, 72)
    _say(f"throughput_b64 at the end of generation: L = {len(text[0]) + len(deep[0])}")
    n, skipped, err = sampled_check(wl.model, W, text, deep, tree, 1, [33], kv_layers=(11,))
    _say(f"  compared {n} skipped {skipped} logit err {err:.2e}")
    assert n + skipped == 1


def test_residual_rows_with_large_mean():
    """Rows of the residual stream whose mean is several times their spread (a common offset on the
    out-projection and FFN biases; the N(0, 0.02) weights never produce one): the LayerNorm folded into the
    next map works on the bf16 copy of the raw residual row and on tile statistics, so its error grows with
    mean / spread (the copy's rounding is relative to the row's magnitude); this case sits where the bf16
    copy still carries the spread to within the tolerance."""
    cfg = small_cfg("bf16", layers=3, d=256, heads=3, V=300, maxpos=256)
    _say("residual rows with a large mean")
    W = make_weights(cfg, 33, std=STD["bf16"], ln_jitter=0.1)
    from synth.weights import round_to_bf16
    for l in range(cfg.n_layers):
        W[f"L{l}.bo"] = round_to_bf16(W[f"L{l}.bo"] + 0.25)
        W[f"L{l}.b2"] = round_to_bf16(W[f"L{l}.b2"] + 0.5)
    rng = np.random.default_rng(34)
    text, prompt = rand_tokens(cfg, rng, 2, (5, 9), (30, 45))
    tree = make_tree(40, (6, 4, 3))
    ls = _lock(cfg, W, text, prompt, 40)
    for tau in (1, 3, 2):
        ls.step(tree, tau)
    ls.check_kv(layers=[0, 2])
    s = ls.stats
    _say(f"  compared {s.compared}/{s.steps} ties {s.tie_root}/{s.tie_list}/{s.tie_edge} logit err {s.max_logit_err:.2e} kv err {s.max_kv_err:.2e}")
    assert s.compared >= 2
