"""Pins for verification with tolerance (Algorithm 1), branch choice (Sec. 2.3),
the whole decode loop, KV commit and the stand-in tree generator."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import vadusa_oracle as O
from synth import make_tree, chain_tree, full_tree
from synth.trees import tree_from_paths, path_probs, TreeSpec
from helpers import SMALL, small_model, planted_lists

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "acceptance_cases.json")


def _tree_from_arrays(parent, rank):
    paths = []
    for n, (p, r) in enumerate(zip(parent, rank)):
        paths.append(() if p < 0 else paths[p] + (r,))
    t = tree_from_paths(paths)
    assert t.parent.tolist() == list(parent)     # fixture is in canonical order
    return t


@pytest.mark.parametrize("case", json.load(open(GOLDEN))["cases"], ids=lambda c: c["name"])
def test_golden_acceptance_cases(case):
    tree = _tree_from_arrays(case["parent"], case["rank"])
    tok = np.array(case["tok"])
    logits = np.array(case["logits"], float)
    path = O.select_path(tree, tok, logits, case["tau"])
    assert path == case["expect_path"]
    assert [int(tok[n]) for n in path] == case["expect_tokens"]
    assert int(O.top_k(logits[path[-1]], 1)[0]) == case["expect_next_root"]


TREES = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "tree_cases.json")))


@pytest.mark.parametrize("case", TREES["cases"], ids=lambda c: c["name"])
def test_golden_tree_expansion_and_mask(case):
    """Hand-drawn trees (Fig. 1(c) and a sparse one): node tokens, depths, K_i and the
    tree-attention mask, every value of the fixture written by hand."""
    tree = tree_from_paths(case["paths"])
    assert tree.parent.tolist() == case["expect_parent"]
    assert tree.depth.tolist() == case["expect_depth"]
    assert O.topk_needed(tree.depth, tree.rank, len(case["lists"])) == case["expect_need"]
    tok = O.expand_tree(case["root"], [np.array(l) for l in case["lists"]], tree)
    assert tok.tolist() == case["expect_tok"]
    mask = np.array([[ch == "1" for ch in row] for row in case["expect_mask"]])
    assert np.array_equal(O.ancestor_mask(tree.parent), mask)


def test_golden_draft_lists():
    """draft_lists = the first K_i ids of each head's logits in descending order, ties to the lower id."""
    c = TREES["draft_lists_case"]
    tree = tree_from_paths(c["paths"])

    class _M:
        class cfg:
            n_draft_heads = 3
    st = O.SeqState(K=None, V=None, L=0, root=0, draft_logits=[np.array(z) for z in c["draft_logits"]])
    got = O.draft_lists(_M, st, tree)
    assert [g.tolist() for g in got] == c["expect_lists"]


def test_verify_branch_is_longest_tolerated_prefix():
    """Algorithm 1 against its definition by exhaustive enumeration on tiny cases: k* is the largest k such that
    every c_{i+1}, i < k, has fewer than tau ids ranked ahead of it in row i."""
    rng = np.random.default_rng(3)
    for trial in range(200):
        k, V1 = int(rng.integers(0, 5)), 6
        logits = rng.integers(0, 4, (k + 1, V1)).astype(float)
        cand = rng.integers(0, V1, k + 1)
        tau = int(rng.integers(1, V1 + 1))
        want = 0
        while want < k and _rank(logits[want], cand[want + 1]) < tau:
            want += 1
        assert O.verify_branch(logits, cand, tau) == want


def _rank(z, t):
    return int((z > z[t]).sum() + (z[:t] == z[t]).sum())


def test_acceptance_invariants_random():
    rng = np.random.default_rng(5)
    for trial in range(60):
        tree = make_tree(int(rng.integers(2, 30)), (4, 3, 3, 2))
        M, V1 = tree.n_nodes, 12
        logits = rng.integers(0, 5, (M, V1)).astype(float) + rng.random((M, V1)) * (trial % 2)
        tok = rng.integers(0, V1, M)
        prev = 0
        for tau in range(1, V1 + 2):
            path = O.select_path(tree, tok, logits, tau)
            # valid root path, every edge within tolerance, first edge beyond the end (if any
            # child exists on a longer accepted route) cannot make a longer accepted path
            assert path[0] == 0
            for a, b in zip(path, path[1:]):
                assert tree.parent[b] == a and _rank(logits[a], tok[b]) < tau
            ok = [True] * M
            for n in range(1, M):
                ok[n] = ok[tree.parent[n]] and _rank(logits[tree.parent[n]], tok[n]) < tau
            depth_ok = [tree.depth[n] for n in range(M) if ok[n]]
            assert len(path) - 1 == max(depth_ok)
            cands = [n for n in range(M) if ok[n] and tree.depth[n] == max(depth_ok)]
            assert path[-1] == min(cands)                      # leftmost among the longest
            assert len(path) >= prev                           # monotone in tau
            prev = len(path)
            if tau == 1:
                for a, b in zip(path, path[1:]):
                    assert tok[b] == O.top_k(logits[a], 1)[0]
        # tau >= V+1 accepts every edge: deepest, then leftmost leaf
        deepest = [n for n in range(M) if tree.depth[n] == tree.max_depth]
        assert path[-1] == deepest[0]


def test_verify_branch_is_algorithm_1_on_paper_notation():
    # k = 3 draft heads, branch (c_0..c_3); L(i) one-hot-ish rows
    V1 = 8
    L = np.zeros((4, V1))
    L[0, 5] = 1; L[1, 6] = 1; L[2, 7] = 1; L[3, 0] = 1
    assert O.verify_branch(L, [1, 5, 6, 7], 1) == 3          # all accepted: k* = k
    assert O.verify_branch(L, [1, 5, 6, 2], 1) == 2
    assert O.verify_branch(L, [1, 5, 2, 7], 1) == 1          # stops at the first miss
    assert O.verify_branch(L, [1, 2, 6, 7], 1) == 0          # output is (c_0) alone
    L[1, 2] = 0.5                                            # id 2 is second best at position 1
    assert O.verify_branch(L, [1, 5, 2, 7], 2) == 3


@pytest.mark.parametrize("tree", [make_tree(16, (4, 2, 2)), chain_tree(4), chain_tree(1),
                                  full_tree((3, 2))])
def test_tau1_generation_equals_plain_greedy(tree):
    """Vanilla verification is lossless (Sec. 2.1): same tokens as plain AR decoding,
    whatever the tree and whatever the draft heads propose."""
    model = small_model(seed=11)
    cfg = model.cfg
    rng = np.random.default_rng(6)
    text = rng.integers(0, cfg.text_vocab, 5)
    prompt = rng.integers(0, cfg.speech_vocab, 8)
    want = O.greedy_ar(model, text, prompt, 24, ignore_eos=True)
    got, lens = O.generate(model, text, prompt, tree, 1, 24, ignore_eos=True)
    assert got == want


@pytest.mark.parametrize("tau", [1, 2, 3])
def test_planted_drafts_long_paths_and_replay(tau):
    """With the true continuation planted among the candidates, paths longer than one
    are accepted; at tau = 1 the output is still plain greedy; at any tau every
    emitted token ranks below tau under a plain causal forward of what precedes it,
    and the committed KV equals that of a fresh prefill over the emitted sequence."""
    model = small_model(seed=12)
    cfg = model.cfg
    rng = np.random.default_rng(7)
    text = rng.integers(0, cfg.text_vocab, 5)
    prompt = rng.integers(0, cfg.speech_vocab, 8)
    tree = make_tree(16, (4, 2, 2))
    greedy = O.greedy_ar(model, text, prompt, 40, ignore_eos=True)
    st = O.prefill(model, text, prompt)
    lens = []
    while len(st.emitted) < 30:
        n = len(st.emitted)
        on_track = st.emitted == greedy[:n] and st.root == greedy[n]
        future = greedy[n + 1:n + 1 + cfg.n_draft_heads] if on_track else []
        lists = planted_lists(future, tree, cfg.n_draft_heads, cfg.n_logits, rng, p_hit=0.8)
        r = O.step(model, st, tree, tau, draft_override=lists, ignore_eos=True)
        lens.append(len(r["accepted"]))
        assert 1 <= lens[-1] <= cfg.n_draft_heads + 1
    assert max(lens) >= 3
    if tau == 1:
        assert st.emitted == greedy[:len(st.emitted)]
    ref = O.causal_forward(model, text, np.concatenate([prompt, st.emitted]))
    L0 = len(text) + len(prompt)
    for j, t in enumerate(st.emitted):
        assert _rank(ref["logits"][L0 + j - 1], t) < tau
    assert st.L == L0 + len(st.emitted)
    err = np.abs(st.K[:, :st.L] - ref["K"]).max() + np.abs(st.V[:, :st.L] - ref["V"]).max()
    assert err < 1e-9
    assert st.root == int(O.top_k(ref["logits"][-1], 1)[0])


def test_eos_truncates_and_finishes():
    model = small_model(seed=13)
    cfg = model.cfg
    st = O.prefill(model, [1, 2, 3], [4, 5, 6])
    tree = chain_tree(3)
    eos = cfg.speech_vocab
    # force the root to EOS: the path is cut after it and nothing more is emitted
    st.root = eos
    r = O.step(model, st, tree, cfg.n_logits, ignore_eos=False)
    assert r["accepted"] == [eos] and st.finished and st.L == 7
    assert O.step(model, st, tree, 1)["accepted"] == []
    st2 = O.prefill(model, [1, 2, 3], [4, 5, 6])
    st2.root = eos
    r2 = O.step(model, st2, tree, cfg.n_logits, ignore_eos=True)
    assert len(r2["accepted"]) == 3 and not st2.finished


def _expected_len(paths_probs):
    return sum(paths_probs)


@pytest.mark.parametrize("caps,M", [((3, 2), 5), ((2, 2, 2), 7), ((3, 3), 6), ((4, 2, 2), 6)])
def test_tree_generator_is_the_best_closed_subset(caps, M):
    """Criterion of Sec. 2.4: maximise the expected accepted length within M nodes.
    Brute force over all ancestor-closed M-subsets of the full tree."""
    full = full_tree(caps)
    p = path_probs(full, caps)
    idx = list(range(1, full.n_nodes))
    best = -1.0
    for sub in itertools.combinations(idx, M - 1):
        s = set(sub) | {0}
        if all(int(full.parent[n]) in s for n in sub):
            best = max(best, sum(p[n] for n in s))
    got = make_tree(M, caps)
    got_p = path_probs(got, caps).sum()
    assert abs(got_p - best) < 1e-12
    assert got.n_nodes == M
