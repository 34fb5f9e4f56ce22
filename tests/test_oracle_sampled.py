"""Pins for the stochastic form of Algorithm 1 (nucleus + temperature sampling of tau
tokens per position, Sec. 3.1.2): the nucleus against hand-worked cases and its set
definition, the draws against the closed-form probabilities of sampling without
replacement, and the limits in which the rule reduces to the deterministic one."""
import copy
import itertools

import numpy as np

from oracle import vadusa_oracle as O
from synth import make_tree, make_uniforms
from helpers import SMALL, small_model


def test_nucleus_hand_cases():
    s = np.log(np.array([0.5, 0.3, 0.1, 0.1]))
    # mass above each token: 0, 0.5, 0.8, 0.8
    assert O.nucleus(s, 0.40).tolist() == [True, False, False, False]
    assert O.nucleus(s, 0.75).tolist() == [True, True, False, False]
    assert O.nucleus(s, 0.79).tolist() == [True, True, False, False]
    assert O.nucleus(s, 0.81).tolist() == [True, True, True, True]     # equal scores go together
    assert O.nucleus(s, 1.0).tolist() == [True] * 4
    assert O.nucleus(s, 0.40, min_keep=2).tolist() == [True, True, False, False]
    assert O.nucleus(s, 0.40, min_keep=3).tolist() == [True, True, True, True]
    # order of the ids does not matter
    perm = np.array([2, 0, 3, 1])
    assert O.nucleus(s[perm], 0.75).tolist() == [False, True, False, True]


def test_nucleus_is_smallest_most_probable_set_reaching_top_p():
    rng = np.random.default_rng(11)
    for trial in range(200):
        V = int(rng.integers(2, 40))
        s = rng.normal(0, 2.0, V)
        if trial % 3 == 0:
            s = np.round(s)                      # many equal scores
        top_p = float(rng.uniform(0.05, 0.999))
        keep = O.nucleus(s, top_p)
        p = np.exp(s - s.max())
        p /= p.sum()
        # set definition, token by token
        want = np.array([p[s > s[v]].sum() < top_p for v in range(V)])
        assert keep.tolist() == want.tolist()
        # a most-probable-first set ...
        assert s[keep].min() > (s[~keep].max() if (~keep).any() else -np.inf)
        # ... that reaches top_p, and would not without its least probable score
        assert p[keep].sum() >= top_p - 1e-12
        assert p[keep & (s > s[keep].min())].sum() < top_p
        # min_keep only ever adds the next most probable tokens
        k = int(rng.integers(1, V + 1))
        keep_k = O.nucleus(s, top_p, min_keep=k)
        assert (keep_k | keep).tolist() == keep_k.tolist() and keep_k.sum() >= k
        assert keep_k.tolist() == (keep | np.array([(s > s[v]).sum() < k for v in range(V)])).tolist()


def _chi2(counts, probs, n):
    exp = np.asarray(probs) * n
    return float(((np.asarray(counts) - exp) ** 2 / exp).sum())


def test_draw_order_matches_sampling_without_replacement():
    # 5 tokens, temperature 0.7, no nucleus cut: P(first = i, second = j) = p_i p_j / (1 - p_i)
    z = np.array([1.0, 0.2, -0.5, 0.7, 0.0])
    T, n = 0.7, 60000
    p = np.exp(z / T) / np.exp(z / T).sum()
    u = np.random.default_rng(3).random((n, 5))
    y = O.perturbed_scores(np.broadcast_to(z, (n, 5)), u, T, 1.0, 2)
    first2 = np.argsort(-y, axis=1)[:, :2]
    pairs = list(itertools.permutations(range(5), 2))
    counts = [int(((first2[:, 0] == i) & (first2[:, 1] == j)).sum()) for i, j in pairs]
    probs = [p[i] * p[j] / (1 - p[i]) for i, j in pairs]
    assert _chi2(counts, probs, n) < 43.8          # 19 degrees of freedom, 0.1 % level
    # a wrong temperature or sampling with the unscaled logits is far outside
    p1 = np.exp(z) / np.exp(z).sum()
    assert _chi2(counts, [p1[i] * p1[j] / (1 - p1[i]) for i, j in pairs], n) > 500


def test_draws_stay_inside_the_nucleus_with_renormalised_probabilities():
    z = np.log(np.array([0.4, 0.25, 0.2, 0.1, 0.05]))
    n = 40000
    u = np.random.default_rng(4).random((n, 5))
    y = O.perturbed_scores(np.broadcast_to(z, (n, 5)), u, 1.0, 0.8, 1)    # keeps tokens 0, 1, 2
    assert np.isinf(y[:, 3:]).all() and np.isfinite(y[:, :3]).all()
    first = np.argmax(y, axis=1)
    counts = [int((first == i).sum()) for i in range(3)]
    assert _chi2(counts, np.array([0.4, 0.25, 0.2]) / 0.85, n) < 13.8    # 2 dof, 0.1 % level
    # tau = 4 draws need four tokens: the nucleus is widened to the four most probable
    y4 = O.perturbed_scores(z, u[0], 1.0, 0.8, 4)
    assert np.isfinite(y4[:4]).all() and np.isinf(y4[4])


def test_gumbel_closed_forms():
    assert abs(O.gumbel(np.exp(-1.0))) < 1e-15                    # -log(-log e^-1) = 0
    assert abs(O.gumbel(np.exp(-np.exp(-2.0))) - 2.0) < 1e-12
    u = np.random.default_rng(5).random(400000)
    g = O.gumbel(u)
    assert abs(g.mean() - 0.5772156649) < 5e-3 and abs(g.var() - np.pi ** 2 / 6) < 2e-2


def _run(model, tree, tau, sample_of_step, steps=6):
    st = O.prefill(model, np.arange(5) % SMALL.text_vocab, np.arange(9) % SMALL.speech_vocab)
    out = []
    for i in range(steps):
        r = O.step(model, st, tree, tau, ignore_eos=True, sample=sample_of_step(i))
        out.append((r["path"], r["accepted"], r["next_root"]))
    return out, st


def test_equal_noise_reduces_to_the_deterministic_rule():
    model = small_model()
    tree = make_tree(14, (3, 3, 2))
    V1 = SMALL.speech_vocab + 1
    for tau in (1, 3):
        want, _ = _run(model, tree, tau, lambda i: None)
        const_u = np.full((tree.n_nodes, V1), 0.37)
        got, _ = _run(model, tree, tau, lambda i: (1.0, 1.0, const_u))
        assert got == want
        # a positive temperature rescales every logit alike: same order, same decisions
        got, _ = _run(model, tree, tau, lambda i: (0.25, 1.0, const_u))
        assert got == want
    # tau = 1 at a very low temperature is greedy decoding whatever the noise
    want, _ = _run(model, tree, 1, lambda i: None)
    got, _ = _run(model, tree, 1, lambda i: (1e-4, 1.0, make_uniforms(1, i, 1, tree.n_nodes, V1)[0]))
    assert got == want


def test_stochastic_step_accepts_exactly_the_drawn_candidates():
    model = small_model()
    tree = make_tree(20, (4, 3, 2))
    V1 = SMALL.speech_vocab + 1
    st = O.prefill(model, np.arange(5) % SMALL.text_vocab, np.arange(9) % SMALL.speech_vocab)
    seen_longer = 0
    for i in range(12):
        tau, T, top_p = 1 + i % 4, (0.9, 1.0)[i % 2], (1.0, 0.9, 0.6)[i % 3]
        u = make_uniforms(2, i, 1, tree.n_nodes, V1)[0]
        before = copy.deepcopy(st)
        r = O.step(model, st, tree, tau, ignore_eos=True, sample=(T, top_p, u))
        # the draws, re-derived position by position from the definition: sort the kept
        # tokens by s + g, take tau
        logits = r["logits"]
        draws = []
        for n in range(tree.n_nodes):
            s = logits[n] / T
            keep = O.nucleus(s, top_p, min_keep=tau)
            y = np.where(keep, s - np.log(-np.log(u[n].astype(np.float64))), -np.inf)
            draws.append([int(v) for v in np.argsort(-y, kind="stable")[:tau]])
            assert keep.sum() >= tau
        ok = [True] * tree.n_nodes
        for n in range(1, tree.n_nodes):
            ok[n] = ok[tree.parent[n]] and int(r["tok"][n]) in draws[tree.parent[n]]
        deepest = max(tree.depth[n] for n in range(tree.n_nodes) if ok[n])
        leftmost = min((n for n in range(tree.n_nodes) if ok[n] and tree.depth[n] == deepest),
                       key=lambda n: tree.paths[n])
        assert r["path"][-1] == leftmost and len(r["path"]) == deepest + 1
        assert r["next_root"] == draws[leftmost][0]                  # continuation = first draw there
        assert st.L == before.L + len(r["path"])
        seen_longer += len(r["path"]) > 1
    assert seen_longer >= 1


def test_tolerance_as_large_as_the_vocabulary_accepts_every_candidate():
    model = small_model()
    tree = make_tree(14, (3, 3, 2))
    V1 = SMALL.speech_vocab + 1
    st = O.prefill(model, np.arange(5) % SMALL.text_vocab, np.arange(9) % SMALL.speech_vocab)
    r = O.step(model, st, tree, V1, ignore_eos=True,
               sample=(1.0, 0.5, make_uniforms(3, 0, 1, tree.n_nodes, V1)[0]))
    deepest = max(tree.depth)
    assert len(r["path"]) == deepest + 1
    assert r["path"][-1] == min((n for n in range(tree.n_nodes) if tree.depth[n] == deepest),
                                key=lambda n: tree.paths[n])
