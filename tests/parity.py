"""Lockstep comparison of the HIP library with the CPU oracle.

Protocol (per step, both sides on identical state):
  * roots and the draft lists' used entries must agree; logits of every tree
    node must agree within the relative-L2 tolerance; edge decisions, the chosen
    path and the committed state must agree;
  * a differing *decision* is tolerated only when the oracle's own margin for
    that decision (gap between the two logits that decide it) is <= MARGIN; it is
    then counted as a tie divergence and the library is re-synchronised to the
    oracle (draft_override for lists, a forced path through vadusa_kv_compact, or
    a fresh prefill of the oracle's sequence for a differing root);
  * any decision mismatch with a larger margin, and any logits error above the
    tolerance, fails.
"""
from dataclasses import dataclass, field

import numpy as np

from oracle import vadusa_oracle as O
from paper_2410_21951_amd import Vadusa, TreeArrays, DBG

MARGIN = 1e-2
TOL = {"fp32": 1e-4, "bf16": 1e-2}
# Stochastic rule: a decision is held to bit-exactness only if the oracle takes the same one with
# the nucleus bound moved by this much either way (the kept probability mass carries the logits'
# error) and with a score margin above MARGIN / temperature.
TOP_P_SLACK = {"fp32": 1e-4, "bf16": 2e-2}


def rel_l2(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), 1e-300))


def top_gap(z, k=1):
    """Smallest gap between consecutive entries among the k+1 largest logits."""
    s = np.sort(np.asarray(z))[::-1][:k + 1]
    return float(np.min(s[:-1] - s[1:])) if len(s) > 1 else np.inf


def edge_margin(z, t, tau):
    """Distance of the accept/reject decision for token t under tolerance tau from flipping."""
    s = np.sort(z)[::-1]
    rank = int((z > z[t]).sum() + (z[:t] == z[t]).sum())
    if rank < tau:
        return float(z[t] - s[tau]) if tau < len(s) else np.inf
    return float(s[tau - 1] - z[t])


def score_variants(logits, sample, tau, slack):
    """The oracle's perturbed scores for top_p - slack, top_p, top_p + slack (one entry if top_p >= 1)."""
    T, top_p, u = sample
    if top_p >= 1.0:
        return [O.perturbed_scores(logits, u, T, top_p, tau)]
    return [O.perturbed_scores(logits, u, T, min(max(p, 1e-6), 0.999999), tau) for p in (top_p - slack, top_p, top_p + slack)]


def firm_edge(variants, parent, t, tau, margin):
    """(decision, firm): the oracle's decision for candidate t under its parent's row, and whether
    every variant takes it with more than `margin` to spare."""
    ds, ms = [], []
    kept = [int(np.isfinite(y[parent]).sum()) for y in variants]
    if min(kept) <= tau:      # the "tau most probable" clause shapes this row: its own near-ties are not modelled
        z = variants[len(variants) // 2][parent]
        return int((z > z[t]).sum() + (z[:t] == z[t]).sum()) < tau, False
    for y in variants:
        z = y[parent]
        ds.append(int((z > z[t]).sum() + (z[:t] == z[t]).sum()) < tau)
        ms.append(edge_margin(z, t, tau))
    mid = ds[len(ds) // 2]
    return mid, all(d == mid for d in ds) and min(ms) > margin


def firm_top(variants, row, margin):
    """Margin of the first draw at `row`: 0 if the variants disagree, else the smallest top-2 gap."""
    tops = [int(O.top_k(y[row], 1)[0]) for y in variants]
    if any(t != tops[0] for t in tops):
        return 0.0
    return min(top_gap(y[row]) for y in variants)


@dataclass
class Stats:
    steps: int = 0
    compared: int = 0
    tie_root: int = 0
    tie_list: int = 0
    tie_edge: int = 0
    max_logit_err: float = 0.0
    max_h_err: float = 0.0
    max_kv_err: float = 0.0
    max_score_err: float = 0.0
    nucleus_sizes: list = field(default_factory=list)
    accepted_hist: list = field(default_factory=list)


class Lockstep:
    def __init__(self, cfg, weights, text, prompt, max_tree_nodes, ignore_eos=True, prefill_chunk=0):
        self.cfg = cfg
        self.model = O.Model(cfg, weights)
        self.text, self.prompt = text, prompt
        self.B = len(text)
        self.ignore_eos = ignore_eos
        self.tol = TOL[cfg.dtype]
        self.dev = Vadusa(cfg, max_batch=self.B, max_tree_nodes=max_tree_nodes, ignore_eos=ignore_eos,
                          prefill_chunk=prefill_chunk)
        self.dev.load_weights(weights)
        self.stats = Stats()
        self.sts = [O.prefill(self.model, t, p) for t, p in zip(text, prompt)]
        self.root_gap = {}     # per sequence: margin of the root when it came from a stochastic step
        self.out_base = [0] * self.B
        self.dev.prefill(text, prompt)
        self.check_prefill()

    # -- comparisons --------------------------------------------------------
    def check_prefill(self):
        L = self.dev.debug(DBG.KV_LEN)
        for b, st in enumerate(self.sts):
            assert L[b] == st.L
        zd = self.dev.debug(DBG.DRAFT_LOGITS)
        for b, st in enumerate(self.sts):
            for i, z in enumerate(st.draft_logits):
                e = rel_l2(zd[b, i], z)
                assert e < self.tol, f"prefill draft logits seq {b} head {i}: rel-L2 {e}"
        self.check_kv(layers=[0, self.cfg.n_layers - 1])

    def check_kv(self, layers, seqs=None):
        for b in (range(self.B) if seqs is None else seqs):
            st = self.sts[b]
            for l in layers:
                for which, ref in ((0, st.K), (1, st.V)):
                    got = self.dev.read_kv(l, b, which, 0, st.L)
                    e = rel_l2(got, ref[l, :st.L])
                    self.stats.max_kv_err = max(self.stats.max_kv_err, e)
                    assert e < self.tol, f"KV layer {l} seq {b} which {which}: rel-L2 {e}"

    def resync(self):
        """Fresh prefill of the library with what the oracle has emitted so far."""
        prompts = [np.concatenate([p, np.asarray(st.emitted, np.int64)]).astype(np.int32)
                   for p, st in zip(self.prompt, self.sts)]
        assert not any(st.finished for st in self.sts), "resync of a finished sequence is not supported"
        self.dev.prefill(self.text, prompts)
        self.out_base = [len(st.emitted) for st in self.sts]

    def step(self, tree, tau, override=None, sample=None, fused=False):
        """One lockstep step.  override: per-sequence per-head candidate lists (or None).
        sample: None, or (temperature, top_p, uniforms [B][M][V+1]) for the stochastic rule.
        fused: run the library's one-call step (vadusa_step, the call the benchmark times) instead of
        verification + compaction; its intermediate results stay readable afterwards.  A path can then not be
        forced where a tie flipped an edge: the library is re-synchronised by a fresh prefill instead."""
        cfg, dev, S = self.cfg, self.dev, self.stats
        margin = MARGIN if sample is None else MARGIN / min(sample[0], 1.0)
        tarr = TreeArrays(tree.parent, tree.rank)
        need = O.topk_needed(tree.depth, tree.rank, cfg.n_draft_heads)
        S.steps += 1
        # (a) roots and lists
        roots = dev.debug(DBG.ROOT)
        lists = dev.debug(DBG.DRAFT_TOPK)
        fin = dev.debug(DBG.FINISHED)
        o_lists = []
        root_diverged = False
        use_override = override is not None
        for b, st in enumerate(self.sts):
            assert bool(fin[b]) == st.finished
            ol = O.draft_lists(self.model, st, tree) if override is None else \
                [np.asarray(a, np.int64) for a in override[b]]
            o_lists.append(ol)
            if st.finished:
                continue
            if roots[b] != st.root:
                # the root came from the previous last-accepted row: margin on that row
                gap = self.root_gap.get(b, top_gap(st.root_logits))
                assert gap <= max(MARGIN, margin), f"root mismatch seq {b}: {roots[b]} vs {st.root}, gap {gap}"
                S.tie_root += 1
                root_diverged = True
            if override is None:
                for i, k in enumerate(need):
                    if k and lists[b, i, :k].tolist() != ol[i].tolist():
                        gap = top_gap(st.draft_logits[i], k)
                        assert gap <= MARGIN, f"draft list mismatch seq {b} head {i}, gap {gap}"
                        S.tie_list += 1
                        use_override = True
        if root_diverged:
            self.resync()
            roots = dev.debug(DBG.ROOT)
            if any(roots[b] != st.root for b, st in enumerate(self.sts)):
                # same tie again: this step cannot be compared; advance the oracle and resync after
                self._oracle_only(tree, tau, o_lists if override is not None else None, sample)
                self.resync()
                return None
            use_override = True
        # (b) verification
        fused_out = None
        if fused:
            fused_out = dev.step(tarr, tau, override=o_lists if use_override else None, sample=sample)
        else:
            dev.verify(tarr, tau, override=o_lists if use_override else None, sample=sample)
        tok = dev.debug(DBG.TREE_TOK)
        logits = dev.debug(DBG.LOGITS)
        scores = dev.debug(DBG.SCORES) if sample is not None else None
        h = dev.debug(DBG.H_NODES)
        edge = dev.debug(DBG.EDGE_OK)
        path = dev.debug(DBG.PATH)
        results = []
        forced = {}
        for b, st in enumerate(self.sts):
            if st.finished:
                assert path[b, 0] == 0
                results.append(O.step(self.model, st, tree, tau))
                continue
            smp = None if sample is None else (sample[0], sample[1], sample[2][b])
            r = O.step(self.model, st, tree, tau, draft_override=o_lists[b], ignore_eos=self.ignore_eos, sample=smp)
            results.append(r)
            assert tok[b].tolist() == r["tok"].tolist(), f"tree tokens differ seq {b}"
            for n in range(tree.n_nodes):
                e = rel_l2(logits[b, n], r["logits"][n])
                S.max_logit_err = max(S.max_logit_err, e)
                assert e < self.tol, f"logits seq {b} node {n}: rel-L2 {e}"
            S.max_h_err = max(S.max_h_err, rel_l2(h[b], r["h"]))
            variants = None
            if sample is not None:
                variants = score_variants(r["logits"], smp, tau, TOP_P_SLACK[cfg.dtype])
                self.check_scores(b, scores[b], variants, r["logits"], smp, tau)
            # edges
            flipped = False
            for n in range(1, tree.n_nodes):
                t = int(r["tok"][n])
                if sample is None:
                    z = r["logits"][tree.parent[n]]
                    want = int((z > z[t]).sum() + (z[:t] == z[t]).sum()) < tau
                    firm = edge_margin(z, t, tau) > MARGIN
                else:
                    want, firm = firm_edge(variants, tree.parent[n], t, tau, margin)
                if bool(edge[b, n]) != want:
                    assert not firm, f"edge decision differs seq {b} node {n}"
                    S.tie_edge += 1
                    flipped = True
            if fused:
                # the compaction has consumed the path: the accepted tokens the call returned stand for it
                # (with equal edge decisions the path choice is a function of the tree alone)
                if not flipped:
                    assert fused_out[b] == r["accepted"], f"accepted tokens differ seq {b}: {fused_out[b]} vs {r['accepted']}"
                elif fused_out[b] != r["accepted"]:
                    forced[b] = r["path"]
            else:
                got_path = path[b, 1:1 + path[b, 0]].tolist()
                if not flipped:
                    assert got_path == r["path"], f"path differs seq {b}: {got_path} vs {r['path']}"
                elif got_path != r["path"]:
                    forced[b] = r["path"]
            S.accepted_hist.append(len(r["path"]))
            if sample is not None:
                self.root_gap[b] = firm_top(variants, r["path"][-1], margin)
            else:
                self.root_gap.pop(b, None)
        # (c) compaction (forced to the oracle's path where a tie flipped an edge)
        if fused:
            if forced:
                self.resync()
                return None
        elif forced:
            for b in range(self.B):
                if b in forced:
                    dev.kv_compact(b, forced[b])
                else:
                    dev.kv_compact(b)
        else:
            dev.kv_compact(-1)
        L = dev.debug(DBG.KV_LEN)
        for b, st in enumerate(self.sts):
            assert L[b] == st.L, f"L differs seq {b}: {L[b]} vs {st.L}"
            out = dev.read_output(b)
            assert out.tolist() == st.emitted[self.out_base[b]:], f"output differs seq {b}"
        S.compared += 1
        return results

    def _oracle_only(self, tree, tau, o_lists, sample=None):
        for b, st in enumerate(self.sts):
            smp = None if sample is None else (sample[0], sample[1], sample[2][b])
            r = O.step(self.model, st, tree, tau, draft_override=None if o_lists is None else o_lists[b],
                       ignore_eos=self.ignore_eos, sample=smp)
            if sample is not None and r["path"]:
                variants = score_variants(r["logits"], smp, tau, TOP_P_SLACK[self.cfg.dtype])
                self.root_gap[b] = firm_top(variants, r["path"][-1], MARGIN / min(sample[0], 1.0))
            else:
                self.root_gap.pop(b, None)

    def check_scores(self, b, got, variants, logits, sample, tau):
        """The library's perturbed scores against the oracle's: a token that every variant of the
        nucleus bound keeps (drops) must be kept (dropped), and the kept values must agree.
        Tokens whose scaled logit lies within the margin of the tau-th / (tau+1)-th largest are
        exempt: the "tau most probable" clause may go either way for them."""
        T = sample[0]
        mid = variants[len(variants) // 2]
        firm_in = np.all([np.isfinite(y) for y in variants], axis=0)
        firm_out = np.all([np.isinf(y) for y in variants], axis=0)
        sc = np.asarray(logits) / T
        srt = -np.sort(-sc, axis=1)
        V1 = sc.shape[1]
        m = MARGIN / min(T, 1.0)
        lo = srt[:, min(tau, V1 - 1)] - m
        hi = srt[:, min(tau, V1) - 1] + m
        fragile = (sc >= lo[:, None]) & (sc <= hi[:, None])
        g = np.isfinite(got)
        bad = ((firm_in & ~g) | (firm_out & g)) & ~fragile
        assert not bad.any(), f"nucleus differs seq {b}: nodes {np.unique(np.nonzero(bad)[0]).tolist()}"
        self.stats.nucleus_sizes.append(float(np.isfinite(mid).sum(axis=1).mean()))
        both = g & np.isfinite(mid)
        e = rel_l2(got[both], mid[both])
        self.stats.max_score_err = max(self.stats.max_score_err, e)
        assert e < self.tol, f"scores seq {b}: rel-L2 {e}"


def sampled_check(cfg, weights, text, prompt, tree, tau, sample, kv_layers=(0,), steps=1):
    """Full-batch run on the GPU, oracle on a sample of the sequences only (for batches whose
    oracle run would take minutes): prefill, then `steps` times verification and compaction
    (tau: one value, or one per step).  Returns (sequence-steps compared, sequence-steps skipped
    because a root or list decision sat inside the margin, largest logit error).  A sampled
    sequence whose root flips inside the margin leaves the sample (the oracle cannot follow it
    any further).  Decisions are held to the same margin rule as Lockstep."""
    B = len(text)
    model = O.Model(cfg, weights)
    tol = TOL[cfg.dtype]
    taus = [tau] * steps if np.isscalar(tau) else list(tau)
    assert len(taus) == steps
    dev = Vadusa(cfg, max_batch=B, max_tree_nodes=tree.n_nodes, ignore_eos=True)
    dev.load_weights(weights)
    dev.prefill(text, prompt)
    need = O.topk_needed(tree.depth, tree.rank, cfg.n_draft_heads)
    states = {b: O.prefill(model, text[b], prompt[b]) for b in sample}
    compared, skipped, max_err = 0, 0, 0.0
    for step_i in range(steps):
        tau_i = taus[step_i]
        roots = dev.debug(DBG.ROOT)
        lists = dev.debug(DBG.DRAFT_TOPK)
        sts = {}
        override = [[lists[b, i].tolist() for i in range(cfg.n_draft_heads)] for b in range(B)]
        for b in list(states):
            st = states[b]
            if roots[b] != st.root:
                assert top_gap(st.root_logits) <= MARGIN, f"root mismatch seq {b} step {step_i}"
                skipped += 1
                del states[b]
                continue
            ol = O.draft_lists(model, st, tree)
            for i, k in enumerate(need):
                if k and lists[b, i, :k].tolist() != ol[i].tolist():
                    assert top_gap(st.draft_logits[i], k) <= MARGIN, f"draft list mismatch seq {b} head {i} step {step_i}"
            override[b] = [np.asarray(a, np.int64).tolist() + [0] * (16 - len(a)) for a in ol]
            sts[b] = (st, ol)
        dev.verify(TreeArrays(tree.parent, tree.rank), tau_i, override=override)
        tok = dev.debug(DBG.TREE_TOK)
        logits = dev.debug(DBG.LOGITS)
        edge = dev.debug(DBG.EDGE_OK)
        path = dev.debug(DBG.PATH)
        forced = {}
        for b, (st, ol) in sts.items():
            r = O.step(model, st, tree, tau_i, draft_override=ol, ignore_eos=True)
            assert tok[b].tolist() == r["tok"].tolist(), f"tree tokens differ seq {b} step {step_i}"
            for n in range(tree.n_nodes):
                e = rel_l2(logits[b, n], r["logits"][n])
                max_err = max(max_err, e)
                assert e < tol, f"logits seq {b} node {n} step {step_i}: rel-L2 {e}"
            flipped = False
            for n in range(1, tree.n_nodes):
                z = r["logits"][tree.parent[n]]
                t = int(r["tok"][n])
                want = int((z > z[t]).sum() + (z[:t] == z[t]).sum()) < tau_i
                if bool(edge[b, n]) != want:
                    assert edge_margin(z, t, tau_i) <= MARGIN, f"edge decision differs seq {b} node {n} step {step_i}"
                    flipped = True
            got = path[b, 1:1 + path[b, 0]].tolist()
            if not flipped:
                assert got == r["path"], f"path differs seq {b} step {step_i}: {got} vs {r['path']}"
            elif got != r["path"]:
                forced[b] = r["path"]
            compared += 1
        for b in range(B):
            if b in forced:
                dev.kv_compact(b, forced[b])
            else:
                dev.kv_compact(b)
        L = dev.debug(DBG.KV_LEN)
        for b, (st, _) in sts.items():
            assert L[b] == st.L, f"L differs seq {b} step {step_i}"
            assert dev.read_output(b).tolist() == st.emitted, f"output differs seq {b} step {step_i}"
    for b, st in states.items():
        for l in kv_layers:
            for which, ref in ((0, st.K), (1, st.V)):
                e = rel_l2(dev.read_kv(l, b, which, 0, st.L), ref[l, :st.L])
                assert e < tol, f"KV layer {l} seq {b} which {which}: rel-L2 {e}"
    dev.close()
    return compared, skipped, max_err
