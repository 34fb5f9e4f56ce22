"""GPU tests of the C ABI's behaviour: call order, error codes, the one-call step
against verify + compact, asynchronous stepping, run-to-run reproducibility."""
import numpy as np
import pytest

from synth import ModelConfig, make_weights, make_tree, chain_tree

pytestmark = pytest.mark.gpu

CFG = ModelConfig(n_layers=2, d_model=128, n_heads=2, head_dim=64, d_ffn=512, speech_vocab=300,
                  text_vocab=50, n_draft_heads=3, max_positions=160, dtype="bf16")


def _dev(cfg=CFG, **kw):
    from paper_2410_21951_amd import Vadusa
    return Vadusa(cfg, **kw)


def _tree(t):
    from paper_2410_21951_amd import TreeArrays
    return TreeArrays(t.parent, t.rank)


def _inputs(rng, B=2):
    text = [rng.integers(0, CFG.text_vocab, 5 + b).astype(np.int32) for b in range(B)]
    prompt = [rng.integers(0, CFG.speech_vocab, 20 + 3 * b).astype(np.int32) for b in range(B)]
    return text, prompt


def test_call_order_and_argument_errors():
    from paper_2410_21951_amd import VadusaError
    print("api errors", flush=True)
    W = make_weights(CFG, 3)
    rng = np.random.default_rng(0)
    text, prompt = _inputs(rng)
    dev = _dev(max_batch=2, max_tree_nodes=16)
    tree = _tree(make_tree(16, (4, 2, 2)))
    with pytest.raises(VadusaError) as e:
        dev.prefill(text, prompt)                       # weights not loaded
    assert e.value.code == -4
    dev.load_weights(W)
    dev.batch = 2
    with pytest.raises(VadusaError) as e:
        dev.step(tree, 1)                               # step before prefill
    assert e.value.code == -4
    dev.prefill(text, prompt)
    with pytest.raises(VadusaError) as e:
        dev.step(tree, 0)                               # tau < 1
    assert e.value.code == -1
    with pytest.raises(VadusaError) as e:
        dev.step(_tree(make_tree(17, (4, 2, 2))), 1)    # more nodes than max_tree_nodes
    assert e.value.code == -1
    with pytest.raises(VadusaError) as e:
        dev.kv_compact(-1)                              # nothing pending
    assert e.value.code == -4
    with pytest.raises(VadusaError) as e:
        dev.prefill([np.array([999], np.int32)] * 2, prompt)   # token outside the vocabulary
    assert e.value.code == -1
    with pytest.raises(VadusaError) as e:
        dev.prefill(text, [np.zeros(150, np.int32)] * 2)       # no room for the tree rows
    assert e.value.code == -3
    # state survived the failed calls
    out = dev.step(tree, 1)
    assert all(len(o) >= 1 for o in out)
    dev.verify(tree, 1)
    with pytest.raises(VadusaError) as e:
        dev.verify(tree, 1)                             # compaction still pending
    assert e.value.code == -4
    with pytest.raises(VadusaError) as e:
        dev.kv_compact(0, [0, 5])                       # node 5 is not a child of the root
    assert e.value.code == -1
    dev.kv_compact(0, [0, 1])
    with pytest.raises(VadusaError) as e:
        dev.kv_compact(0)                               # sequence 0 already compacted
    assert e.value.code == -4
    dev.kv_compact(1)
    dev.step(tree, 2)


def test_kv_full_is_reported_not_overrun():
    from paper_2410_21951_amd import VadusaError
    print("kv full", flush=True)
    W = make_weights(CFG, 3)
    rng = np.random.default_rng(1)
    dev = _dev(max_batch=1, max_tree_nodes=16, ignore_eos=True)
    dev.load_weights(W)
    dev.prefill([np.zeros(4, np.int32)], [rng.integers(0, 300, 130).astype(np.int32)])
    tree = _tree(chain_tree(4))
    n = 0
    with pytest.raises(VadusaError) as e:
        for _ in range(40):
            n += len(dev.step(tree, 301)[0])            # accepts 4 tokens per step
    assert e.value.code == -3
    assert 134 + n + 4 > 160 and 134 + n <= 160
    assert len(dev.read_output(0)) == n


def test_step_equals_verify_plus_compact_and_async_and_reproducible():
    from paper_2410_21951_amd import DBG
    print("step paths", flush=True)
    W = make_weights(CFG, 4, std=0.08)
    rng = np.random.default_rng(2)
    text, prompt = _inputs(rng)
    tree = _tree(make_tree(16, (4, 2, 2)))
    outs, logits = [], []
    for mode in ("sync", "split", "async", "sync"):
        dev = _dev(max_batch=2, max_tree_nodes=16, ignore_eos=True)
        dev.load_weights(W)
        dev.prefill(text, prompt)
        for i in range(12):
            tau = 1 + i % 3
            if mode == "sync":
                dev.step(tree, tau)
            elif mode == "async":
                dev.step(tree, tau, sync=False)
            else:
                dev.verify(tree, tau)
                dev.kv_compact(-1)
        outs.append([dev.read_output(b).tolist() for b in range(2)])
        logits.append(dev.debug(DBG.LOGITS).copy())
        dev.close()
    assert outs[0] == outs[1] == outs[2] == outs[3]
    for l in logits[1:]:
        assert np.array_equal(logits[0], l)             # bit-reproducible
    assert all(len(o) >= 12 for o in outs[0])


def test_a_kernel_that_gave_up_is_reported_and_prefill_recovers():
    """The failure path of the persistent kernel without disturbing any kernel: the host sets the error word a
    workgroup raises when its bounded barrier wait runs out.  The next synchronising call reports VADUSA_EHIP,
    every later call (the debug readers included) refuses with VADUSA_ESTATE, vadusa_prefill resets the barrier
    state, and the context then decodes the same tokens as a fresh one."""
    from paper_2410_21951_amd import VadusaError, DBG
    print("give-up path", flush=True)
    W = make_weights(CFG, 4, std=0.08)
    rng = np.random.default_rng(2)
    text, prompt = _inputs(rng)
    tree = _tree(make_tree(16, (4, 2, 2)))

    def run(dev):
        dev.prefill(text, prompt)
        return [dev.step(tree, 1 + i % 3) for i in range(6)]

    ref = _dev(max_batch=2, max_tree_nodes=16, ignore_eos=True)
    ref.load_weights(W)
    want = run(ref)
    ref.close()
    dev = _dev(max_batch=2, max_tree_nodes=16, ignore_eos=True)
    dev.load_weights(W)
    dev.prefill(text, prompt)
    dev.step(tree, 1)
    for how in ("sync step", "async step then reader"):
        dev.debug_raise_error()
        with pytest.raises(VadusaError) as e:
            if how == "sync step":
                dev.step(tree, 1)
            else:
                dev.step(tree, 1, sync=False)            # nothing is checked here ...
                dev.debug(DBG.ROOT)                      # ... the reader must not hand out that launch's data
        assert e.value.code == -5, how                   # VADUSA_EHIP
        for call in (lambda: dev.step(tree, 1), lambda: dev.debug(DBG.LOGITS), lambda: dev.read_kv(0, 0, 0, 0, 4),
                     lambda: dev.read_output(0), lambda: dev.verify(tree, 1)):
            with pytest.raises(VadusaError) as e2:
                call()
            assert e2.value.code == -4, how              # VADUSA_ESTATE until the prefill
        assert run(dev) == want, how
    dev.close()


def test_stochastic_entry_points():
    """vadusa_step_sampled = vadusa_verify_sampled + vadusa_kv_compact; uniforms from host or
    device memory give the same stream; argument errors are reported, not run."""
    import ctypes as C
    import torch
    from paper_2410_21951_amd import DBG, VadusaError
    from paper_2410_21951_amd.vadusa import _Sampling
    from synth import make_uniforms
    print("stochastic entry points", flush=True)
    W = make_weights(CFG, 4, std=0.08)
    rng = np.random.default_rng(6)
    text, prompt = _inputs(rng)
    tree = _tree(make_tree(16, (4, 2, 2)))
    outs = []
    for mode in ("step", "split", "device"):
        dev = _dev(max_batch=2, max_tree_nodes=16, ignore_eos=True)
        dev.load_weights(W)
        dev.prefill(text, prompt)
        for i in range(8):
            u = make_uniforms(9, i, 2, 16, CFG.n_logits)
            smp = (0.9, 0.9, u)
            if mode == "step":
                dev.step(tree, 1 + 5 * (i % 3), sample=smp)
            elif mode == "split":
                dev.verify(tree, 1 + 5 * (i % 3), sample=smp)
                dev.kv_compact(-1)
            else:
                dev.step(tree, 1 + 5 * (i % 3), sample=(0.9, 0.9, torch.from_numpy(u).cuda()), sync=False)
        outs.append([dev.read_output(b).tolist() for b in range(2)])
        if mode == "step":
            sc = dev.debug(DBG.SCORES)
            assert np.isfinite(sc).any() and np.isinf(sc).any()
            # errors: nothing runs, the context stays usable
            u = make_uniforms(9, 99, 2, 16, CFG.n_logits)
            for bad in ((0.0, 0.9), (-1.0, 0.9), (float("nan"), 0.9), (1.0, 0.0), (1.0, -0.5)):
                with pytest.raises(VadusaError) as e:
                    dev.step(tree, 1, sample=(bad[0], bad[1], u))
                assert e.value.code != 0
            sp = _Sampling(1.0, 1.0, None, 0)
            assert dev.lib.vadusa_step_sampled(dev.h, C.byref(tree.c), 1, C.byref(sp), None, None, None) != 0
            assert dev.lib.vadusa_step_sampled(dev.h, C.byref(tree.c), 1, None, None, None, None) != 0
            dev.step(tree, 1)                       # a deterministic step: no scores to read afterwards
            with pytest.raises(VadusaError):
                dev.debug(DBG.SCORES)
        dev.close()
    assert outs[0] == outs[1] == outs[2]
    assert all(len(o) >= 8 for o in outs[0])


def test_stochastic_rule_refuses_vocabularies_beyond_its_lds_row():
    """The perturbation kernel keeps a row of V + 1 floats in 64 KiB of LDS: a larger vocabulary is
    refused with VADUSA_ESHAPE before anything runs; the deterministic step still works."""
    from paper_2410_21951_amd import VadusaError
    from synth import make_uniforms
    print("stochastic rule, vocabulary too large", flush=True)
    cfg = ModelConfig(n_layers=1, d_model=64, n_heads=1, head_dim=64, d_ffn=128, speech_vocab=16400,
                      text_vocab=20, n_draft_heads=2, max_positions=64, dtype="bf16")
    W = make_weights(cfg, 5, std=0.05)
    rng = np.random.default_rng(3)
    dev = _dev(cfg, max_batch=1, max_tree_nodes=8, ignore_eos=True)
    dev.load_weights(W)
    dev.prefill([rng.integers(0, 20, 3).astype(np.int32)], [rng.integers(0, 16400, 9).astype(np.int32)])
    tree = _tree(make_tree(8, (3, 2)))
    with pytest.raises(VadusaError) as e:
        dev.step(tree, 2, sample=(1.0, 0.9, make_uniforms(1, 0, 1, 8, cfg.n_logits)))
    assert e.value.code == -2
    assert len(dev.step(tree, 2)[0]) >= 1
    dev.close()
