"""Child process of tests/test_emulated_kernel.py: one lockstep run of the emulated kernels
against the oracle.  usage: run_case.py <libvadusa_emu.so> <dtype | bf16-40rows>"""
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, HERE)
sys.path.insert(0, os.path.dirname(HERE))
import emulate
emulate.install(sys.argv[1])
import numpy as np
from synth import ModelConfig, make_weights, make_tree, make_uniforms
from parity import Lockstep

dtype = sys.argv[2]
if dtype == "bf16-40rows":
    # More than 32 rows: QKV and FFN1 run as 32 x 32 units, the second row block ragged (rows
    # 32..39: one row tile of two); two layers, so the per-layer advance of the descriptor table counts.
    cfg = ModelConfig(n_layers=2, d_model=64, n_heads=1, head_dim=64, d_ffn=192, speech_vocab=71, text_vocab=20,
                      n_draft_heads=2, max_positions=192, dtype="bf16")
    W = make_weights(cfg, 71, std=0.05)
    rng = np.random.default_rng(72)
    text = [rng.integers(0, cfg.text_vocab, 2).astype(np.int32)]
    prompt = [rng.integers(0, cfg.speech_vocab, 45).astype(np.int32)]
    tree = make_tree(40, (10, 10))
    t0 = time.time()
    ls = Lockstep(cfg, W, text, prompt, 40)
    ls.step(tree, 2)
    ls.step(tree, 1)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    print(f"emulated {dtype}: compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e} "
          f"ties {s.tie_root}/{s.tie_list}/{s.tie_edge} in {time.time() - t0:.0f} s", flush=True)
    assert s.compared >= 1
    sys.stdout.flush()
    os._exit(0)
if dtype == "bf16-72rows":
    # 65 to 255 rows: the kernel variant whose QKV / FFN1 run as 64 x 32 units and whose residual maps run as
    # 32 x 16 units; 72 rows leave the second row block of 64 (and the third of 32) ragged.  The prompt of 70 tokens
    # goes through one causal pass of 72 rows (the same variant for the prefill).
    cfg = ModelConfig(n_layers=2, d_model=64, n_heads=1, head_dim=64, d_ffn=192, speech_vocab=71, text_vocab=20,
                      n_draft_heads=3, max_positions=224, dtype="bf16")
    W = make_weights(cfg, 81, std=0.05)
    rng = np.random.default_rng(82)
    text = [rng.integers(0, cfg.text_vocab, 3).astype(np.int32)]
    prompt = [rng.integers(0, cfg.speech_vocab, 67).astype(np.int32)]
    tree = make_tree(72, (10, 10, 10))
    t0 = time.time()
    ls = Lockstep(cfg, W, text, prompt, 72)
    ls.step(tree, 2)
    ls.check_kv(layers=[0, 1])
    s = ls.stats
    print(f"emulated {dtype}: compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e} "
          f"ties {s.tie_root}/{s.tie_list}/{s.tie_edge} in {time.time() - t0:.0f} s", flush=True)
    assert s.compared >= 1
    sys.stdout.flush()
    os._exit(0)
if dtype == "bf16-256rows":
    # 256 rows (8 sequences x 32 nodes): the many-row kernel, its 128 x 128 units forced on for these small maps (value
    # columns through LDS as 16-byte pieces with ragged cache positions, query / key / GELU outputs as pieces swapped
    # between lanes 16 apart, a last column block of 64 of the 192-wide FFN), 64 x 64 units for the residual maps and
    # the vocabulary map, whole-head attention units of two (sequence, head) pairs, four rows per embedding unit,
    # compaction units over layers.
    os.environ["VADUSA_BIG_MIN_UNITS"] = "1"
    cfg = ModelConfig(n_layers=1, d_model=64, n_heads=1, head_dim=64, d_ffn=192, speech_vocab=71, text_vocab=20,
                      n_draft_heads=2, max_positions=64, dtype="bf16")
    W = make_weights(cfg, 91, std=0.05)
    rng = np.random.default_rng(92)
    text = [rng.integers(0, cfg.text_vocab, int(rng.integers(1, 4))).astype(np.int32) for _ in range(8)]
    prompt = [rng.integers(0, cfg.speech_vocab, int(rng.integers(3, 12))).astype(np.int32) for _ in range(8)]
    tree = make_tree(32, (6, 6))
    t0 = time.time()
    ls = Lockstep(cfg, W, text, prompt, 32)
    ls.step(tree, 2)
    ls.check_kv(layers=[0])
    s = ls.stats
    print(f"emulated {dtype}: compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e} "
          f"ties {s.tie_root}/{s.tie_list}/{s.tie_edge} in {time.time() - t0:.0f} s", flush=True)
    assert s.compared >= 1
    sys.stdout.flush()
    os._exit(0)
if dtype == "bf16-giveup":
    # the failure path: the host raises the error word of a kernel that gave up at a grid barrier; the next
    # synchronising call reports it, later calls refuse, a prefill recovers and decodes the same tokens
    from paper_2410_21951_amd import Vadusa, TreeArrays, VadusaError, DBG
    cfg = ModelConfig(n_layers=1, d_model=64, n_heads=1, head_dim=64, d_ffn=128, speech_vocab=70, text_vocab=20,
                      n_draft_heads=2, max_positions=64, dtype="bf16")
    W = make_weights(cfg, 71, std=0.08)
    rng = np.random.default_rng(73)
    text = [rng.integers(0, cfg.text_vocab, 3).astype(np.int32)]
    prompt = [rng.integers(0, cfg.speech_vocab, 9).astype(np.int32)]
    t = make_tree(8, (3, 2))
    tree = TreeArrays(t.parent, t.rank)
    dev = Vadusa(cfg, max_batch=1, max_tree_nodes=8, ignore_eos=True)
    dev.load_weights(W)

    def run():
        dev.prefill(text, prompt)
        return [dev.step(tree, 1 + i % 2) for i in range(3)]
    want = run()
    dev.debug_raise_error()
    codes = []
    for call in (lambda: dev.step(tree, 1), lambda: dev.debug(DBG.ROOT), lambda: dev.step(tree, 1)):
        try:
            call()
            codes.append(0)
        except VadusaError as e:
            codes.append(e.code)
    assert codes == [-5, -4, -4], codes
    assert run() == want
    print("emulated give-up path: reported, refused, recovered", flush=True)
    sys.stdout.flush()
    os._exit(0)
if dtype in ("bf16-nan", "fp32-nan"):
    # A model whose logits are all NaN (a NaN in the final LayerNorm's scale): no row has a largest entry, so the
    # arg-max and the draft lists have nothing to return.  The step must still stay inside its buffers (the arena sits
    # between guard pages) and hand back token ids of the vocabulary.
    from paper_2410_21951_amd import Vadusa, TreeArrays
    cfg = ModelConfig(n_layers=1, d_model=64, n_heads=1, head_dim=64, d_ffn=128, speech_vocab=70, text_vocab=20,
                      n_draft_heads=2, max_positions=64, dtype=dtype[:4])
    W = make_weights(cfg, 71, std=0.08)
    W["lnf_g"] = W["lnf_g"].copy()
    W["lnf_g"][3] = np.nan
    rng = np.random.default_rng(74)
    text = [rng.integers(0, cfg.text_vocab, 3).astype(np.int32)]
    prompt = [rng.integers(0, cfg.speech_vocab, 9).astype(np.int32)]
    t = make_tree(8, (3, 2))
    tree = TreeArrays(t.parent, t.rank)
    dev = Vadusa(cfg, max_batch=1, max_tree_nodes=8, ignore_eos=True)
    dev.load_weights(W)
    dev.prefill(text, prompt)
    for i in range(3):
        out = dev.step(tree, 1 + i % 2)
        for toks in out:
            assert all(0 <= int(v) <= cfg.speech_vocab for v in toks), toks
    print("emulated NaN logits: stayed in bounds", flush=True)
    sys.stdout.flush()
    os._exit(0)
cfg = ModelConfig(n_layers=1, d_model=64, n_heads=1, head_dim=64, d_ffn=128, speech_vocab=70, text_vocab=20,
                  n_draft_heads=2, max_positions=64, dtype=dtype)
W = make_weights(cfg, 71, std=0.08)
rng = np.random.default_rng(72)
text = [rng.integers(0, cfg.text_vocab, 2).astype(np.int32), rng.integers(0, cfg.text_vocab, 3).astype(np.int32)]
prompt = [rng.integers(0, cfg.speech_vocab, 9).astype(np.int32), rng.integers(0, cfg.speech_vocab, 5).astype(np.int32)]
tree = make_tree(8, (3, 2))
t0 = time.time()
ls = Lockstep(cfg, W, text, prompt, 8)
for tau in (1, 3):
    ls.step(tree, tau)
# the stochastic rule on a 4-node tree (its kernel does not depend on the model's dtype, so the
# search regimes run once): every token kept for the bf16 model, whose step launch is split around
# the perturbation; a nucleus cut and a nucleus smaller than tau for the fp32 model
small = make_tree(4, (2, 1))
regimes = ((2, 0.9, 1.0),) if dtype == "bf16" else ((3, 1.0, 0.7), (4, 0.5, 0.02))
for i, (tau, T, top_p) in enumerate(regimes):
    ls.step(small, tau, sample=(T, top_p, make_uniforms(73, i, 2, small.n_nodes, cfg.speech_vocab + 1)))
ls.step(tree, 1)
ls.check_kv(layers=[0])
s = ls.stats
print(f"emulated {dtype}: compared {s.compared}/{s.steps} logit err {s.max_logit_err:.2e} score err "
      f"{s.max_score_err:.2e} nucleus sizes {[round(x, 1) for x in s.nucleus_sizes]} ties {s.tie_root}/{s.tie_list}/{s.tie_edge} in {time.time() - t0:.0f} s", flush=True)
assert s.compared >= 1
sys.stdout.flush()
os._exit(0)   # the emulation's worker threads never end
