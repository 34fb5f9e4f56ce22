"""GPU test of vadusa_debug_read_kv_static, the entry point for callers that cannot allocate: it stages the
rows in the library's static device array instead of the arena.  Its output must equal that of
vadusa_debug_read_kv bit for bit (same kernel, other staging memory), on two calls in a row, the second with
a smaller range (the array keeps the first call's rows behind the second call's), for K and V, an fp32 and a
bf16 model; a range beyond the array's size is refused."""
import numpy as np
import pytest

from synth import ModelConfig, make_weights, make_tree

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_static_staging_equals_arena_staging(dtype):
    from paper_2410_21951_amd import Vadusa, TreeArrays, VadusaError
    print(f"no-alloc KV read, {dtype}", flush=True)
    cfg = ModelConfig(n_layers=2, d_model=128, n_heads=2, head_dim=64, d_ffn=512, speech_vocab=300,
                      text_vocab=50, n_draft_heads=3, max_positions=4096, dtype=dtype)
    W = make_weights(cfg, 5, std=0.05)
    rng = np.random.default_rng(6)
    text = [rng.integers(0, cfg.text_vocab, 7 + b).astype(np.int32) for b in range(2)]
    prompt = [rng.integers(0, cfg.speech_vocab, 40 + 9 * b).astype(np.int32) for b in range(2)]
    t = make_tree(16, (4, 2, 2))
    tree = TreeArrays(t.parent, t.rank)
    dev = Vadusa(cfg, max_batch=2, max_tree_nodes=16, ignore_eos=True)
    dev.load_weights(W)
    dev.prefill(text, prompt)
    for i in range(3):
        dev.step(tree, 1 + i)
    for layer, seq, which in ((0, 0, 0), (1, 1, 1)):
        for pos0, npos in ((0, 45), (3, 11)):              # the second call is the smaller one
            want = dev.read_kv(layer, seq, which, pos0, npos)
            got = dev.read_kv(layer, seq, which, pos0, npos, static=True)
            assert np.abs(want).max() > 0
            assert np.array_equal(got, want), (layer, seq, which, pos0, npos)
    # 262 144 floats = 2048 rows of 128: one row more is refused before anything is launched
    assert dev.read_kv(0, 0, 0, 0, 2048, static=True).shape == (2048, 128)
    with pytest.raises(VadusaError) as e:
        dev.read_kv(0, 0, 0, 0, 2049, static=True)
    assert e.value.code == -2                               # VADUSA_ESHAPE
    assert np.array_equal(dev.read_kv(0, 1, 0, 2, 5, static=True), dev.read_kv(0, 1, 0, 2, 5))
    dev.close()
