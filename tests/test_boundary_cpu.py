"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and its host-only helpers validate configurations and trees."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2410_21951_amd import vadusa as V
from synth import PRESETS, make_tree, chain_tree, full_tree

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return V.load_library()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "vadusa.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(vadusa_[a-z_]+)\s*\(", hdr))
    assert declared == set(V.EXPORTS), declared ^ set(V.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_the_library_with_timing_points_exports_the_same_symbols():
    """libvadusa_clock.so (the step kernel's timing points compiled in; the binding loads it when
    VADUSA_PHASE_CLOCK is set) is the same library otherwise."""
    path = V._LIB_CLOCK_PATH
    assert os.path.exists(path), "build it with `python -m paper_2410_21951_amd.build`"
    clock = V.load_library(path)
    for name in V.EXPORTS:
        assert getattr(clock, name) is not None


def _cfg(model, **kw):
    c = V.make_config(model, kw.pop("max_batch", 1), kw.pop("max_tree_nodes", 64))
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def test_config_check_and_sizes(lib):
    for wl in PRESETS.values():
        c = _cfg(wl.model, max_batch=wl.batch, max_tree_nodes=wl.tree_nodes)
        msg = C.create_string_buffer(256)
        assert lib.vadusa_config_check(C.byref(c), msg, 256) == 0, msg.value
        m = wl.model
        d, F, V1 = m.d_model, m.d_ffn, m.n_logits
        per_layer = 4 * d + 3 * d * d + 3 * d + d * d + d + F * d + F + d * F + d
        want = (m.text_vocab + V1 + m.max_positions) * d + m.n_layers * per_layer + 2 * d + V1 * d \
            + m.n_draft_heads * (d * d + d + V1 * d)
        assert lib.vadusa_blob_floats(C.byref(c)) == want
        kv = 2 * m.n_layers * wl.batch * m.max_positions * d * (2 if m.dtype == "bf16" else 4)
        assert lib.vadusa_arena_bytes(C.byref(c)) > kv
    m = PRESETS["tiny"].model
    msg = C.create_string_buffer(256)
    assert lib.vadusa_config_check(C.byref(_cfg(m, head_dim=32)), msg, 256) == -2 and b"head_dim" in msg.value
    assert lib.vadusa_config_check(C.byref(_cfg(m, dtype=2)), msg, 256) == -1
    assert lib.vadusa_config_check(C.byref(_cfg(m, n_draft_heads=9)), msg, 256) == -2
    assert lib.vadusa_config_check(C.byref(_cfg(m, max_tree_nodes=129)), msg, 256) == -2
    assert lib.vadusa_config_check(C.byref(_cfg(m, prefill_chunk=-1)), msg, 256) == -1
    assert lib.vadusa_config_check(C.byref(_cfg(m, prefill_chunk=1025)), msg, 256) == -2
    assert lib.vadusa_config_check(C.byref(_cfg(m, prefill_chunk=256)), msg, 256) == 0
    small, big = _cfg(m), _cfg(m, prefill_chunk=256)
    assert lib.vadusa_arena_bytes(C.byref(big)) > lib.vadusa_arena_bytes(C.byref(small))
    assert lib.vadusa_config_check(None, msg, 256) == -1
    assert lib.vadusa_arena_bytes(C.byref(_cfg(m, head_dim=32))) == 0


def _check(lib, cfg, parent, rank):
    t = V.TreeArrays(parent, rank)
    msg = C.create_string_buffer(256)
    return lib.vadusa_tree_check(C.byref(cfg), C.byref(t.c), msg, 256), msg.value.decode()


def test_tree_check(lib):
    cfg = _cfg(PRESETS["valle_b1"].model, max_tree_nodes=128)
    for tree in (make_tree(64, (10,) * 4), make_tree(128, (10,) * 4), chain_tree(5), chain_tree(1),
                 full_tree((3, 2, 2))):
        rc, msg = _check(lib, cfg, tree.parent, tree.rank)
        assert rc == 0, msg
    assert _check(lib, cfg, [0, 0], [0, 0])[0] == -1                 # parent[0] must be -1
    assert _check(lib, cfg, [-1, 1], [0, 0])[0] == -1                # parent must precede
    assert _check(lib, cfg, [-1, 0, 0], [0, 1, 0])[0] == -1          # siblings out of order
    assert _check(lib, cfg, [-1, 0, 0], [0, 1, 1])[0] == -1          # equal siblings
    assert _check(lib, cfg, [-1, 0, 1, 0], [0, 0, 0, 1])[0] == -1    # depth order broken
    assert _check(lib, cfg, [-1, 0], [0, 16])[0] == -1               # rank too large
    rc, msg = _check(lib, cfg, chain_tree(6).parent, chain_tree(6).rank)
    assert rc == -1 and "deeper" in msg                              # 5 levels, 4 heads
    small = _cfg(PRESETS["valle_b1"].model, max_tree_nodes=32)
    assert _check(lib, small, make_tree(64, (10,) * 4).parent, make_tree(64, (10,) * 4).rank)[0] == -1


def test_blob_order_matches_generator():
    from synth import weight_names
    for wl in (PRESETS["tiny"], PRESETS["longform_b1"]):
        assert [n for n, _, _ in weight_names(wl.model)] == V.blob_order(wl.model)


def test_build_tree_matches_bruteforce_and_reference_generator():
    """vadusa_build_tree (Sec. 2.4): the chosen set is ancestor-closed, canonical, and has the
    largest expected accepted length of all ancestor-closed sets of its size (brute force on a
    small full tree); on larger tables it picks the same nodes as an independent best-first
    search written in Python."""
    import heapq
    import itertools
    import numpy as np
    from paper_2410_21951_amd import build_tree, VadusaError
    rng = np.random.default_rng(5)
    # brute force: 2 heads x 3 ranks -> 1 + 3 + 9 = 13 nodes, choose the best 6
    acc = rng.uniform(0.05, 0.9, (2, 3)).astype(np.float32)
    t = build_tree(acc, 6)
    paths = [()] + [(r,) for r in range(3)] + [(a, b) for a in range(3) for b in range(3)]
    prob = {p: float(np.prod([np.float64(acc[i][r]) for i, r in enumerate(p)])) for p in paths}
    best = max((sum(prob[p] for p in sub), sub) for sub in itertools.combinations(paths, 6)
               if () in sub and all(p[:-1] in sub for p in sub if p))
    got = []
    for n in range(t.n_nodes):
        p, m = [], n
        while m > 0:
            p.append(int(t.rank[m])); m = int(t.parent[m])
        got.append(tuple(reversed(p)))
    assert sorted(got) == sorted(best[1])
    assert got == sorted(got, key=lambda p: (len(p), p))          # canonical order
    # larger: 4 heads x 10 ranks, 64 nodes, against a heap-based search
    acc = np.sort(rng.uniform(0.01, 0.8, (4, 10)).astype(np.float32), axis=1)[:, ::-1].copy()
    t = build_tree(acc, 64)
    heap, chosen = [(-1.0, 0, ())], []
    while len(chosen) < 64:
        negp, dep, path = heapq.heappop(heap)
        chosen.append(path)
        if dep < 4:
            for r in range(10):
                heapq.heappush(heap, (negp * float(np.float64(acc[dep][r])), dep + 1, path + (r,)))
    want = sorted(chosen, key=lambda p: (len(p), p))
    got = []
    for n in range(t.n_nodes):
        p, m = [], n
        while m > 0:
            p.append(int(t.rank[m])); m = int(t.parent[m])
        got.append(tuple(reversed(p)))
    assert got == want
    # the library accepts its own tree, and refuses bad arguments
    with pytest.raises(VadusaError):
        build_tree(np.full((2, 3), 1.5, np.float32), 4)
    with pytest.raises(VadusaError):
        build_tree(acc, 500)


def test_bench_prices_the_step_as_the_paper_sized_model_implies():
    """bench.py's algorithmic bytes and flops per step, against the figures that follow from the
    model sizes of Sec. 3.1.1 (12 layers, d = 1024, FFN 4096, 1025 logits, four draft heads, bf16):
    302.0 MB of layer weights, 2.1 MB vocabulary map, 16.8 MB draft heads, 48 KiB of K/V per position."""
    import importlib.util
    import os
    spec = importlib.util.spec_from_file_location("bench", os.path.join(os.path.dirname(os.path.dirname(__file__)), "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    m = PRESETS["valle_b1"].model
    weights = (12 * (4 * 1024 * 1024 + 2 * 1024 * 4096) + 1025 * 1024 + 4 * (1024 * 1024 + 1025 * 1024)) * 2
    kv = 12 * 2 * 1024 * 2
    assert kv == 48 * 1024
    for L in (289, 664, 1039):
        assert bench.algorithmic_bytes(m, 1, 64, L) == weights + (L + 64) * kv
    assert abs(bench.algorithmic_bytes(m, 1, 64, 664) / 1e6 - 356.7) < 0.5
    # 64 rows through the layers and the base head, one row through the draft heads, attention over
    # L + M/2 keys: 19.5 GFLOP of maps + attention
    f = bench.algorithmic_flops(m, 1, 64, 664)
    maps = 2 * 64 * (12 * (4 * 1024 * 1024 + 2 * 1024 * 4096) + 1025 * 1024) + 2 * 4 * (1024 * 1024 + 1025 * 1024)
    assert abs(f - (maps + 4 * 64 * (664 + 32) * 1024 * 12)) < 1e-6 * f
    assert 19.4e9 < maps < 19.6e9
