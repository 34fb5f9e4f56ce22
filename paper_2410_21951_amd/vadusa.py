"""ctypes binding of the C ABI in include/vadusa.h.

Argument marshalling only: every step of the decode path runs inside the
library's HIP kernels.  PyTorch is used to allocate the device arena and to
supply the stream.  There is no CPU fallback: if the library is missing or no
GPU is present, construction fails.
"""
import atexit
import ctypes as C
import os
import weakref

import numpy as np

MAX_TREE_NODES = 128
MAX_TOPK = 16
MAX_DRAFT_HEADS = 8

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libvadusa.so")
_LIB_CLOCK_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libvadusa_clock.so")
_lib = None


class VadusaError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"vadusa error {code}: {text}")
        self.code = code


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "speech_vocab", "text_vocab",
        "n_draft_heads", "max_positions", "max_batch", "max_tree_nodes", "dtype", "ignore_eos",
        "prefill_chunk")]


class _Tree(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("parent", C.POINTER(C.c_int32)), ("rank", C.POINTER(C.c_int32))]


class _Sampling(C.Structure):
    _fields_ = [("temperature", C.c_float), ("top_p", C.c_float), ("uniforms", C.c_void_p),
                ("uniforms_on_device", C.c_int32)]


class DBG:
    (LOGITS, H_NODES, TREE_TOK, DRAFT_TOPK, KV_LEN, ROOT, EDGE_OK, PATH, FINISHED, DRAFT_LOGITS, PHASE_CLOCK,
     SCORES) = range(12)


EXPORTS = {
    "vadusa_config_check": (C.c_int, [C.POINTER(_Config), C.c_char_p, C.c_size_t]),
    "vadusa_tree_check": (C.c_int, [C.POINTER(_Config), C.POINTER(_Tree), C.c_char_p, C.c_size_t]),
    "vadusa_build_tree": (C.c_int, [C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                    C.POINTER(C.c_int32)]),
    "vadusa_arena_bytes": (C.c_size_t, [C.POINTER(_Config)]),
    "vadusa_blob_floats": (C.c_size_t, [C.POINTER(_Config)]),
    "vadusa_create": (C.c_int, [C.POINTER(_Config), C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]),
    "vadusa_destroy": (None, [C.c_void_p]),
    "vadusa_last_error": (C.c_char_p, [C.c_void_p]),
    "vadusa_load_weights": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]),
    "vadusa_prefill": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "vadusa_verify": (C.c_int, [C.c_void_p, C.POINTER(_Tree), C.c_int32, C.c_void_p]),
    "vadusa_kv_compact": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32]),
    "vadusa_step": (C.c_int, [C.c_void_p, C.POINTER(_Tree), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "vadusa_verify_sampled": (C.c_int, [C.c_void_p, C.POINTER(_Tree), C.c_int32, C.POINTER(_Sampling), C.c_void_p]),
    "vadusa_step_sampled": (C.c_int, [C.c_void_p, C.POINTER(_Tree), C.c_int32, C.POINTER(_Sampling), C.c_void_p,
                                      C.c_void_p, C.c_void_p]),
    "vadusa_read_output": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]),
    "vadusa_debug_read": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t]),
    "vadusa_debug_read_kv": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]),
    "vadusa_debug_raise_error": (C.c_int, [C.c_void_p]),
    "vadusa_debug_read_kv_static": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]),
}


def load_library(path=None):
    """dlopen libvadusa.so and declare every exported signature."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    # VADUSA_LIB: another build of the same library; with VADUSA_PHASE_CLOCK set, the build that has the timing points
    p = path or os.environ.get("VADUSA_LIB") or (_LIB_CLOCK_PATH if os.environ.get("VADUSA_PHASE_CLOCK") else _LIB_PATH)
    if not os.path.exists(p):
        raise FileNotFoundError(f"{p} not found: build it with `python -m paper_2410_21951_amd.build`")
    lib = C.CDLL(p)
    for name, (res, args) in EXPORTS.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    if path is None:
        _lib = lib
    return lib


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


class TreeArrays:
    """Host arrays of a candidate tree (kept alive as long as the object lives)."""

    def __init__(self, parent, rank):
        self.parent = _i32(parent)
        self.rank = _i32(rank)
        self.n_nodes = int(self.parent.shape[0])
        self.c = _Tree(self.n_nodes, self.parent.ctypes.data_as(C.POINTER(C.c_int32)),
                       self.rank.ctypes.data_as(C.POINTER(C.c_int32)))


def build_tree(acc, n_nodes):
    """Sparse candidate tree from per-head, per-rank acceptance probabilities acc [n_heads][width]
    (vadusa_build_tree; needs no GPU).  Returns TreeArrays."""
    lib = load_library()
    acc = np.ascontiguousarray(acc, dtype=np.float32)
    parent = np.zeros(n_nodes, np.int32)
    rank = np.zeros(n_nodes, np.int32)
    n = C.c_int32(0)
    rc = lib.vadusa_build_tree(acc.shape[0], acc.shape[1], _ptr(acc), int(n_nodes), _ptr(parent), _ptr(rank), C.byref(n))
    if rc:
        raise VadusaError(rc, "vadusa_build_tree: bad arguments")
    return TreeArrays(parent[:n.value], rank[:n.value])


def make_config(model, max_batch, max_tree_nodes, ignore_eos=False, prefill_chunk=0):
    """model: any object or dict with the fields of the model description."""
    g = (lambda k: model[k]) if isinstance(model, dict) else (lambda k: getattr(model, k))
    return _Config(g("n_layers"), g("d_model"), g("n_heads"), g("head_dim"), g("d_ffn"), g("speech_vocab"),
                   g("text_vocab"), g("n_draft_heads"), g("max_positions"), max_batch, max_tree_nodes,
                   {"fp32": 0, "bf16": 1}[g("dtype")], int(bool(ignore_eos)), int(prefill_chunk))


def blob_order(cfg):
    """Tensor names in blob order (the order documented in vadusa.h)."""
    names = ["E_text", "E_speech", "P"]
    for l in range(cfg.n_layers):
        names += [f"L{l}.{k}" for k in ("ln1_g", "ln1_b", "Wqkv", "bqkv", "Wo", "bo",
                                        "ln2_g", "ln2_b", "W1", "b1", "W2", "b2")]
    names += ["lnf_g", "lnf_b", "W_out"]
    for i in range(cfg.n_draft_heads):
        names += [f"D{i}.{k}" for k in ("W1", "b1", "W2")]
    return names


def pack_blob(cfg, weights):
    """Concatenate the named fp32 tensors into the flat blob of vadusa_load_weights."""
    return np.concatenate([np.asarray(weights[n], dtype=np.float32).ravel() for n in blob_order(cfg)])


_OPEN = weakref.WeakSet()   # contexts not yet closed


@atexit.register
def _close_all():
    for v in list(_OPEN):
        v.close()


class Vadusa:
    """One decoding context on the current CUDA/HIP device."""

    def __init__(self, model, max_batch=1, max_tree_nodes=64, ignore_eos=False, stream=None, prefill_chunk=0):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the VADUSA step has no CPU fallback")
        self.lib = load_library()
        self.cfg = make_config(model, max_batch, max_tree_nodes, ignore_eos, prefill_chunk)
        msg = C.create_string_buffer(256)
        rc = self.lib.vadusa_config_check(C.byref(self.cfg), msg, 256)
        if rc:
            raise VadusaError(rc, msg.value.decode())
        nbytes = self.lib.vadusa_arena_bytes(C.byref(self.cfg))
        self._torch = torch
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
        base = (self.arena.data_ptr() + 255) // 256 * 256
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        rc = self.lib.vadusa_create(C.byref(self.cfg), C.c_void_p(base), nbytes,
                                    C.c_void_p(self.stream.cuda_stream), C.byref(h))
        if rc:
            raise VadusaError(rc, "vadusa_create failed")
        self.h = h
        _OPEN.add(self)
        self.batch = 0
        self.M = 0
        self.Hh = self.cfg.n_draft_heads
        self.V1 = self.cfg.speech_vocab + 1

    def close(self):
        """Drains the stream and frees the context.  Idempotent.  Contexts still open at interpreter exit are
        closed by an exit handler that runs before torch's own teardown; __del__ only frees the host object
        (vadusa_destroy makes no HIP call), so a late finaliser cannot touch a runtime that is already gone."""
        if getattr(self, "h", None):
            try:
                self.stream.synchronize()
            except Exception:
                pass
            self.lib.vadusa_destroy(self.h)
            self.h = None
        _OPEN.discard(self)

    def __del__(self):
        h = getattr(self, "h", None)
        if h:
            try:
                self.lib.vadusa_destroy(h)
            except Exception:
                pass
            self.h = None

    def _check(self, rc):
        if rc:
            raise VadusaError(rc, self.lib.vadusa_last_error(self.h).decode())

    # ---- model ----
    def load_weights(self, weights):
        blob = pack_blob(self.cfg, weights)
        self._check(self.lib.vadusa_load_weights(self.h, _ptr(blob), blob.size, 0))

    def load_blob_device(self, blob_tensor):
        self._check(self.lib.vadusa_load_weights(self.h, C.c_void_p(blob_tensor.data_ptr()), blob_tensor.numel(), 1))

    # ---- decoding ----
    def prefill(self, text, prompt):
        """text, prompt: lists (one entry per sequence) of int arrays.  Returns the first roots."""
        B = len(text)
        tl = _i32([len(t) for t in text])
        pl = _i32([len(p) for p in prompt])
        tt = _i32(np.concatenate([_i32(t) for t in text])) if tl.sum() else np.zeros(1, np.int32)
        pt = _i32(np.concatenate([_i32(p) for p in prompt])) if pl.sum() else np.zeros(1, np.int32)
        roots = np.zeros(B, np.int32)
        self._check(self.lib.vadusa_prefill(self.h, B, _ptr(tt), _ptr(tl), _ptr(pt), _ptr(pl), _ptr(roots)))
        self.batch = B
        return roots

    def _override(self, override):
        """override: [B][Hh] lists of ids -> padded int32 [B][Hh][MAX_TOPK] (or None)."""
        if override is None:
            return None
        buf = np.zeros((self.batch, self.Hh, MAX_TOPK), np.int32)
        for b, per_head in enumerate(override):
            for i, ids in enumerate(per_head):
                ids = _i32(ids)
                buf[b, i, :len(ids)] = ids
        return buf

    def _sampling(self, tree, sample):
        """sample = (temperature, top_p, uniforms): uniforms a host array [batch][n_nodes][V+1]
        or a CUDA tensor of that many floats.  Returns (struct, object to keep alive)."""
        temperature, top_p, u = sample
        if hasattr(u, "data_ptr"):
            assert u.is_cuda and u.is_contiguous() and u.numel() == self.batch * tree.n_nodes * self.V1
            return _Sampling(float(temperature), float(top_p), C.c_void_p(u.data_ptr()), 1), u
        u = np.ascontiguousarray(u, dtype=np.float32)
        assert u.size == self.batch * tree.n_nodes * self.V1, "uniforms must be [batch][n_nodes][V+1]"
        return _Sampling(float(temperature), float(top_p), u.ctypes.data_as(C.c_void_p), 0), u

    def verify(self, tree, tau, override=None, sample=None):
        """sample = None: deterministic tolerance; (temperature, top_p, uniforms): the stochastic rule."""
        buf = self._override(override)
        if sample is None:
            self._check(self.lib.vadusa_verify(self.h, C.byref(tree.c), int(tau), _ptr(buf)))
        else:
            sp, keep = self._sampling(tree, sample)
            self._check(self.lib.vadusa_verify_sampled(self.h, C.byref(tree.c), int(tau), C.byref(sp), _ptr(buf)))
        self.M = tree.n_nodes

    def kv_compact(self, seq=-1, path=None):
        if path is None:
            self._check(self.lib.vadusa_kv_compact(self.h, int(seq), None, 0))
        else:
            p = _i32(path)
            self._check(self.lib.vadusa_kv_compact(self.h, int(seq), _ptr(p), len(p)))

    def step(self, tree, tau, override=None, sync=True, sample=None):
        """One speculative step.  sync=True returns a list of accepted-token lists.
        sample = (temperature, top_p, uniforms) selects the stochastic rule."""
        buf = self._override(override)
        self.M = tree.n_nodes
        tok = np.zeros((self.batch, self.Hh + 1), np.int32) if sync else None
        ln = np.zeros(self.batch, np.int32) if sync else None
        if sample is None:
            self._check(self.lib.vadusa_step(self.h, C.byref(tree.c), int(tau), _ptr(buf), _ptr(tok), _ptr(ln)))
        else:
            sp, keep = self._sampling(tree, sample)
            self._check(self.lib.vadusa_step_sampled(self.h, C.byref(tree.c), int(tau), C.byref(sp), _ptr(buf),
                                                     _ptr(tok), _ptr(ln)))
        if not sync:
            return None
        return [tok[b, :ln[b]].tolist() for b in range(self.batch)]

    def read_output(self, seq=0):
        n = C.c_int32(0)
        self._check(self.lib.vadusa_read_output(self.h, seq, None, 0, C.byref(n)))
        out = np.zeros(max(n.value, 1), np.int32)
        self._check(self.lib.vadusa_read_output(self.h, seq, _ptr(out), n.value, C.byref(n)))
        return out[:n.value]

    # ---- inspection ----
    def debug(self, what):
        B, M, Hh, V1, d = self.batch, self.M, self.Hh, self.V1, self.cfg.d_model
        shapes = {
            DBG.LOGITS: ((B, M, V1), np.float32), DBG.SCORES: ((B, M, V1), np.float32), DBG.H_NODES: ((B, M, d), np.float32),
            DBG.TREE_TOK: ((B, M), np.int32), DBG.DRAFT_TOPK: ((B, Hh, MAX_TOPK), np.int32),
            DBG.KV_LEN: ((B,), np.int32), DBG.ROOT: ((B,), np.int32), DBG.EDGE_OK: ((B, M), np.int32),
            DBG.PATH: ((B, Hh + 2), np.int32), DBG.FINISHED: ((B,), np.int32),
            DBG.DRAFT_LOGITS: ((B, Hh, V1), np.float32), DBG.PHASE_CLOCK: ((128, 8), np.int64),
        }
        shape, dt = shapes[what]
        out = np.zeros(shape, dt)
        self._check(self.lib.vadusa_debug_read(self.h, what, _ptr(out), out.nbytes))
        return out

    def debug_raise_error(self):
        """Test aid: sets the error word of a kernel that gave up at a grid barrier."""
        self._check(self.lib.vadusa_debug_raise_error(self.h))

    def read_kv(self, layer, seq, which, pos0, npos, static=False):
        """static=True: through vadusa_debug_read_kv_static (staging in the library's static device array)."""
        out = np.zeros((npos, self.cfg.d_model), np.float32)
        f = self.lib.vadusa_debug_read_kv_static if static else self.lib.vadusa_debug_read_kv
        self._check(f(self.h, layer, seq, which, pos0, npos, _ptr(out)))
        return out
