"""Seeded random-init weights.

Every tensor is drawn from its own stream (master seed, tensor index) so that a
tensor's values do not depend on which other tensors were drawn before it.
All linear maps are stored [out_features, in_features] (y = W x + b).

Recipe: weights and biases N(0, 0.02) in fp32, LayerNorm gain 1 and shift 0
(optionally jittered so tests exercise those terms).  For bf16 models every
value is rounded to the nearest bf16 (ties to even) and returned as fp32, so
both consumers start from bit-identical numbers.
"""
import numpy as np

from .configs import ModelConfig


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def weight_names(cfg: ModelConfig):
    """Ordered (name, shape, kind) list; the order is also the flat-blob order."""
    d, F, V1 = cfg.d_model, cfg.d_ffn, cfg.n_logits
    out = [("E_text", (cfg.text_vocab, d), "w"),
           ("E_speech", (V1, d), "w"),
           ("P", (cfg.max_positions, d), "w")]
    for l in range(cfg.n_layers):
        p = f"L{l}."
        out += [(p + "ln1_g", (d,), "g"), (p + "ln1_b", (d,), "s"),
                (p + "Wqkv", (3 * d, d), "w"), (p + "bqkv", (3 * d,), "w"),
                (p + "Wo", (d, d), "w"), (p + "bo", (d,), "w"),
                (p + "ln2_g", (d,), "g"), (p + "ln2_b", (d,), "s"),
                (p + "W1", (F, d), "w"), (p + "b1", (F,), "w"),
                (p + "W2", (d, F), "w"), (p + "b2", (d,), "w")]
    out += [("lnf_g", (d,), "g"), ("lnf_b", (d,), "s"), ("W_out", (V1, d), "w")]
    for i in range(cfg.n_draft_heads):
        p = f"D{i}."
        out += [(p + "W1", (d, d), "w"), (p + "b1", (d,), "w"), (p + "W2", (V1, d), "w")]
    return out


def make_weights(cfg: ModelConfig, seed: int = 20241021, std: float = 0.02,
                 ln_jitter: float = 0.0):
    """Return {name: fp32 array}.  ln_jitter>0 draws gain 1+N(0,j) and shift N(0,j)."""
    W = {}
    for idx, (name, shape, kind) in enumerate(weight_names(cfg)):
        rng = np.random.default_rng(np.random.SeedSequence([seed, idx]))
        if kind == "w":
            a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        elif kind == "g":
            a = np.ones(shape, np.float32)
            if ln_jitter:
                a += rng.standard_normal(shape, dtype=np.float32) * np.float32(ln_jitter)
        else:
            a = np.zeros(shape, np.float32)
            if ln_jitter:
                a += rng.standard_normal(shape, dtype=np.float32) * np.float32(ln_jitter)
        if cfg.dtype == "bf16":
            a = round_to_bf16(a)
        W[name] = a
    return W
