"""Seeded text / prompt token streams (ragged per sequence)."""
import numpy as np

from .configs import Workload


def make_tokens(wl: Workload, seed=None, batch=None):
    """Return (text, prompt): two lists of int32 arrays, one per sequence.

    Text tokens are uniform over the text vocabulary, prompt speech tokens
    uniform over [0, V) (never EOS); lengths uniform over the workload's
    inclusive ranges.
    """
    seed = wl.seed if seed is None else seed
    B = wl.batch if batch is None else batch
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x70C]))
    text, prompt = [], []
    for _ in range(B):
        tl = int(rng.integers(wl.text_len[0], wl.text_len[1] + 1))
        pl = int(rng.integers(wl.prompt_len[0], wl.prompt_len[1] + 1))
        text.append(rng.integers(0, wl.model.text_vocab, tl).astype(np.int32))
        prompt.append(rng.integers(0, wl.model.speech_vocab, pl).astype(np.int32))
    return text, prompt


def make_uniforms(seed: int, step: int, batch: int, n_nodes: int, n_logits: int) -> np.ndarray:
    """Uniform random numbers for one stochastic verification step, fp32 [batch, n_nodes, n_logits].

    One independent stream per (seed, step); every value lies strictly inside (0, 1).
    """
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x5A3, step]))
    u = rng.random((batch, n_nodes, n_logits), dtype=np.float32)
    tiny = np.float32(2.0 ** -24)
    return np.clip(u, tiny, np.float32(1.0) - tiny).astype(np.float32)
