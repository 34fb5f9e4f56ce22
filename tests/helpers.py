"""Shared test helpers (no method arithmetic beyond what a test needs to state)."""
import numpy as np

from oracle import vadusa_oracle as O
from synth import ModelConfig, make_weights

SMALL = ModelConfig(n_layers=2, d_model=64, n_heads=4, head_dim=16, d_ffn=128,
                    speech_vocab=40, text_vocab=16, n_draft_heads=3,
                    max_positions=96, dtype="fp32")


def small_model(seed=7, ln_jitter=0.1, std=0.2, cfg=SMALL):
    """A small model with lively logits (std 0.2) and non-trivial LayerNorm terms."""
    from oracle.vadusa_oracle import Model
    return Model(cfg, make_weights(cfg, seed=seed, std=std, ln_jitter=ln_jitter))


def planted_lists(future, tree, n_heads, vocab, rng, p_hit=0.7, p_first=0.0):
    """Per-head candidate lists with the true future token planted at a random rank (with probability
    p_first at rank 0: sparse trees reach their full depth along low ranks only).

    future[i] is the token that head i+1 should have predicted (may be missing
    near the end).  Lists hold distinct ids like a real top-k list.
    """
    need = O.topk_needed(tree.depth, tree.rank, n_heads)
    lists = []
    for i, k in enumerate(need):
        t = int(future[i]) if i < len(future) else -1
        pool = np.array([v for v in range(vocab) if v != t], dtype=np.int64)
        ids = rng.choice(pool, size=k, replace=False)
        if t >= 0 and k > 0 and rng.random() < p_hit:
            ids[0 if rng.random() < p_first else int(rng.integers(0, k))] = t
        lists.append(ids)
    return lists
