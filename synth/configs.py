"""Model shapes and workload presets.

The five presets mirror the five benchmark configurations of this build: a tiny
fp32 decoder, the 12-layer d=1024 decoder the paper describes (Sec. 3.1.1: 12
layers, 16 heads, 1024 hidden, 4096 feed-forward) at batch 1, a ragged batch
with the 2048-entry k-means vocabulary (Sec. 3.1.1), a long-form run with a
128-node tree (Sec. 3.1.3 ablation size), and a 64-sequence throughput batch.
"""
from dataclasses import dataclass, field, asdict
from typing import Tuple


@dataclass(frozen=True)
class ModelConfig:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    speech_vocab: int        # V; the EOS id is V, logits have V+1 entries
    text_vocab: int
    n_draft_heads: int
    max_positions: int       # rows of the position table == KV rows per sequence
    dtype: str               # "fp32" or "bf16"

    @property
    def n_logits(self) -> int:
        return self.speech_vocab + 1

    def as_dict(self):
        return asdict(self)


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelConfig
    batch: int
    text_len: Tuple[int, int]      # inclusive range; equal ends = fixed length
    prompt_len: Tuple[int, int]
    n_generate: int
    tree_nodes: int                # M, root included
    topk_caps: Tuple[int, ...]     # max rank+1 usable per draft head
    taus: Tuple[int, ...]
    seed: int = 20241021


def _vall_e(vocab, heads, max_pos):
    return ModelConfig(n_layers=12, d_model=1024, n_heads=16, head_dim=64, d_ffn=4096,
                       speech_vocab=vocab, text_vocab=512, n_draft_heads=heads,
                       max_positions=max_pos, dtype="bf16")


PRESETS = {
    # 1: tiny fp32 parity configuration
    "tiny": Workload(
        name="tiny",
        model=ModelConfig(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=1024,
                          speech_vocab=512, text_vocab=128, n_draft_heads=3,
                          max_positions=512, dtype="fp32"),
        batch=1, text_len=(32, 32), prompt_len=(75, 75), n_generate=150,
        tree_nodes=16, topk_caps=(4, 2, 2), taus=(1, 3)),
    # 2: the configuration the headline metric is quoted on
    "valle_b1": Workload(
        name="valle_b1", model=_vall_e(1024, 4, 1280),
        batch=1, text_len=(64, 64), prompt_len=(225, 225), n_generate=750,
        tree_nodes=64, topk_caps=(10, 10, 10, 10), taus=(1, 2, 4, 8)),
    # 3: ragged batch, 2048-entry vocabulary
    "hubert_b16": Workload(
        name="hubert_b16", model=_vall_e(2048, 4, 1024),
        batch=16, text_len=(20, 80), prompt_len=(100, 200), n_generate=500,
        tree_nodes=64, topk_caps=(10, 10, 10, 10), taus=(3,)),
    # 4: long-form, 5 heads, 128-node tree
    "longform_b1": Workload(
        name="longform_b1", model=_vall_e(1024, 5, 3328),
        batch=1, text_len=(64, 64), prompt_len=(750, 750), n_generate=2250,
        tree_nodes=128, topk_caps=(10, 10, 10, 10, 10), taus=(1, 4)),
    # 5: throughput batch
    "throughput_b64": Workload(
        name="throughput_b64", model=_vall_e(1024, 4, 1200),
        batch=64, text_len=(64, 64), prompt_len=(225, 225), n_generate=750,
        tree_nodes=32, topk_caps=(10, 10, 10, 10), taus=(1, 2, 4, 8)),
    # beyond the five configurations: configuration 2 with a 16k-entry speech vocabulary (the
    # vocabulary map and every draft head's second map grow to 32.8 MB, top-k over 16001 logits)
    "vocab16k_b1": Workload(
        name="vocab16k_b1", model=_vall_e(16000, 4, 1280),
        batch=1, text_len=(64, 64), prompt_len=(225, 225), n_generate=750,
        tree_nodes=64, topk_caps=(10, 10, 10, 10), taus=(1, 4)),
}


def preset(name: str) -> Workload:
    return PRESETS[name]
