"""Workload shapes: the five benchmark configurations plus scaled-down test shapes.

Symbols follow the paper's Section 3.1: l_I initial tokens, l_L local tokens,
l_C current (chunk) tokens, k selected middle tokens, d_c = d' compressed size.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional


@dataclass(frozen=True)
class EsaConfig:
    name: str
    dtype: str            # "f32" or "bf16": storage type of Q, K, V, W, K', O
    H: int                # query heads
    H_kv: int             # key/value heads (GQA)
    d: int                # head dimension
    S: int                # tokens in the sequence (prefill) or in the cache incl. the new token (decode)
    l_I: int
    l_L: int
    l_C: int
    k: int
    d_c: int
    needles: int          # planted middle tokens per chunk
    needle_span: int = 1  # contiguous tokens per planted span
    rope_base: Optional[float] = None
    seed: int = 0
    batch: int = 1
    decode: bool = False  # one step with l_C = 1 on a cache of S-1 earlier tokens

    @property
    def d_Hq(self) -> int:
        return self.H * self.d

    @property
    def d_K(self) -> int:
        return self.H_kv * self.d

    def scaled(self, **kw) -> "EsaConfig":
        return replace(self, **kw)


CONFIGS = {
    # Tiny fp32 layer.
    "C1": EsaConfig("C1", "f32", H=4, H_kv=2, d=64, S=2048, l_I=32, l_L=256, l_C=128,
                    k=256, d_c=32, needles=16, seed=0),
    # Llama-3-8B-shaped attention layer, 32k chunked prefill.
    "C2": EsaConfig("C2", "bf16", H=32, H_kv=8, d=128, S=32768, l_I=128, l_L=2048, l_C=512,
                    k=2048, d_c=128, needles=64, rope_base=500000.0, seed=2),
    # Same layer, 128k chunked prefill.
    "C3": EsaConfig("C3", "bf16", H=32, H_kv=8, d=128, S=131072, l_I=128, l_L=2048, l_C=512,
                    k=2048, d_c=128, needles=64, rope_base=500000.0, seed=3),
    # Decode step on a 256k-token cache.
    "C4": EsaConfig("C4", "bf16", H=32, H_kv=8, d=128, S=262144, l_I=128, l_L=2048, l_C=1,
                    k=2048, d_c=128, needles=64, rope_base=500000.0, seed=4, decode=True),
    # 256k chunked prefill with clustered needles.
    "C5": EsaConfig("C5", "bf16", H=32, H_kv=8, d=128, S=262144, l_I=128, l_L=8192, l_C=1024,
                    k=8192, d_c=128, needles=8, needle_span=32, rope_base=500000.0, seed=5),
    # Mistral-7B-shaped attention layer (the paper's second model: same head layout, its local length 4096,
    # rotary base 1e6), 128k chunked prefill.
    "C6": EsaConfig("C6", "bf16", H=32, H_kv=8, d=128, S=131072, l_I=128, l_L=4096, l_C=512,
                    k=2048, d_c=128, needles=64, rope_base=1000000.0, seed=6),
}


def get_config(name: str) -> EsaConfig:
    return CONFIGS[name]


def segment_bounds(t0: int, l_I: int, l_L: int):
    """Split the t0 preceding tokens into I=[0,i_end), M=[i_end,l_start), L=[l_start,t0)."""
    i_end = min(l_I, t0)
    l_start = max(t0 - l_L, i_end)
    return i_end, l_start


def chunk_starts(cfg: EsaConfig):
    """First position of every step: all chunks of a prefill, or the single decode step."""
    if cfg.decode:
        return [cfg.S - 1]
    return list(range(0, cfg.S, cfg.l_C))
