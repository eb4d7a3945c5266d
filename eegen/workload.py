"""Seeded synthetic workloads: prompts, corrupted drafts, embedding prefixes.

Stand-ins for the paper's text prompts and camera frames: only their shapes and
structure are kept (prompt length, draft count, image-patch prefix then text).
Nothing here computes any part of the decoding method; the greedy continuation
that drafts are derived from is supplied by the caller.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np

from .format import ModelConfig, f32_to_bf16

# shapes of the benchmark configurations
TINY = ModelConfig(n_layers=4, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024,
                   exit_layers=(2,))
LLAMA7B = ModelConfig(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008,
                      vocab=32000, exit_layers=(8, 16, 24))
LLAMA13B = ModelConfig(n_layers=40, d_model=5120, n_heads=40, head_dim=128, d_ffn=13824,
                       vocab=32000, exit_layers=(20,))


def _rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1),
                                                     hash_stream(stream)]))


def hash_stream(stream: Sequence[int]) -> int:
    h = 0xCBF29CE484222325
    for s in stream:
        for b in int(s).to_bytes(8, "little", signed=False):
            h = ((h ^ b) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h


def prompt_tokens(seed: int, n: int, vocab: int, session: int = 0) -> np.ndarray:
    """n token ids uniform in [0, vocab)."""
    return _rng(seed, 1, session).integers(0, vocab, size=n, dtype=np.int32)


def corrupt_drafts(greedy: Sequence[int], p: float, vocab: int, seed: int, round_idx: int,
                   session: int = 0) -> np.ndarray:
    """Each position of the greedy continuation is independently replaced, with
    probability p, by a uniform-random id (which may equal the original)."""
    g = np.asarray(greedy, dtype=np.int32)
    r = _rng(seed, 2, session, round_idx)
    mask = r.random(g.shape[0]) < p
    rnd = r.integers(0, vocab, size=g.shape[0], dtype=np.int32)
    return np.where(mask, rnd, g).astype(np.int32)


def session_corruption_p(seed: int, session: int, lo: float = 0.1, hi: float = 0.6) -> float:
    return float(_rng(seed, 3, session).uniform(lo, hi))


def embedding_prefix(seed: int, n_rows: int, d_model: int, session: int = 0) -> np.ndarray:
    """n_rows vectors ~ N(0,1) rounded to bf16 (raw uint16), image-patch stand-ins."""
    x = _rng(seed, 4, session).standard_normal((n_rows, d_model), dtype=np.float32)
    return f32_to_bf16(x).reshape(n_rows, d_model)
