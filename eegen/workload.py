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


def draft_distributions(greedy: Sequence[int], vocab: int, seed: int, round_idx: int, session: int = 0,
                        n_other: int = 12, floor: float = 0.02):
    """Stand-in for a draft model's output in probabilistic verification: per position a
    distribution over the vocabulary (float32 rows that sum to 1), a draft token drawn from it,
    and the uniform numbers of the round.  A position's distribution puts a share alpha ~ U[0.3, 0.95]
    on the supplied continuation token, spreads `floor` evenly over the whole vocabulary and the rest
    over n_other random tokens with random shares -- so that drafts agree with a greedy target most
    of the time, as a trained draft model's do, without any model being run here.
    Returns (probs [gamma][vocab] float32, drafts [gamma] int32, u [gamma] float32, v [gamma+1] float32)."""
    g = np.asarray(greedy, dtype=np.int64)
    gamma = g.shape[0]
    r = _rng(seed, 5, session, round_idx)
    probs = np.full((gamma, vocab), floor / vocab, dtype=np.float64)
    for i in range(gamma):
        alpha = r.uniform(0.3, 0.95)
        probs[i, g[i]] += alpha
        others = r.integers(0, vocab, size=n_other)
        share = r.dirichlet(np.ones(n_other)) * (1.0 - floor - alpha)
        np.add.at(probs[i], others, share)
    probs32 = probs.astype(np.float32)
    pick = r.random(gamma)
    cdf = np.cumsum(probs32.astype(np.float64), axis=1)
    drafts = np.array([min(vocab - 1, int(np.searchsorted(cdf[i], pick[i] * cdf[i, -1], side="right"))) for i in range(gamma)],
                      dtype=np.int32)
    lim = np.float32(1.0) - np.float32(2.0 ** -24)
    u = np.minimum(r.random(gamma).astype(np.float32), lim)
    v = np.minimum(r.random(gamma + 1).astype(np.float32), lim)
    return probs32, drafts, u, v
