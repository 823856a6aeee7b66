"""Seeded CTC log-likelihood tensors shaped like an acoustic model's output."""
from __future__ import annotations

import numpy as np


def random_lengths(seed: int, batch: int, lo: int, hi: int) -> np.ndarray:
    """Utterance lengths in frames, uniform on {lo..hi}."""
    rng = np.random.default_rng([seed, 0x1E46])
    return rng.integers(lo, hi + 1, size=batch).astype(np.int32)


def ctc_loglikes(seed: int, lengths, T: int, V: int, sigma: float = 2.0,
                 p_blank: float = 0.65, blank_boost: float = 6.0,
                 token_boost: float = 4.0, out: np.ndarray | None = None) -> np.ndarray:
    """float32 [B, T, V] log-softmax rows.  Logits are N(0, sigma) (sigma = standard
    deviation); on a fraction p_blank of the frames the blank logit (class 0) gets
    +blank_boost, on the other frames one uniformly random non-blank class gets
    +token_boost.  Rows at t >= lengths[b] are zero and must never be read by a decoder.
    Utterance b depends on (seed, b) only, so any sub-batch reproduces."""
    lengths = np.asarray(lengths, dtype=np.int64)
    B = len(lengths)
    if out is None:
        out = np.zeros((B, T, V), dtype=np.float32)
    for b in range(B):
        n = int(lengths[b])
        rng = np.random.default_rng([seed, 0xAC0, b])
        x = rng.normal(0.0, sigma, size=(n, V))
        is_blank = rng.random(n) < p_blank
        tok = rng.integers(1, V, size=n)
        rows = np.arange(n)
        x[rows[is_blank], 0] += blank_boost
        if token_boost != 0.0:
            nb = rows[~is_blank]
            x[nb, tok[nb]] += token_boost
        x -= x.max(axis=1, keepdims=True)
        x -= np.log(np.exp(x).sum(axis=1, keepdims=True))
        out[b, :n, :] = x.astype(np.float32)
        out[b, n:, :] = 0.0
    return out
