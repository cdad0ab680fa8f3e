"""Seeded logit rows for the distillation-loss kernel: float32 arrays only, no arithmetic of
the loss itself.  Row kinds cover language-model-like rows (a normal bulk with a few tokens
standing out), ties, monotone rows and constant rows."""
from __future__ import annotations

import numpy as np


def _rng(seed, *tag):
    return np.random.Generator(np.random.SFC64(np.random.SeedSequence((seed, 0x10661) + tuple(tag))))


def lm_like_logits(seed: int, n_pos: int, vocab: int, scale: float = 2.5, tag: int = 0) -> np.ndarray:
    """Normal bulk (std `scale`) plus a handful of boosted tokens per row, as next-token logits
    of a language model look: a few candidates carry most of the mass."""
    rng = _rng(seed, n_pos, vocab, tag)
    x = rng.normal(0.0, scale, (n_pos, vocab)).astype(np.float32)
    for t in range(n_pos):
        n_top = int(rng.integers(1, 12))
        idx = rng.choice(vocab, size=min(n_top, vocab), replace=False)
        x[t, idx] += rng.uniform(2.0, 9.0, len(idx)).astype(np.float32)
    return x


def special_rows(seed: int, vocab: int) -> np.ndarray:
    """One row of each hard shape: heavy ties (rounded values), ascending, descending, constant,
    one dominant token, two-valued."""
    rng = _rng(seed, vocab, 1)
    rows = [np.round(rng.normal(0, 2, vocab)),
            np.linspace(-8, 8, vocab),
            np.linspace(8, -8, vocab),
            np.full(vocab, 1.25),
            np.concatenate([[40.0], rng.normal(0, 1, vocab - 1)]),
            (rng.random(vocab) < 0.01) * 6.0]
    return np.stack(rows).astype(np.float32)


def position_mask(seed: int, n_pos: int, keep: float = 0.7) -> np.ndarray:
    m = (_rng(seed, n_pos, 2).random(n_pos) < keep).astype(np.uint8)
    return m
