"""Seeded synthetic sentence pairs, batches and direction samples.

Token ids follow a Zipf law (exponent 1.1) over the content ranks of a shared vocabulary
(id 0 = pad, 1 = BOS, 2 = EOS are never drawn as content).  Lengths are uniform (set-up 1) or
log-uniform with correlated source/target lengths (set-ups 2-5).  Pairs are sorted by length and
cut into batches whose padded target size stays within the token budget, standing in for the
paper's 4096-token batches of subword-tokenised parallel text (section 4, "Setup").
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

from .configs import Setup

PAD, BOS, EOS = 0, 1, 2


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed)))


def zipf_cdf(vocab: int, s: float = 1.1) -> np.ndarray:
    """Cumulative distribution over content ranks 1..vocab-3 with p(r) ~ r**-s."""
    r = np.arange(1, vocab - 2, dtype=np.float64)
    w = r ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


def draw_content_ids(rng: np.random.Generator, cdf: np.ndarray, n: int) -> np.ndarray:
    """n content ids in [3, vocab) by inverse-CDF sampling (rank r -> id r + 2)."""
    u = rng.random(n)
    rank0 = np.searchsorted(cdf, u, side="right")  # 0-based rank
    rank0 = np.minimum(rank0, len(cdf) - 1)
    return (rank0 + 3).astype(np.int32)


def draw_lengths(rng: np.random.Generator, setup: Setup, n: int) -> np.ndarray:
    """[n, 2] int32 = (source length, target length incl. BOS and EOS)."""
    lo, hi = setup.len_lo, setup.len_hi
    if setup.len_mode == "uniform":
        s = rng.integers(lo, hi + 1, size=n)
        t = rng.integers(lo, hi + 1, size=n)
    else:
        u = rng.random(n)
        ell = np.floor(lo * (hi / lo) ** u).astype(np.int64)
        ell = np.clip(ell, lo, hi)
        rho = rng.uniform(0.8, 1.25, size=n)
        s = ell
        t = np.clip(np.rint(ell * rho).astype(np.int64), lo, hi)
    return np.stack([s, t], axis=1).astype(np.int32)


@dataclass
class Batch:
    src_ids: np.ndarray  # [B, S_max] int32, content ids, pad 0 after s_b
    tgt_ids: np.ndarray  # [B, T_max] int32, BOS content... EOS, pad 0 after t_b
    lengths: np.ndarray  # [B, 2] int32 = (s_b, t_b)

    @property
    def n_src_tokens(self) -> int:
        return int(self.lengths[:, 0].sum())

    @property
    def n_tgt_tokens(self) -> int:
        """Real decoder positions U = sum(t_b - 1)."""
        return int((self.lengths[:, 1] - 1).sum())


def _fill_batch(rng: np.random.Generator, cdf: np.ndarray, lengths: np.ndarray) -> Batch:
    B = len(lengths)
    s_max = int(lengths[:, 0].max())
    t_max = int(lengths[:, 1].max())
    src = np.zeros((B, s_max), dtype=np.int32)
    tgt = np.zeros((B, t_max), dtype=np.int32)
    for b in range(B):
        s, t = int(lengths[b, 0]), int(lengths[b, 1])
        src[b, :s] = draw_content_ids(rng, cdf, s)
        tgt[b, 0] = BOS
        tgt[b, 1:t - 1] = draw_content_ids(rng, cdf, t - 2)
        tgt[b, t - 1] = EOS
    return Batch(src, tgt, lengths.astype(np.int32).copy())


def make_pool(setup: Setup) -> np.ndarray:
    """All sentence-pair lengths of the set-up's pool, [pool_pairs, 2]."""
    return draw_lengths(_rng(setup.data_seed), setup, setup.pool_pairs)


def make_batches(setup: Setup, n_batches: int | None = None) -> List[Batch]:
    """Length-bucketed batches (or fixed-size ones for set-up 1), order shuffled by seed."""
    rng = _rng(setup.data_seed)
    lengths = draw_lengths(rng, setup, setup.pool_pairs)
    groups: List[np.ndarray] = []
    if setup.fixed_batch:
        for i in range(0, len(lengths) - setup.fixed_batch + 1, setup.fixed_batch):
            groups.append(lengths[i:i + setup.fixed_batch])
    else:
        order = np.lexsort((lengths[:, 0], lengths[:, 1]))  # by target, then source length
        lengths = lengths[order]
        budget = setup.shape.batch_tokens
        start = 0
        while start < len(lengths):
            end = start + 1
            while end < len(lengths) and (end + 1 - start) * int(lengths[end, 1]) <= budget:
                end += 1
            groups.append(lengths[start:end])
            start = end
    perm = rng.permutation(len(groups))
    groups = [groups[i] for i in perm]
    if n_batches is not None:
        groups = groups[:n_batches]
    cdf = zipf_cdf(setup.shape.vocab)
    return [_fill_batch(rng, cdf, g) for g in groups]


def small_batch(vocab: int, lengths, seed: int) -> Batch:
    """A batch with explicitly given (s_b, t_b) pairs; for tests."""
    rng = _rng(seed)
    return _fill_batch(rng, zipf_cdf(vocab), np.asarray(lengths, dtype=np.int32).reshape(-1, 2))


def task_probabilities(n_tasks: int, temperature: float, skew: float = 1.0) -> np.ndarray:
    """Sampling weights for skewed data: task k (in the set-up's order) stands for a corpus of size
    proportional to (k+1)^-skew, and is drawn with probability proportional to size^(1/temperature):
    temperature 1 follows the corpus sizes, a large temperature tends to uniform."""
    size = (np.arange(n_tasks, dtype=np.float64) + 1.0) ** (-skew)
    w = size ** (1.0 / temperature)
    return w / w.sum()


def sample_directions(setup: Setup, n_steps: int, temperature: float = None, skew: float = 1.0) -> np.ndarray:
    """Task index per step: uniform over the set-up's tasks, or, with a temperature, drawn from
    task_probabilities (the single-GPU stand-in for temperature-based sampling over corpora of
    unequal size)."""
    rng = _rng(setup.direction_seed + 1)
    if temperature is None:
        return rng.integers(0, len(setup.tasks), size=n_steps).astype(np.int32)
    p = task_probabilities(len(setup.tasks), temperature, skew)
    return rng.choice(len(setup.tasks), size=n_steps, p=p).astype(np.int32)
