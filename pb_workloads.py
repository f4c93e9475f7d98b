"""Seeded synthetic inputs for the phrase-boosting-tree hot path.

This module only *draws inputs*: tokenized phrase lists, hypothesis states and
acoustic log-probability tensors with the shapes, sizes and value distributions
of the five benchmark configurations.  It contains none of the method's
arithmetic (no tree, no boost scores, no fusion), so the CPU oracle and the HIP
path can both be fed from it without sharing any code of the method itself.

The inputs stand in for the paper's workloads (a 1024-token BPE vocabulary,
context lists of 200-991 phrases, the 20K-phrase robustness list, batch 32,
beam 8/3 -- Sec. III, Table I, Sec. IV-C); no item of those datasets is used.

Every array is a plain numpy array; the same arrays go to both sides.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Iterator, Optional, Tuple

import numpy as np

BASE_SEED = 20250807


@dataclass(frozen=True)
class Config:
    """One synthetic workload (index = position in the benchmark config list, 1-based)."""
    index: int
    name: str
    vocab_size: int
    blank_id: int            # -1 = blank-free
    n_phrases: int
    len_lo: int
    len_hi: int
    token_dist: str          # "uniform" | "zipf"
    zipf_s: float
    batch: int               # hypotheses per step (U*K for beam)
    beam: int                # 1 = greedy
    steps: int               # T
    sigma: float             # std of the raw logits
    alpha: float = 0.5
    weight: float = 1.0      # per-phrase boost (uniform arc score)

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


CONFIGS = {
    1: Config(1, "tiny_greedy", 128, 0, 10, 2, 6, "uniform", 0.0, 4, 1, 50, 2.0),
    2: Config(2, "greedy_1k", 1024, 0, 1000, 2, 10, "zipf", 1.1, 32, 1, 500, 2.0),
    3: Config(3, "greedy_20k", 1024, 0, 20000, 2, 12, "zipf", 1.1, 128, 1, 1000, 2.0),
    4: Config(4, "beam_5k", 1024, 0, 5000, 2, 10, "zipf", 1.1, 128, 4, 500, 2.0),
    5: Config(5, "largevocab_20k", 8192, -1, 20000, 2, 8, "zipf", 1.1, 256, 1, 200, 3.0),
}


def _token_probs(cfg: Config) -> np.ndarray:
    """Probability of token ids 1..V-1 (id 0 is never drawn: it is the blank where one exists)."""
    ids = np.arange(1, cfg.vocab_size, dtype=np.float64)
    if cfg.token_dist == "uniform":
        p = np.ones_like(ids)
    elif cfg.token_dist == "zipf":
        p = ids ** (-cfg.zipf_s)
    else:
        raise ValueError(cfg.token_dist)
    return p / p.sum()


def make_phrases(cfg: Config, seed: Optional[int] = None,
                 n_phrases: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Draw the tokenized context list.

    Returns (tokens int32[sum(len)], offsets int64[n+1]); phrase i is
    tokens[offsets[i]:offsets[i+1]].  Lengths are uniform on [len_lo, len_hi],
    token ids follow the config's distribution over 1..V-1.  Duplicates and
    phrases that are prefixes of others arise naturally and are kept.
    """
    rng = np.random.Generator(np.random.PCG64(cfg.seed if seed is None else seed))
    n = cfg.n_phrases if n_phrases is None else n_phrases
    lens = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=n, dtype=np.int64)
    offsets = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    p = _token_probs(cfg)
    toks = rng.choice(np.arange(1, cfg.vocab_size, dtype=np.int32), size=int(offsets[-1]), p=p)
    return toks.astype(np.int32), offsets


def log_softmax_rows(logits64: np.ndarray) -> np.ndarray:
    """Row-wise log-softmax in float64, rounded once to float32."""
    m = logits64.max(axis=-1, keepdims=True)
    z = logits64 - m
    lse = np.log(np.exp(z).sum(axis=-1, keepdims=True))
    return (z - lse).astype(np.float32)


@dataclass
class Planting:
    """Structured variant: push hypotheses along listed phrases.

    On about `cover` of the frames of every hypothesis, consecutive frames get
    `bump` added to the raw logit of the next token of a phrase drawn from the
    list; a fraction `truncate` of the plantings stops midway so that
    partial-match exits, end-of-phrase exits and deep failure chains all occur.
    """
    tokens: np.ndarray
    offsets: np.ndarray
    cover: float = 0.2
    truncate: float = 0.3
    bump: float = 8.0


def _plant_plan(cfg_steps: int, batch: int, pl: Planting, rng: np.random.Generator):
    """Returns arrays (t, b, v) of the logit entries to bump."""
    n = len(pl.offsets) - 1
    lens = np.diff(pl.offsets)
    mean_len = float(lens.mean()) * (1.0 - 0.5 * pl.truncate)
    p_start = pl.cover / max(1e-9, (1.0 - pl.cover) * mean_len)
    ts, bs, vs = [], [], []
    for b in range(batch):
        t = 0
        while t < cfg_steps:
            if rng.random() < p_start:
                i = int(rng.integers(0, n))
                L = int(lens[i])
                if L > 1 and rng.random() < pl.truncate:
                    L = int(rng.integers(1, L))
                for j in range(L):
                    if t + j >= cfg_steps:
                        break
                    ts.append(t + j)
                    bs.append(b)
                    vs.append(int(pl.tokens[pl.offsets[i] + j]))
                t += L
            else:
                t += 1
    return (np.asarray(ts, dtype=np.int64), np.asarray(bs, dtype=np.int64),
            np.asarray(vs, dtype=np.int64))


def logp_chunks(cfg: Config, seed: Optional[int] = None, steps: Optional[int] = None,
                batch: Optional[int] = None, planting: Optional[Planting] = None,
                blank_bias: float = 0.0, blank_frac: float = 0.0,
                chunk_frames: int = 32) -> Iterator[Tuple[int, np.ndarray]]:
    """Yield (t0, logp float32[n_frames, batch, V]) chunks of the acoustic log-probs.

    Raw logits are N(0, sigma) in float64, optionally bumped (planting, blank
    domination), then log-softmaxed per row in float64 and rounded to float32.
    The stream of random numbers does not depend on the chunk size.
    """
    T = cfg.steps if steps is None else steps
    B = cfg.batch if batch is None else batch
    V = cfg.vocab_size
    base = cfg.seed if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(base + 1000003))
    aux = np.random.Generator(np.random.PCG64(base + 2000003))
    plan = _plant_plan(T, B, planting, aux) if planting is not None else None
    blank_mask = None
    if blank_frac > 0.0 and cfg.blank_id >= 0:
        blank_mask = aux.random((T, B)) < blank_frac
    for t0 in range(0, T, chunk_frames):
        n = min(chunk_frames, T - t0)
        x = rng.standard_normal((n, B, V)) * cfg.sigma
        if plan is not None:
            ts, bs, vs = plan
            sel = (ts >= t0) & (ts < t0 + n)
            np.add.at(x, (ts[sel] - t0, bs[sel], vs[sel]), planting.bump)
        if blank_mask is not None:
            x[:, :, cfg.blank_id] += np.where(blank_mask[t0:t0 + n], blank_bias, 0.0)
        yield t0, log_softmax_rows(x)


def make_logp(cfg: Config, **kw) -> np.ndarray:
    """All frames at once: float32[T, batch, V]."""
    T = cfg.steps if kw.get("steps") is None else kw["steps"]
    B = cfg.batch if kw.get("batch") is None else kw["batch"]
    out = np.empty((T, B, cfg.vocab_size), dtype=np.float32)
    for t0, chunk in logp_chunks(cfg, **kw):
        out[t0:t0 + chunk.shape[0]] = chunk
    return out


def sticky_logp(seed: int, T: int, B: int, V: int, blank: int, sigma: float = 2.0, bump: float = 4.0,
                p_repeat: float = 0.35, p_blank: float = 0.25, p_bump: float = 0.85,
                grid: Optional[float] = 64.0) -> np.ndarray:
    """CTC-shaped acoustic rows float32[T, B, V]: the arg-max path has blanks and repeated labels.

    Every frame has a target label -- the previous frame's target again (p_repeat), the blank
    (p_blank, if there is one) or a fresh uniform token -- whose N(0, sigma) logit is raised by
    `bump` with probability p_bump.  With `grid` the values are rounded to multiples of 1/grid
    (sums with dyadic boosts stay exact in fp32); with grid=None the rows are log-softmaxed.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((T, B, V)) * sigma
    for b in range(B):
        target = -1
        for t in range(T):
            r = rng.random()
            if r < p_repeat and target >= 0:
                pass
            elif r < p_repeat + p_blank and blank >= 0:
                target = blank
            else:
                target = int(rng.integers(0, V))
            if rng.random() < p_bump:
                x[t, b, target] += bump
    if grid is None:
        return log_softmax_rows(x)
    return (np.round(x * grid) / grid).astype(np.float32)


def sample_states(num_states: int, count: int, seed: int) -> np.ndarray:
    """States drawn uniformly from all tree states (deep failure chains included)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, num_states, size=count, dtype=np.int64).astype(np.int32)


def tiny_case(seed: int, vocab_size: int = 6, max_phrases: int = 6, max_len: int = 5,
              blank_id: int = 0):
    """A tiny random phrase list over a tiny vocabulary, so that suffix overlaps are dense.

    Returns (tokens, offsets, weights float32[n]).  Token ids avoid `blank_id`
    when it is >= 0.  Weights are small dyadic rationals (exact in fp32).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    n = int(rng.integers(1, max_phrases + 1))
    lens = rng.integers(1, max_len + 1, size=n)
    offsets = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    allowed = np.array([v for v in range(vocab_size) if v != blank_id], dtype=np.int32)
    toks = rng.choice(allowed, size=int(offsets[-1]))
    weights = (rng.integers(1, 9, size=n) * 0.25).astype(np.float32)
    return toks.astype(np.int32), offsets, weights
