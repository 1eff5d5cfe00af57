"""Seeded synthetic path sets that stand in for multi-sample reasoning traces.

This module only *draws inputs* (token ids, generation probabilities, ragged
append counts, verification targets).  It contains none of the drafting
method's arithmetic and is the one module that both the CPU oracle's tests and
the GPU path's tests/bench consume.

Why these inputs: parallel samples of one prompt share sub-steps that recur in
different order and with small lexical variation (paper, Introduction and the
"Fuzzy Suffix Matching" paragraph).  A shared pool of token segments models the
shared sub-steps, a per-path permutation models the re-ordering, and random
substitutions / insertions model the variation.  Token ids follow a Zipf law so
that low ids are frequent, which exercises the lowest-id tie-break.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

import numpy as np

BASE_SEED = 20250305

# purposes of the independent random streams of one problem
_POOL, _ORDER, _NOISE, _PROB, _RAGGED, _TARGET = range(6)


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration (shapes + noise recipe + draft arguments)."""
    name: str
    n_problems: int      # P
    n_paths: int         # N
    max_len: int         # tokens per path
    vocab: int           # V
    pool: int            # number of shared segments per problem
    seg_lo: int          # segment length, inclusive bounds
    seg_hi: int
    zipf_s: float
    r_sub: float         # per-token substitution probability
    r_ins: float = 0.0   # per-token probability of a random insertion burst
    ins_lo: int = 1
    ins_hi: int = 4
    with_replacement: bool = False   # True: draw segments i.i.d.; False: permutation per path
    query_len: int = 3   # k
    draft_len: int = 8   # L
    seed: int = BASE_SEED


WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", 1, 4, 256, 32000, 64, 8, 24, 1.1, 0.05,
                   with_replacement=True, query_len=3, draft_len=5),
    "C2": Workload("C2", 1, 16, 1024, 32000, 256, 8, 32, 1.1, 0.05,
                   query_len=3, draft_len=8),
    "C3": Workload("C3", 1, 32, 2048, 128256, 512, 8, 48, 1.05, 0.08,
                   r_ins=0.10, ins_lo=1, ins_hi=4, query_len=4, draft_len=10),
    "C4": Workload("C4", 64, 16, 1024, 32000, 256, 8, 32, 1.1, 0.05,
                   query_len=3, draft_len=8),
    "C5": Workload("C5", 1, 64, 4096, 152064, 2048, 4, 64, 1.0, 0.20,
                   query_len=4, draft_len=16),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields changed (smaller test shapes)."""
    return replace(w, **kw)


def _rng(seed: int, problem: int, purpose: int, path: int = 0) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, problem, purpose, path]))


def _zipf_cdf(vocab: int, s: float) -> np.ndarray:
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


def _zipf_draw(rng: np.random.Generator, cdf: np.ndarray, n: int) -> np.ndarray:
    ids = np.searchsorted(cdf, rng.random(n), side="right")
    return np.minimum(ids, len(cdf) - 1).astype(np.int32)


def make_paths(w: Workload):
    """Draw the full token paths of a workload.

    Returns (tokens int32 [P][N][max_len], probs float32 [P][N][max_len]).
    probs are stand-ins for the probability the model gave each token when it
    sampled it: U(0.5, 1) for pool tokens, U(0.01, 0.3) for noise tokens.
    """
    P, N, T = w.n_problems, w.n_paths, w.max_len
    tokens = np.empty((P, N, T), dtype=np.int32)
    probs = np.empty((P, N, T), dtype=np.float32)
    cdf = _zipf_cdf(w.vocab, w.zipf_s)
    for p in range(P):
        pr = _rng(w.seed, p, _POOL)
        seg_len = pr.integers(w.seg_lo, w.seg_hi + 1, size=w.pool)
        seg_tok = _zipf_draw(pr, cdf, int(seg_len.sum()))
        seg_off = np.concatenate([[0], np.cumsum(seg_len)])
        segs = [seg_tok[seg_off[s]:seg_off[s + 1]] for s in range(w.pool)]
        for i in range(N):
            orr = _rng(w.seed, p, _ORDER, i)
            parts, have = [], 0
            while have < T:
                if w.with_replacement:
                    order = orr.integers(0, w.pool, size=w.pool)
                else:
                    order = orr.permutation(w.pool)
                for s in order:
                    parts.append(segs[s])
                    have += len(segs[s])
                    if have >= T:
                        break
            src = np.concatenate(parts)[:T].copy()
            nr = _rng(w.seed, p, _NOISE, i)
            noise = nr.random(T) < w.r_sub
            src[noise] = nr.integers(0, w.vocab, size=int(noise.sum()), dtype=np.int32)
            if w.r_ins > 0.0:
                burst = np.where(nr.random(T) < w.r_ins,
                                 nr.integers(w.ins_lo, w.ins_hi + 1, size=T), 0)
                end = np.cumsum(burst + 1)          # index after each source token
                out = nr.integers(0, w.vocab, size=int(end[-1]), dtype=np.int32)
                out_noise = np.ones(int(end[-1]), dtype=bool)
                out[end - 1] = src
                out_noise[end - 1] = noise
                src, noise = out[:T], out_noise[:T]
            tokens[p, i] = src
            qr = _rng(w.seed, p, _PROB, i)
            hi = qr.uniform(0.5, 1.0, size=T)
            lo = qr.uniform(0.01, 0.3, size=T)
            probs[p, i] = np.where(noise, lo, hi).astype(np.float32)
    return tokens, probs


def make_targets(tokens: np.ndarray, t: int, draft_len: int) -> np.ndarray:
    """Verification targets after `t` tokens per path were appended: each
    path's own next `draft_len` tokens (what the model goes on to sample),
    padded with -1 past the end.  int32 [P][N][draft_len]."""
    P, N, T = tokens.shape
    out = np.full((P, N, draft_len), -1, dtype=np.int32)
    m = max(0, min(draft_len, T - t))
    out[:, :, :m] = tokens[:, :, t:t + m]
    return out


def make_noisy_targets(w: Workload, tokens: np.ndarray, t: int, draft_len: int,
                       r_flip: float = 0.15) -> np.ndarray:
    """Targets as in make_targets but with a fraction of positions replaced by
    a uniform random id, so that accept lengths cover the whole 0..L range."""
    tg = make_targets(tokens, t, draft_len)
    r = _rng(w.seed, t, _TARGET)
    flip = r.random(tg.shape) < r_flip
    tg[flip] = r.integers(0, w.vocab, size=int(flip.sum()), dtype=np.int32)
    return tg


def make_ragged_counts(w: Workload, n_max: int, steps: int) -> np.ndarray:
    """Per-step, per-path append counts in [0, n_max]: int32 [steps][P][N]."""
    r = _rng(w.seed, 0, _RAGGED)
    return r.integers(0, n_max + 1, size=(steps, w.n_problems, w.n_paths)).astype(np.int32)
