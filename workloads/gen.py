"""Seeded generators for the synthetic workloads.

Every array is drawn from ``numpy.random.Generator(PCG64)`` seeded with the
integer sequence ``[BASE_SEED, config index, stream, block]`` so that any block
of any tensor can be regenerated on its own.  Matrices are drawn in blocks of
``ROWS_PER_BLOCK`` rows.  bf16 tensors are returned as ``uint16`` bit patterns
(round-to-nearest-even of the fp32 draw); ``as_f64`` widens either storage type
exactly.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .configs import Workload

BASE_SEED = 20260304
ROWS_PER_BLOCK = 256

STREAM_H = 0
STREAM_W = 1
STREAM_W_OLD = 2
STREAM_W_REF = 3
STREAM_TOK = 4
STREAM_LEN = 5
STREAM_REWARD = 6
STREAM_LOGZ = 7
STREAM_SUBSET = 8
STREAM_PERTURB = 9


def _rng(cfg: Workload, stream: int, block: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([BASE_SEED, cfg.index, stream, block]))


# ---------------------------------------------------------------------------
# storage-type conversion (exact; no method arithmetic)
# ---------------------------------------------------------------------------

def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 with round-to-nearest-even; returns the uint16 bit patterns.

    Inputs are finite (the generators never produce NaN/Inf).
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def f32_from_bf16_bits(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of a stored tensor (uint16 bf16 bits or fp32) to fp64."""
    if a.dtype == np.uint16:
        return f32_from_bf16_bits(a).astype(np.float64)
    return a.astype(np.float64)


# ---------------------------------------------------------------------------
# per-response / per-prompt vectors
# ---------------------------------------------------------------------------

def lengths(cfg: Workload) -> np.ndarray:
    """Valid response lengths, int32[R]."""
    rng = _rng(cfg, STREAM_LEN)
    if cfg.len_dist == "uniform":
        ln = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.R)
    elif cfg.len_dist == "loguniform":
        u = rng.uniform(np.log(cfg.len_lo), np.log(cfg.len_hi), size=cfg.R)
        ln = np.clip(np.rint(np.exp(u)), cfg.len_lo, cfg.len_hi)
    else:
        raise ValueError(cfg.len_dist)
    return np.minimum(ln, cfg.T).astype(np.int32)


def rewards(cfg: Workload) -> np.ndarray:
    """One scalar reward per response, float32[R]."""
    rng = _rng(cfg, STREAM_REWARD)
    if cfg.reward_dist == "bernoulli":
        return (rng.random(cfg.R) < cfg.reward_p).astype(np.float32)
    if cfg.reward_dist == "uniform":
        return rng.random(cfg.R).astype(np.float32)
    raise ValueError(cfg.reward_dist)


def log_z(cfg: Workload) -> np.ndarray:
    """Per-prompt log-partition estimate, float32[P]."""
    if cfg.log_z == "zero":
        return np.zeros(cfg.P, dtype=np.float32)
    return _rng(cfg, STREAM_LOGZ).standard_normal(cfg.P).astype(np.float32)


def tokens(cfg: Workload) -> np.ndarray:
    """Sampled token ids, int32[N].

    "uniform": uniform over [0, V).  "zipf1.1": finite-support Zipf,
    P(id = k-1) proportional to k**-1.1 for k = 1..V, drawn by inverting the CDF
    (id = rank - 1, so the hot ids sit at the start of the vocabulary).
    """
    rng = _rng(cfg, STREAM_TOK)
    if cfg.tok_dist == "uniform":
        return rng.integers(0, cfg.V, size=cfg.N).astype(np.int32)
    if cfg.tok_dist == "zipf1.1":
        w = np.arange(1, cfg.V + 1, dtype=np.float64) ** -1.1
        cdf = np.cumsum(w)
        cdf /= cdf[-1]
        u = rng.random(cfg.N)
        return np.minimum(np.searchsorted(cdf, u, side="right"), cfg.V - 1).astype(np.int32)
    raise ValueError(cfg.tok_dist)


# ---------------------------------------------------------------------------
# matrices
# ---------------------------------------------------------------------------

def _std(stream: int) -> float:
    return 1.0 if stream == STREAM_H else 0.02


def _block(cfg: Workload, stream: int, block: int, rows: int, cols: int) -> np.ndarray:
    x = _rng(cfg, stream, block).standard_normal((rows, cols), dtype=np.float32)
    s = _std(stream)
    if s != 1.0:
        x *= np.float32(s)
    return bf16_bits_from_f32(x) if cfg.dtype == "bf16" else x


def _shape(cfg: Workload, stream: int):
    return (cfg.N, cfg.d) if stream == STREAM_H else (cfg.V, cfg.d)


def matrix(cfg: Workload, stream: int, threads: int | None = None) -> np.ndarray:
    """Full tensor of a stream: H (N x d, N(0,1)) or a weight matrix (V x d, N(0, 0.02^2)).

    Returns uint16 bf16 bits for bf16 configs, float32 otherwise.
    """
    rows, cols = _shape(cfg, stream)
    out = np.empty((rows, cols), dtype=np.uint16 if cfg.dtype == "bf16" else np.float32)
    nblk = (rows + ROWS_PER_BLOCK - 1) // ROWS_PER_BLOCK

    def fill(b: int) -> None:
        r0 = b * ROWS_PER_BLOCK
        r1 = min(rows, r0 + ROWS_PER_BLOCK)
        out[r0:r1] = _block(cfg, stream, b, r1 - r0, cols)

    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    if nblk <= 4 or threads <= 1:
        for b in range(nblk):
            fill(b)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(nblk)))
    return out


def matrix_rows(cfg: Workload, stream: int, row_ids) -> np.ndarray:
    """Selected rows of a stream's tensor, regenerated block by block (same values as ``matrix``)."""
    rows, cols = _shape(cfg, stream)
    row_ids = np.asarray(row_ids, dtype=np.int64)
    out = np.empty((row_ids.size, cols), dtype=np.uint16 if cfg.dtype == "bf16" else np.float32)
    blocks = row_ids // ROWS_PER_BLOCK
    for b in np.unique(blocks):
        r0 = int(b) * ROWS_PER_BLOCK
        r1 = min(rows, r0 + ROWS_PER_BLOCK)
        blk = _block(cfg, stream, int(b), r1 - r0, cols)
        sel = np.nonzero(blocks == b)[0]
        out[sel] = blk[row_ids[sel] - r0]
    return out


def hidden(cfg: Workload, threads: int | None = None) -> np.ndarray:
    return matrix(cfg, STREAM_H, threads)


def weight(cfg: Workload, which: str = "theta", threads: int | None = None) -> np.ndarray:
    stream = {"theta": STREAM_W, "old": STREAM_W_OLD, "ref": STREAM_W_REF}[which]
    return matrix(cfg, stream, threads)


def perturbed_weight(cfg: Workload, base: np.ndarray, rel: float = 0.05) -> np.ndarray:
    """``base + rel * N(0, 0.02^2)`` re-rounded to the storage type.

    Gives an old policy close to the current one, so that importance ratios
    stay near 1 and the unclipped branch of the surrogate is exercised.
    """
    rows, cols = base.shape
    noise = _rng(cfg, STREAM_PERTURB).standard_normal((rows, cols), dtype=np.float32)
    noise *= np.float32(0.02 * rel)
    if base.dtype == np.uint16:
        return bf16_bits_from_f32(f32_from_bf16_bits(base) + noise)
    return (base + noise).astype(np.float32)


# ---------------------------------------------------------------------------
# row subsets for full-size parity checks
# ---------------------------------------------------------------------------

def sample_valid_rows(cfg: Workload, lens: np.ndarray, tok: np.ndarray, count: int) -> np.ndarray:
    """A seeded, stratified subset of valid slot indices (sorted, unique).

    Strata: first and last valid token of sampled responses, slots whose target
    is the most frequent id, slots with rare ids (upper half of the vocabulary),
    and uniformly drawn valid slots for the remainder.
    """
    rng = _rng(cfg, STREAM_SUBSET)
    T = cfg.T
    resp = np.nonzero(lens > 0)[0]
    valid = np.concatenate([np.arange(r * T, r * T + int(lens[r])) for r in resp]) if resp.size else np.zeros(0, np.int64)
    if valid.size <= count:
        return valid.astype(np.int64)
    picks = []
    k = max(1, count // 8)
    rs = rng.choice(resp, size=min(k, resp.size), replace=False)
    picks.append(rs * T)                               # first valid token
    picks.append(rs * T + lens[rs].astype(np.int64) - 1)  # last valid token (next to padding)
    tv = tok[valid]
    hot = valid[tv == np.bincount(tv).argmax()]
    if hot.size:
        picks.append(rng.choice(hot, size=min(k, hot.size), replace=False))
    rare = valid[tv >= cfg.V // 2]
    if rare.size:
        picks.append(rng.choice(rare, size=min(k, rare.size), replace=False))
    got = np.unique(np.concatenate(picks))
    rest = np.setdiff1d(valid, got)
    need = count - got.size
    if need > 0:
        got = np.concatenate([got, rng.choice(rest, size=need, replace=False)])
    return np.sort(got)[:count].astype(np.int64)


# ---------------------------------------------------------------------------
# synthetic stand-ins for intermediate tensors (full-size checks of single stages)
# ---------------------------------------------------------------------------

STREAM_SYN_LOGP = 10
STREAM_SYN_GRAD = 11


def synthetic_logprobs(cfg: Workload):
    """Seeded stand-ins for (logp, logp_old, logp_ref), float32[N] each.

    Values have the scale of real token log-probs (about -ln V with a spread), the old policy
    is a small perturbation of the current one (so both clip branches occur) and the reference
    a larger one.  Used to check the O(N) loss kernels at full size without first running
    the vocabulary-sized forward in the oracle.
    """
    rng = _rng(cfg, STREAM_SYN_LOGP)
    base = -np.abs(rng.standard_normal(cfg.N)) * 2.0 - 0.5 * np.log(cfg.V)
    old = base + rng.standard_normal(cfg.N) * 0.15
    ref = base + rng.standard_normal(cfg.N) * 0.5
    return base.astype(np.float32), old.astype(np.float32), ref.astype(np.float32)


def synthetic_upstream_grad(cfg: Workload, lens: np.ndarray) -> np.ndarray:
    """Seeded stand-in for dL/dlogp, float32[N]: N(0,1)/(R*len_r) on valid slots, 0 on padding."""
    rng = _rng(cfg, STREAM_SYN_GRAD)
    g = rng.standard_normal((cfg.R, cfg.T)).astype(np.float32)
    t = np.arange(cfg.T)[None, :]
    ln = np.asarray(lens, dtype=np.int64)[:, None]
    w = np.where(t < ln, 1.0 / (cfg.R * np.maximum(ln, 1)), 0.0)
    return (g * w).astype(np.float32).reshape(cfg.N)
