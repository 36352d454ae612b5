"""Seeded synthetic inputs for the token-adaptive KV compression path (spectral gate, ragged
store, low-rank reconstruction).

Only random draws, an orthogonal factor from a library QR and storage rounding live here: none
of the method's arithmetic.  Shapes follow the paper's notation: a token's pre-RoPE key (or value)
state ``x`` has ``d_kv`` entries; ``U`` is the spectral basis, ``W`` and ``b`` the gate layer.

Recipe (stands in for the activations of an 8B model, which are not available offline):
  * ``Q``: orthogonal factor of a seeded Gaussian ``d x d`` matrix;
  * ``x = (z * sigma) Q^T`` with ``z ~ N(0,1)`` and ``sigma_j = (j+1)^-0.5``: in the basis ``Q``
    the energy is ordered and decays like a PCA spectrum;
  * ``U = Q + 0.02 N(0,1)/sqrt(d)``: a basis initialised at the PCA eigenvectors and then moved
    a little by training, so it is invertible but not orthogonal; ``U_inv`` is its fp64 inverse;
  * gate: ``W ~ N(0, w_std^2)`` and a bias bump ``b_j = h exp(-(j-c)^2 / (2 s^2))`` centred at
    ``c = 0.35 d`` with ``s = 0.12 d``: cut-off positions vary token by token around the bump.
All four parameter tensors and ``x`` are rounded to the storage type.
For the gate's backward pass: upstream gradients ``g_xhat ~ N(0, 1/n)`` (storage type; the scale of
a mean-reduced loss) and, optionally, ``g_m ~ N(0, 1/n)`` (float32).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

from .gen import BASE_SEED, bf16_bits_from_f32

STREAM_X = 20
STREAM_Q = 21
STREAM_U = 22
STREAM_GATE_W = 23
STREAM_G_XHAT = 24
STREAM_G_M = 25
ROWS_PER_BLOCK = 4096


@dataclass(frozen=True)
class KvWorkload:
    index: int          # seeds depend on it
    name: str
    n: int              # tokens (batch x sequence of one layer's key or value stream)
    d: int              # d_kv
    dtype: str          # "f32" | "bf16"
    tau: float = 0.1    # hard-mask threshold
    w_std: float = 1.5
    bump_height: float = 6.0

    def scaled(self, **kw) -> "KvWorkload":
        return replace(self, **kw)


KV_CONFIGS = [
    KvWorkload(100, "kv-tiny-f32", n=300, d=128, dtype="f32"),
    KvWorkload(101, "kv-small-bf16", n=1000, d=512, dtype="bf16"),
    # one layer's key stream of an 8-KV-head x 128 model: 16 sequences of 16K tokens
    KvWorkload(102, "kv-bf16-256k-x1024", n=262144, d=1024, dtype="bf16"),
]


def _rng(cfg: KvWorkload, stream: int, block: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([BASE_SEED, cfg.index, stream, block]))


def _store(cfg: KvWorkload, a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return bf16_bits_from_f32(a) if cfg.dtype == "bf16" else a


def basis_q(cfg: KvWorkload) -> np.ndarray:
    """Seeded orthogonal matrix, fp64 [d x d]."""
    g = _rng(cfg, STREAM_Q).standard_normal((cfg.d, cfg.d))
    q, r = np.linalg.qr(g)
    return q * np.sign(np.diag(r))


def spectrum(cfg: KvWorkload) -> np.ndarray:
    return (np.arange(cfg.d) + 1.0) ** -0.5


def states(cfg: KvWorkload, q: np.ndarray | None = None) -> np.ndarray:
    """Token states x, stored type [n x d]."""
    q = basis_q(cfg) if q is None else q
    qt = np.ascontiguousarray(q.T, dtype=np.float32)
    sig = spectrum(cfg).astype(np.float32)
    out = np.empty((cfg.n, cfg.d), dtype=np.uint16 if cfg.dtype == "bf16" else np.float32)
    for blk, r0 in enumerate(range(0, cfg.n, ROWS_PER_BLOCK)):
        r1 = min(cfg.n, r0 + ROWS_PER_BLOCK)
        z = _rng(cfg, STREAM_X, blk).standard_normal((r1 - r0, cfg.d), dtype=np.float32)
        out[r0:r1] = _store(cfg, (z * sig) @ qt)
    return out


def basis(cfg: KvWorkload, q: np.ndarray | None = None):
    """(U, U_inv) in the stored type, each [d x d]; U_inv is the fp64 inverse of the unrounded U."""
    q = basis_q(cfg) if q is None else q
    u = q + 0.02 * _rng(cfg, STREAM_U).standard_normal((cfg.d, cfg.d)) / np.sqrt(cfg.d)
    return _store(cfg, u), _store(cfg, np.linalg.inv(u))


def gate_params(cfg: KvWorkload):
    """(W stored type [d x d], b float32 [d])."""
    w = cfg.w_std * _rng(cfg, STREAM_GATE_W).standard_normal((cfg.d, cfg.d), dtype=np.float32)
    j = np.arange(cfg.d, dtype=np.float64)
    b = cfg.bump_height * np.exp(-((j - 0.35 * cfg.d) ** 2) / (2 * (0.12 * cfg.d) ** 2))
    return _store(cfg, w), b.astype(np.float32)


def kv_inputs(cfg: KvWorkload) -> dict:
    q = basis_q(cfg)
    u, u_inv = basis(cfg, q)
    w, b = gate_params(cfg)
    return dict(x=states(cfg, q), U=u, U_inv=u_inv, W=w, b=b)


def upstream(cfg: KvWorkload, rows: np.ndarray | None = None, with_g_m: bool = False):
    """(g_xhat stored type [n x d], g_m float32 [n x d] or None).  With `rows`, every other row is 0."""
    scale = np.float32(1.0 / np.sqrt(cfg.n))
    g = np.empty((cfg.n, cfg.d), dtype=np.float32)
    gm = np.empty((cfg.n, cfg.d), dtype=np.float32) if with_g_m else None
    for blk, r0 in enumerate(range(0, cfg.n, ROWS_PER_BLOCK)):
        r1 = min(cfg.n, r0 + ROWS_PER_BLOCK)
        g[r0:r1] = scale * _rng(cfg, STREAM_G_XHAT, blk).standard_normal((r1 - r0, cfg.d), dtype=np.float32)
        if with_g_m:
            gm[r0:r1] = scale * _rng(cfg, STREAM_G_M, blk).standard_normal((r1 - r0, cfg.d), dtype=np.float32)
    if rows is not None:
        keep = np.zeros(cfg.n, dtype=bool)
        keep[rows] = True
        g[~keep] = 0
        if with_g_m:
            gm[~keep] = 0
    return _store(cfg, g), gm
