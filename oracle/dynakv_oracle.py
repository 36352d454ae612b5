"""CPU oracle for the token-adaptive KV compression path (TEST INFRASTRUCTURE ONLY).

Plain fp64 NumPy statement of Sec. 3 of the paper ("Dynamic Compressing"), one function per
equation, in the paper's notation: a token's pre-RoPE key or value state is the row vector
``x`` (d = d_kv entries), ``U`` the spectral basis, ``W, b`` the gate layer, ``tau`` the
threshold.  Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this file; it shares no code with the HIP path.

Readings taken where the paper leaves a choice (each is listed in the design notes too):

* Eq. 6 writes ``m = Flip(cumsum(p))``, i.e. ``m_i = sum_{j <= d-1-i} p_j``, while the sentence
  after it describes a mask that is about 1 before the predicted cut-off index k and 0 after
  it, which is the reverse cumulative sum ``m_i = sum_{j >= i} p_j``.  The two differ only by
  relabelling the gate's output columns ``j <-> d-1-j``.  ``order="suffix"`` (default) is the
  reverse cumulative sum, ``order="literal"`` the formula as printed.
* The spectral state is kept in the model's storage type: ``x~`` is rounded to that type
  (``store_dtype``) before it enters the gate layer and the cache.  ``None`` keeps fp64.
* Eq. 8 compares in the kernel's precision: ``float32(m_i) > float32(tau)``.
* The ragged store keeps ``x~[0:k]`` per token at an offset that is a multiple of ``granule``
  elements (the paper does not say how segments are packed); the tail of the last granule is 0.
* Eq. 3 takes ``U^-1`` as an input (for an orthogonal ``U`` it is ``U^T``); nothing is inverted.
* The overall retain rate of Eq. 4 and Eq. 9 is the plain mean over the tokens passed in.
"""
from __future__ import annotations

import numpy as np


def round_to(x, store_dtype):
    """Round fp64 values to a storage type and return them as fp64: "bf16" (round to nearest
    even on the upper 16 bits of the fp32 pattern, after rounding to fp32), "f32", or None."""
    x = np.asarray(x, dtype=np.float64)
    if store_dtype is None:
        return x
    f = x.astype(np.float32)
    if store_dtype == "f32":
        return f.astype(np.float64)
    if store_dtype != "bf16":
        raise ValueError(store_dtype)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(x.shape)


def spectral(x, U):
    """Eq. 1: ``x~ = x U`` (rows are tokens)."""
    return np.asarray(x, dtype=np.float64) @ np.asarray(U, dtype=np.float64)


def gate_probs(xt, W, b):
    """Eq. 5: ``p = Softmax(x~ W + b)`` over the d cut-off positions of each token."""
    z = np.asarray(xt, dtype=np.float64) @ np.asarray(W, dtype=np.float64) + np.asarray(b, dtype=np.float64)
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def soft_mask(p, order: str = "suffix"):
    """Eq. 6: the soft truncation mask, non-increasing from m_0 = 1."""
    p = np.asarray(p, dtype=np.float64)
    d = p.shape[1]
    m = np.empty_like(p)
    if order == "suffix":
        for i in range(d):
            m[:, i] = p[:, i:].sum(axis=1)
    elif order == "literal":
        for i in range(d):
            m[:, i] = p[:, : d - i].sum(axis=1)
    else:
        raise ValueError(order)
    return m


def hard_mask(m, tau: float):
    """Eq. 8: ``m_hard_i = 1[m_i > tau]``, decided in fp32."""
    return (np.asarray(m).astype(np.float32) > np.float32(tau)).astype(np.uint8)


def retained(m, tau: float):
    """k = number of retained leading components per token (the hard mask is a prefix)."""
    return hard_mask(m, tau).sum(axis=1).astype(np.int32)


def gate(x, U, W, b, tau: float, order: str = "suffix", store_dtype=None):
    """Eqs. 1, 5, 6, 7, 8 for a batch of tokens.

    Returns dict(xt, p, m, xhat, k): the stored spectral state, cut-off distribution, soft mask,
    softly gated state ``x~ * m`` (Eq. 7, rounded to the storage type) and retained counts.
    """
    xt = round_to(spectral(x, U), store_dtype)
    p = gate_probs(xt, W, b)
    m = soft_mask(p, order)
    return dict(xt=xt, p=p, m=m, xhat=round_to(xt * m, store_dtype), k=retained(m, tau))


def store(xt, k, granule: int = 8):
    """The persisted part of Eq. 2: per token the leading k components, packed.

    Returns (off int64[n+1], packed fp64[off[n]]): token i occupies ``packed[off[i] : off[i] +
    k[i]]``; ``off[i+1] - off[i]`` is k[i] rounded up to the granule and the padding is 0.
    """
    xt = np.asarray(xt, dtype=np.float64)
    n = xt.shape[0]
    off = np.zeros(n + 1, dtype=np.int64)
    for i in range(n):
        off[i + 1] = off[i] + (int(k[i]) + granule - 1) // granule * granule
    packed = np.zeros(int(off[n]), dtype=np.float64)
    for i in range(n):
        packed[off[i]: off[i] + int(k[i])] = xt[i, : int(k[i])]
    return off, packed


def reconstruct(packed, off, k, U_inv, store_dtype=None):
    """Eq. 3: ``x_bar = x^[I] U^-1[I, :]`` with I = {0..k-1}: a rank-k product per token."""
    U_inv = np.asarray(U_inv, dtype=np.float64)
    n, d = len(k), U_inv.shape[1]
    out = np.zeros((n, d), dtype=np.float64)
    for i in range(n):
        ki = int(k[i])
        out[i] = np.asarray(packed[off[i]: off[i] + ki], dtype=np.float64) @ U_inv[:ki, :]
    return round_to(out, store_dtype)


def retain_rate_hard(k, d: int) -> float:
    """Eq. 4 averaged over the tokens: mean_i k_i / d."""
    return float(np.mean(np.asarray(k, dtype=np.float64)) / d) if len(k) else 0.0


def retain_rate_soft(m) -> float:
    """The differentiable retain rate used in Eq. 9: the mean of the soft mask."""
    m = np.asarray(m, dtype=np.float64)
    return float(m.mean()) if m.size else 0.0


def retain_penalty(m, alpha: float):
    """The regulariser of Eq. 9, ``alpha * R^2`` with the soft R, and its gradient w.r.t. m:
    ``d/dm_{i,j} = 2 alpha R / (n d)``.  Returns (penalty, R, grad)."""
    m = np.asarray(m, dtype=np.float64)
    R = retain_rate_soft(m)
    return alpha * R * R, R, np.full_like(m, 2.0 * alpha * R / max(m.size, 1))


def gate_bwd(x, U, W, b, g_xhat, g_m=None, order: str = "suffix", store_dtype=None):
    """Gradients of a scalar L through the training-time gate (Eqs. 1, 5, 6, 7), given
    ``g_xhat = dL/dx^`` and optionally a direct ``g_m = dL/dm`` (e.g. the retain-rate regulariser's).

    With ``x~ = xU``, ``l = x~W + b``, ``p = softmax(l)``, ``m`` the cumulative mask and ``x^ = x~ * m``:
        q   = dL/dm   = g_xhat * x~ + g_m
        r   = dL/dp:   r_j = sum_{i <= j} q_i            (suffix mask: p_j feeds m_0 .. m_j)
                       r_j = sum_{i <= d-1-j} q_i        (mask as printed in Eq. 6)
        g_l = dL/dl   = p * (r - sum_k p_k r_k)           (softmax Jacobian)
        g_xt = dL/dx~ = g_xhat * m + g_l W^T
        dW = x~^T g_l,  db = sum_tokens g_l,  dU = x^T g_xt,  dx = g_xt U^T.
    With ``store_dtype`` the forward quantities (x~, p, m) are those of ``gate``: x~ rounded to the
    storage type, and that rounding is treated as the identity in the chain rule (straight-through);
    nothing else is rounded.  The paper gives the forward pass only and calls the gate differentiable;
    this is the plain chain rule through it, pinned in the tests by central differences of the forward
    functions above (themselves pinned to the equations) and by identities.
    Returns dict(dx, dU, dW, db, g_l, g_xt).
    """
    x = np.asarray(x, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    g_xhat = np.asarray(g_xhat, dtype=np.float64)
    xt = round_to(spectral(x, U), store_dtype)
    p = gate_probs(xt, W, b)
    m = soft_mask(p, order)
    q = g_xhat * xt
    if g_m is not None:
        q = q + np.asarray(g_m, dtype=np.float64)
    d = x.shape[1]
    pre = np.zeros_like(q)
    for j in range(d):
        pre[:, j] = q[:, : j + 1].sum(axis=1)
    r = pre if order == "suffix" else pre[:, ::-1]
    g_l = p * (r - (p * r).sum(axis=1, keepdims=True))
    g_xt = g_xhat * m + g_l @ W.T
    return dict(dx=g_xt @ U.T, dU=x.T @ g_xt, dW=xt.T @ g_l, db=g_l.sum(axis=0), g_l=g_l, g_xt=g_xt)
