"""CPU oracle for the fused LM-head log-probability objective (TEST INFRASTRUCTURE ONLY).

This file is the slow, plain definition of what the GPU library computes.  It is
test infrastructure: only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import it.  It shares no code with the HIP path and is
written in fp64 NumPy, one formula per step, with no blocking, fusion or
re-ordering, so it can be checked against the mathematics by eye.

What the paper fixes and what it does not
-----------------------------------------
The paper's training objective (Sec. 3.3 "Training Objective", Eq. 9) is
``L = L_CE + alpha * R^2`` where ``L_CE`` is the standard cross-entropy over
target tokens.  ``L_CE`` is the negative mean of the token log-probabilities
``log pi(y_i) = z[i, y_i] - logsumexp_v z[i, v]`` with logits ``z = H W^T``.
That log-softmax/LM-head part (``logits``, ``lmhead_logprob_fwd``, ``ce_loss``
and the softmax Jacobian inside ``lmhead_logprob_bwd``) is the part pinned by
the paper.  The policy-optimisation pieces (group advantages, the clipped
importance-ratio surrogate with the k3 KL term, the trajectory-balance
residual) are stated only by the benchmark's problem statement, not by the
paper: for the paper they are PARITY UNPINNED, and they are pinned here only by
the closed forms, invariants, brute-force and finite-difference checks in
``tests/test_oracle_*.py``.

Layout conventions: P prompts, G responses per prompt, T slots per response,
R = P*G, N = R*T; slot ``i = r*T + t`` is valid iff ``t < len[r]`` (right
padding).  H is N x d, W is V x d (row v = output embedding of token v).
All outputs on padded slots are 0.
"""
from __future__ import annotations

import numpy as np


# ---------------------------------------------------------------------------
# indexing (integer work; compared bit-exactly)
# ---------------------------------------------------------------------------

def index_build(lens, T: int):
    """Right-padding mask and group indexing.

    Returns (mask u8[N], cu_len i32[R+1], row_slot i32[N_v], resp_of_row i32[N_v]):
    ``mask[r*T+t] = (t < len[r])``; ``cu_len`` is the exclusive prefix sum of the
    lengths; ``row_slot[k]`` is the slot of the k-th valid token in slot order and
    ``resp_of_row[k]`` the response it belongs to.
    """
    lens = np.asarray(lens, dtype=np.int64)
    R = lens.size
    if np.any(lens < 0) or np.any(lens > T):
        raise ValueError("length outside [0, T]")
    t = np.arange(T, dtype=np.int64)
    mask2 = t[None, :] < lens[:, None]
    mask = mask2.reshape(R * T).astype(np.uint8)
    cu_len = np.zeros(R + 1, dtype=np.int64)
    for r in range(R):
        cu_len[r + 1] = cu_len[r] + lens[r]
    row_slot = np.nonzero(mask)[0].astype(np.int32)
    resp_of_row = (row_slot // T).astype(np.int32)
    return mask, cu_len.astype(np.int32), row_slot, resp_of_row


# ---------------------------------------------------------------------------
# LM head: logits, log-sum-exp, target log-prob, entropy  (Eq. 9, L_CE term)
# ---------------------------------------------------------------------------

def logits(H, W):
    """z = H W^T in fp64 (H: n x d, W: V x d)."""
    return np.asarray(H, dtype=np.float64) @ np.asarray(W, dtype=np.float64).T


def quantize_e4m3(x, exp2: int):
    """The value that the 8-bit variant of the logits path sees for x: ``x * 2^exp2`` clamped to
    [-448, 448] and rounded to the nearest OCP e4m3 number (4 exponent bits, bias 7, 3 mantissa bits,
    subnormals down to 2^-9, ties to even), then scaled back by ``2^-exp2``.  Returns fp64.

    (This variant is the benchmark's, not the paper's: parity unpinned for the paper.  The rounding
    itself is pinned against an independent implementation in the tests.)
    """
    y = np.clip(np.asarray(x, dtype=np.float64) * 2.0 ** exp2, -448.0, 448.0)
    a = np.abs(y)
    # spacing of the e4m3 grid around |y|: 2^(floor(log2|y|) - 3), and 2^-9 in the subnormal range
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -6)))
    step = 2.0 ** (e - 3)
    q = np.rint(a / step) * step          # numpy rounds halves to even, as the format requires
    return np.sign(y) * q * 2.0 ** -exp2


def logprob_rows(H_rows, W, tok_rows):
    """Log-softmax statistics of given rows, all treated as valid.

    For each row: ``M = max_v z_v``, ``S = sum_v exp(z_v - M)``, ``lse = M + log S``,
    ``logp = z[y] - lse`` (log of the softmax probability of the target token,
    i.e. minus its cross-entropy term, Eq. 9) and the entropy of the softmax
    ``ent = lse - (sum_v exp(z_v - M) z_v) / S``.
    Returns (logp, lse, ent) as fp64[n].
    """
    z = logits(H_rows, W)
    tok_rows = np.asarray(tok_rows, dtype=np.int64)
    n, V = z.shape
    if np.any(tok_rows < 0) or np.any(tok_rows >= V):
        raise ValueError("token id outside [0, V)")
    M = z.max(axis=1)
    e = np.exp(z - M[:, None])
    S = e.sum(axis=1)
    lse = M + np.log(S)
    logp = z[np.arange(n), tok_rows] - lse
    ent = lse - (e * z).sum(axis=1) / S
    return logp, lse, ent


def lmhead_logprob_fwd(H, W, tok, lens, T: int, block: int = 256):
    """logp, lse, entropy for every slot (fp64[N]); padded slots give 0.

    Rows are processed ``block`` at a time only to bound memory; every row is
    computed independently by ``logprob_rows``.
    """
    mask, _, row_slot, _ = index_build(lens, T)
    N = mask.size
    logp = np.zeros(N)
    lse = np.zeros(N)
    ent = np.zeros(N)
    H = np.asarray(H)
    tok = np.asarray(tok)
    for b0 in range(0, row_slot.size, block):
        rows = row_slot[b0:b0 + block]
        lp, ls, en = logprob_rows(H[rows], W, tok[rows])
        logp[rows], lse[rows], ent[rows] = lp, ls, en
    return logp, lse, ent


def lse_merge(parts):
    """Combine partial softmax statistics of disjoint column ranges of one row.

    ``parts`` is a sequence of (m, s, t) with ``m`` the range's maximum,
    ``s = sum exp(z - m)`` and ``t = sum exp(z - m) z`` over the range.  The
    merged statistics are those of the union: with ``m* = max m_j``,
    ``s* = sum_j s_j exp(m_j - m*)`` and ``t* = sum_j t_j exp(m_j - m*)``.
    An empty range is (-inf, 0, 0).  This is the re-association that makes a
    vocabulary-chunked evaluation exact.
    """
    ms = np.array([p[0] for p in parts], dtype=np.float64)
    m = ms.max()
    if not np.isfinite(m):
        return (-np.inf, 0.0, 0.0)
    s = 0.0
    t = 0.0
    for (mj, sj, tj) in parts:
        if np.isfinite(mj):
            w = np.exp(mj - m)
            s += sj * w
            t += tj * w
    return (m, s, t)


def ce_loss(logp, lens, T: int):
    """Cross-entropy over the target tokens (the L_CE term of Eq. 9).

    ``L_CE = -(1/N_v) sum_{valid i} logp_i`` and its gradient with respect to
    logp, ``g_i = -1/N_v`` on valid slots, 0 on padding.
    """
    mask, *_ = index_build(lens, T)
    nv = int(mask.sum())
    g = np.where(mask == 1, -1.0 / max(nv, 1), 0.0)
    return float(-(np.asarray(logp, dtype=np.float64) * mask).sum() / max(nv, 1)), g


# ---------------------------------------------------------------------------
# group-relative advantages (problem statement; not in the paper)
# ---------------------------------------------------------------------------

def group_advantage(reward, P: int, G: int, eps: float = 1e-6, ddof: int = 0):
    """A[p,g] = (r[p,g] - mean_g r[p,:]) / (std_g r[p,:] + eps), fp64[R].

    ``ddof`` 0 = population standard deviation (default), 1 = sample standard
    deviation (for G = 1 the sample std is taken as 0).  A group whose rewards
    are all equal gets A = 0.
    """
    r = np.asarray(reward, dtype=np.float64).reshape(P, G)
    A = np.zeros((P, G))
    for p in range(P):
        mu = r[p].sum() / G
        dev = r[p] - mu
        denom = G - ddof
        var = (dev * dev).sum() / denom if denom > 0 else 0.0
        A[p] = dev / (np.sqrt(var) + eps)
    return A.reshape(P * G)


# ---------------------------------------------------------------------------
# clipped importance-ratio surrogate with k3 KL (problem statement)
# ---------------------------------------------------------------------------

def _token_weights(lens, P, G, T, agg_mode):
    """Per-slot reduction weights w_i (0 on padding).

    agg_mode 0: mean over responses of the per-response token mean,
    ``w = 1/(R len_r)`` (a response of length 0 contributes nothing but still
    counts in R).  agg_mode 1: global token mean, ``w = 1/N_v``.
    """
    lens = np.asarray(lens, dtype=np.int64)
    R = P * G
    mask, *_ = index_build(lens, T)
    w = np.zeros((R, T))
    if agg_mode == 0:
        for r in range(R):
            if lens[r] > 0:
                w[r, :lens[r]] = 1.0 / (R * lens[r])
    elif agg_mode == 1:
        nv = int(lens.sum())
        if nv > 0:
            w[:] = 1.0 / nv
        w *= mask.reshape(R, T)
    else:
        raise ValueError("agg_mode")
    return w.reshape(R * T), mask


def grpo_loss(logp, logp_old, logp_ref, adv, lens, P, G, T,
              clip_lo: float = 0.2, clip_hi: float = 0.2, kl_coef: float = 0.04, agg_mode: int = 0):
    """Clipped surrogate + k3 KL penalty; returns (loss, g_logp fp64[N], stats fp64[4]).

    Per valid slot i of response r (advantage A = adv[r]):
      rho   = exp(logp - logp_old)
      surr  = min(rho * A, clip(rho, 1 - clip_lo, 1 + clip_hi) * A)
      delta = logp_ref - logp,   k3 = exp(delta) - delta - 1     (>= 0)
      l_i   = -surr + kl_coef * k3          (no KL term when logp_ref is None)
      L     = sum_i w_i l_i
    Gradient w.r.t. logp_i: the surrogate carries gradient ``rho * A`` exactly when
    the unclipped branch is the one selected by the min, i.e. when
    (A >= 0 and rho <= 1 + clip_hi) or (A < 0 and rho >= 1 - clip_lo) (on ties
    the unclipped branch is taken); d k3 / d logp = 1 - exp(delta).
      g_i = w_i * ( -A * rho * sel_i + kl_coef * (1 - exp(delta_i)) )
    stats = [fraction of valid tokens on the clipped branch, token-mean k3,
             token-mean rho, N_v].
    """
    lp = np.asarray(logp, dtype=np.float64)
    lo = np.asarray(logp_old, dtype=np.float64)
    R = P * G
    w, mask = _token_weights(lens, P, G, T, agg_mode)
    A = np.repeat(np.asarray(adv, dtype=np.float64).reshape(R), T)
    valid = mask == 1
    rho = np.exp(np.where(valid, lp - lo, 0.0))
    clipped = np.clip(rho, 1.0 - clip_lo, 1.0 + clip_hi)
    surr = np.minimum(rho * A, clipped * A)
    sel = np.where(A >= 0, rho <= 1.0 + clip_hi, rho >= 1.0 - clip_lo)
    if logp_ref is not None:
        delta = np.where(valid, np.asarray(logp_ref, dtype=np.float64) - lp, 0.0)
        k3 = np.exp(delta) - delta - 1.0
        dk3 = 1.0 - np.exp(delta)
    else:
        k3 = np.zeros_like(lp)
        dk3 = np.zeros_like(lp)
    ell = -surr + kl_coef * k3
    loss = float((w * ell).sum())
    g = w * (-A * rho * sel + kl_coef * dk3)
    nv = float(valid.sum())
    inv = 1.0 / nv if nv > 0 else 0.0
    stats = np.array([
        float((valid & ~sel).sum()) * inv,
        float(k3[valid].sum()) * inv,
        float(rho[valid].sum()) * inv,
        nv,
    ])
    return loss, g, stats


def grpo_abs_scale(logp, logp_old, logp_ref, adv, lens, P, G, T,
                   clip_lo=0.2, clip_hi=0.2, kl_coef=0.04, agg_mode=0):
    """sum_i w_i |l_i|: the magnitude against which a near-zero loss is compared."""
    lp = np.asarray(logp, dtype=np.float64)
    lo = np.asarray(logp_old, dtype=np.float64)
    w, mask = _token_weights(lens, P, G, T, agg_mode)
    A = np.repeat(np.asarray(adv, dtype=np.float64).reshape(P * G), T)
    valid = mask == 1
    rho = np.exp(np.where(valid, lp - lo, 0.0))
    surr = np.minimum(rho * A, np.clip(rho, 1.0 - clip_lo, 1.0 + clip_hi) * A)
    k3 = 0.0
    if logp_ref is not None:
        delta = np.where(valid, np.asarray(logp_ref, dtype=np.float64) - lp, 0.0)
        k3 = np.exp(delta) - delta - 1.0
    return float((w * np.abs(-surr + kl_coef * k3)).sum())


# ---------------------------------------------------------------------------
# trajectory-balance residual (problem statement)
# ---------------------------------------------------------------------------

def flowrl_tb_loss(logp, logp_ref, reward, logZ, lens, P, G, T, beta: float):
    """Squared trajectory-balance residual; returns (loss, g_logp[N], g_logZ[P], resid[R]).

    For response r of prompt p = r // G with length len_r:
      sbar_theta = (1/len_r) sum_t logp[r,t],  sbar_ref likewise (valid t only)
      delta_r = logZ[p] + sbar_theta - beta * reward[r] - sbar_ref
      L = (1/R) sum_r delta_r^2
      dL/dlogp[r,t] = 2 delta_r / (R len_r)   on valid slots
      dL/dlogZ[p]   = (2/R) sum_g delta_{pG+g}
    A response of length 0 has sbar = 0 for both policies.
    """
    R = P * G
    lens = np.asarray(lens, dtype=np.int64)
    lp = np.asarray(logp, dtype=np.float64).reshape(R, T)
    lr = np.asarray(logp_ref, dtype=np.float64).reshape(R, T)
    rew = np.asarray(reward, dtype=np.float64)
    lz = np.asarray(logZ, dtype=np.float64)
    resid = np.zeros(R)
    g = np.zeros((R, T))
    gz = np.zeros(P)
    for r in range(R):
        n = int(lens[r])
        st = lp[r, :n].sum() / n if n > 0 else 0.0
        sr = lr[r, :n].sum() / n if n > 0 else 0.0
        resid[r] = lz[r // G] + st - beta * rew[r] - sr
    loss = float((resid * resid).sum() / R)
    for r in range(R):
        n = int(lens[r])
        if n > 0:
            g[r, :n] = 2.0 * resid[r] / (R * n)
        gz[r // G] += 2.0 * resid[r] / R
    return loss, g.reshape(R * T), gz, resid


# ---------------------------------------------------------------------------
# backward through the softmax (softmax Jacobian; CE special case is Eq. 9's L_CE)
# ---------------------------------------------------------------------------

def bwd_rows(H_rows, W, tok_rows, g_rows, H_logits=None, W_logits=None):
    """Gradients of sum_i g_i * logp_i for the given rows (all treated as valid).

    ``H_logits`` / ``W_logits`` (default: H_rows / W) are the operands that the logits are formed
    from; the 8-bit variant passes the e4m3-rounded copies there while the two contractions below
    use the full-precision operands.

    ``d logp_i / d z_{i,v} = 1[v == y_i] - softmax(z_i)_v`` so
    ``dZ[i,v] = g_i (1[v == y_i] - exp(z_{i,v} - lse_i))``,
    ``dH[i,:] = sum_v dZ[i,v] W[v,:]`` and ``dW[v,:] = sum_i dZ[i,v] H[i,:]``
    (the latter is the contribution of these rows only).
    Returns (dH_rows fp64[n,d], dW fp64[V,d]).
    """
    H64 = np.asarray(H_rows, dtype=np.float64)
    W64 = np.asarray(W, dtype=np.float64)
    z = logits(H64 if H_logits is None else H_logits, W64 if W_logits is None else W_logits)
    n = z.shape[0]
    M = z.max(axis=1)
    lse = M + np.log(np.exp(z - M[:, None]).sum(axis=1))
    dZ = -np.exp(z - lse[:, None])
    dZ[np.arange(n), np.asarray(tok_rows, dtype=np.int64)] += 1.0
    dZ *= np.asarray(g_rows, dtype=np.float64)[:, None]
    return dZ @ W64, dZ.T @ H64


def lmhead_logprob_bwd(H, W, tok, lens, T: int, g_logp, block: int = 256, H_logits=None, W_logits=None):
    """dH (fp64[N,d], zero on padded rows) and dW (fp64[V,d]) for upstream g_logp[N]."""
    _, _, row_slot, _ = index_build(lens, T)
    H = np.asarray(H)
    tok = np.asarray(tok)
    g_logp = np.asarray(g_logp, dtype=np.float64)
    N, d = H.shape
    V = np.asarray(W).shape[0]
    dH = np.zeros((N, d))
    dW = np.zeros((V, d))
    for b0 in range(0, row_slot.size, block):
        rows = row_slot[b0:b0 + block]
        dh, dw = bwd_rows(H[rows], W, tok[rows], g_logp[rows],
                          None if H_logits is None else np.asarray(H_logits)[rows], W_logits)
        dH[rows] = dh
        dW += dw
    return dH, dW
