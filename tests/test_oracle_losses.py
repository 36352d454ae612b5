"""Pins for the oracle's advantage / GRPO / trajectory-balance parts.

These formulas come from the benchmark's problem statement (the paper does not
state them), so they are pinned by invariants, closed forms, pure-Python brute
force, finite differences and torch autograd over an independent re-statement.
"""
import math

import numpy as np
import pytest
import torch

from oracle import lmhead_oracle as O


# ------------------------------------------------------------------ advantages

def test_advantage_zero_mean_unit_std():
    rng = np.random.default_rng(0)
    P, G = 5, 8
    r = rng.random(P * G)
    for ddof in (0, 1):
        A = O.group_advantage(r, P, G, eps=0.0, ddof=ddof).reshape(P, G)
        assert np.allclose(A.mean(axis=1), 0, atol=1e-12)
        assert np.allclose(A.std(axis=1, ddof=ddof), 1, atol=1e-12)


def test_advantage_against_torch_and_affine_invariance():
    rng = np.random.default_rng(1)
    P, G = 3, 6
    r = rng.random(P * G)
    t = torch.from_numpy(r).reshape(P, G)
    for ddof in (0, 1):
        ref = ((t - t.mean(1, keepdim=True)) / (t.std(1, correction=ddof, keepdim=True) + 1e-6)).reshape(-1).numpy()
        A = O.group_advantage(r, P, G, eps=1e-6, ddof=ddof)
        assert np.allclose(A, ref, atol=1e-12)
    A0 = O.group_advantage(r, P, G, eps=0.0)
    A1 = O.group_advantage(3.5 * r - 2.0, P, G, eps=0.0)
    assert np.allclose(A0, A1, atol=1e-10)


def test_advantage_degenerate_group_and_binary_closed_form():
    # all-equal rewards -> exactly 0; binary rewards with k ones of G: A(1) = sqrt((G-k)/k), A(0) = -sqrt(k/(G-k))
    r = np.array([1, 1, 1, 1, 0, 1, 0, 0], dtype=float)
    A = O.group_advantage(r, 2, 4, eps=1e-6)
    assert np.all(A[:4] == 0)
    A = O.group_advantage(r[4:], 1, 4, eps=0.0)
    assert np.allclose(A, [-math.sqrt(1 / 3), math.sqrt(3), -math.sqrt(1 / 3), -math.sqrt(1 / 3)], atol=1e-12)
    assert np.all(O.group_advantage(np.array([0.3, 0.9]), 2, 1, ddof=1) == 0)  # G = 1


# ------------------------------------------------------------------------ GRPO

def _grpo_case(seed=0, P=2, G=3, T=5, spread=0.5):
    rng = np.random.default_rng(seed)
    R = P * G
    lens = rng.integers(1, T + 1, size=R)
    lp = -rng.random(R * T) * 3
    lo = lp + rng.standard_normal(R * T) * spread
    lr = lp + rng.standard_normal(R * T) * spread
    adv = rng.standard_normal(R)
    return lp, lo, lr, adv, lens, P, G, T


def test_grpo_bruteforce_python():
    lp, lo, lr, adv, lens, P, G, T = _grpo_case(1)
    for agg in (0, 1):
        loss, g, stats = O.grpo_loss(lp, lo, lr, adv, lens, P, G, T, 0.2, 0.3, 0.04, agg)
        R = P * G
        nv = int(lens.sum())
        tot = 0.0
        for r in range(R):
            for t in range(int(lens[r])):
                i = r * T + t
                rho = math.exp(lp[i] - lo[i])
                c = min(max(rho, 0.8), 1.3)
                s = min(rho * adv[r], c * adv[r])
                dl = lr[i] - lp[i]
                k3 = math.exp(dl) - dl - 1
                w = 1 / (R * lens[r]) if agg == 0 else 1 / nv
                tot += w * (-s + 0.04 * k3)
        assert abs(loss - tot) < 1e-12


def test_grpo_same_policy_closed_forms():
    lp, lo, lr, adv, lens, P, G, T = _grpo_case(2)
    # pi_theta == pi_old: rho = 1 exactly, surrogate = A, so L = -mean_r A_r (no KL)
    loss, g, stats = O.grpo_loss(lp, lp, None, adv, lens, P, G, T, 0.2, 0.2, 0.04, 0)
    assert stats[2] == 1.0 and stats[0] == 0.0
    assert abs(loss + adv.mean()) < 1e-12
    mask, *_ = O.index_build(lens, T)
    w = np.repeat(1.0 / (P * G * lens), T) * mask
    assert np.allclose(g, -np.repeat(adv, T) * w, atol=1e-15)
    # pi_theta == pi_ref: k3 = 0 and its gradient is 0
    loss2, g2, stats2 = O.grpo_loss(lp, lp, lp, adv, lens, P, G, T, 0.2, 0.2, 7.0, 0)
    assert stats2[1] == 0.0 and abs(loss2 - loss) < 1e-15 and np.allclose(g2, g, atol=1e-15)


def test_grpo_k3_nonnegative_and_zero_advantage():
    lp, lo, lr, adv, lens, P, G, T = _grpo_case(3, spread=1.5)
    loss, g, stats = O.grpo_loss(lp, lo, lr, np.zeros_like(adv), lens, P, G, T, 0.2, 0.2, 0.04, 0)
    assert stats[1] >= 0 and loss >= 0   # only the KL term remains
    mask, *_ = O.index_build(lens, T)
    w = np.repeat(1.0 / (P * G * lens), T) * mask
    assert np.allclose(g, 0.04 * w * (1 - np.exp(lr - lp)), atol=1e-14)


def test_grpo_wide_clip_is_plain_importance_weighting():
    lp, lo, lr, adv, lens, P, G, T = _grpo_case(4)
    loss, g, stats = O.grpo_loss(lp, lo, None, adv, lens, P, G, T, 1.0, 1e9, 0.0, 1)
    mask, *_ = O.index_build(lens, T)
    rho = np.exp(lp - lo)
    ref = -(rho * np.repeat(adv, T) * mask).sum() / lens.sum()
    assert abs(loss - ref) < 1e-12 and stats[0] == 0.0


def test_grpo_clip_branches():
    # one response, one token each case: (A>0, rho>1+eps) clipped & no gradient; (A<0, rho>1+eps) unclipped
    P, G, T = 1, 1, 1
    for A, dlp, want_val, want_sel in [
        (2.0, math.log(1.5), 1.2 * 2.0, 0),
        (-2.0, math.log(1.5), 1.5 * -2.0, 1),
        (2.0, math.log(0.5), 0.5 * 2.0, 1),
        (-2.0, math.log(0.5), 0.8 * -2.0, 0),
        (2.0, 0.0, 2.0, 1),
    ]:
        loss, g, stats = O.grpo_loss([dlp], [0.0], None, [A], [1], P, G, T, 0.2, 0.2, 0.0, 0)
        assert abs(loss + want_val) < 1e-12
        assert abs(g[0] - (-A * math.exp(dlp) * want_sel)) < 1e-12
        assert stats[0] == 1 - want_sel


def test_grpo_gradient_vs_autograd_and_fd():
    lp, lo, lr, adv, lens, P, G, T = _grpo_case(5)
    for agg in (0, 1):
        loss, g, _ = O.grpo_loss(lp, lo, lr, adv, lens, P, G, T, 0.2, 0.25, 0.04, agg)
        # independent re-statement in torch with autograd
        R = P * G
        x = torch.tensor(lp, requires_grad=True)
        mask, *_ = O.index_build(lens, T)
        m = torch.from_numpy(mask.astype(np.float64))
        A = torch.from_numpy(np.repeat(adv, T))
        ratio = torch.exp(x - torch.from_numpy(lo))
        s = torch.minimum(ratio * A, torch.clamp(ratio, 0.8, 1.25) * A)
        dl = torch.from_numpy(lr) - x
        ell = -s + 0.04 * (torch.exp(dl) - dl - 1)
        if agg == 0:
            w = m / torch.from_numpy(np.repeat(lens.astype(np.float64), T)) / R
        else:
            w = m / float(lens.sum())
        L = (w * ell).sum()
        L.backward()
        assert abs(L.item() - loss) < 1e-12
        assert np.allclose(x.grad.numpy(), g, atol=1e-13)
        # central differences on a few entries
        for i in np.nonzero(mask)[0][:6]:
            h = 1e-6
            a = lp.copy(); a[i] += h
            b = lp.copy(); b[i] -= h
            fd = (O.grpo_loss(a, lo, lr, adv, lens, P, G, T, 0.2, 0.25, 0.04, agg)[0]
                  - O.grpo_loss(b, lo, lr, adv, lens, P, G, T, 0.2, 0.25, 0.04, agg)[0]) / (2 * h)
            assert abs(fd - g[i]) < 1e-7
        assert np.all(g[mask == 0] == 0)


def test_grpo_abs_scale_bruteforce_python():
    # sum_i w_i |l_i| term by term, both aggregation modes, with and without the KL term; a scale off by
    # a constant factor (which would loosen every near-zero loss tolerance) fails here
    lp, lo, lr, adv, lens, P, G, T = _grpo_case(7, spread=1.0)
    R, nv = P * G, int(lens.sum())
    for agg in (0, 1):
        for ref in (lr, None):
            tot = 0.0
            for r in range(R):
                for t in range(int(lens[r])):
                    i = r * T + t
                    rho = math.exp(lp[i] - lo[i])
                    s = min(rho * adv[r], min(max(rho, 0.75), 1.25) * adv[r])
                    k3 = 0.0
                    if ref is not None:
                        dl = ref[i] - lp[i]
                        k3 = math.exp(dl) - dl - 1
                    w = 1 / (R * lens[r]) if agg == 0 else 1 / nv
                    tot += w * abs(-s + 0.07 * k3)
            got = O.grpo_abs_scale(lp, lo, ref, adv, lens, P, G, T, 0.25, 0.25, 0.07, agg)
            assert abs(got - tot) < 1e-12 * max(1.0, tot)
    # single token, hand value: A = 2, rho = 1, no KL: |l| = 2, w = 1
    one = O.grpo_abs_scale(np.array([-1.0]), np.array([-1.0]), None, np.array([2.0]), np.array([1]), 1, 1, 1)
    assert one == 2.0


def test_grpo_abs_scale_bounds_loss():
    lp, lo, lr, adv, lens, P, G, T = _grpo_case(6)
    loss, _, _ = O.grpo_loss(lp, lo, lr, adv, lens, P, G, T)
    assert O.grpo_abs_scale(lp, lo, lr, adv, lens, P, G, T) >= abs(loss) - 1e-15


# ------------------------------------------------------------- trajectory balance

def _tb_case(seed=0, P=3, G=4, T=6):
    rng = np.random.default_rng(seed)
    R = P * G
    lens = rng.integers(1, T + 1, size=R)
    lp = -rng.random(R * T) * 3
    lr = -rng.random(R * T) * 3
    rew = rng.random(R)
    lz = rng.standard_normal(P)
    return lp, lr, rew, lz, lens, P, G, T


def test_tb_bruteforce_python():
    lp, lr, rew, lz, lens, P, G, T = _tb_case(1)
    beta = 15.0
    loss, g, gz, resid = O.flowrl_tb_loss(lp, lr, rew, lz, lens, P, G, T, beta)
    tot = 0.0
    for r in range(P * G):
        n = int(lens[r])
        st = sum(lp[r * T + t] for t in range(n)) / n
        sr = sum(lr[r * T + t] for t in range(n)) / n
        dl = lz[r // G] + st - beta * rew[r] - sr
        assert abs(dl - resid[r]) < 1e-12
        tot += dl * dl
    assert abs(loss - tot / (P * G)) < 1e-12 and loss >= 0


def test_tb_residual_vanishes_at_optimum():
    lp, lr, rew, lz, lens, P, G, T = _tb_case(2)
    beta = 2.5
    R = P * G
    mask, *_ = O.index_build(lens, T)
    st = (lp * mask).reshape(R, T).sum(1) / lens
    sr = (lr * mask).reshape(R, T).sum(1) / lens
    # (i) one logZ per response (P' = R, G' = 1): logZ* = beta r + sbar_ref - sbar_theta gives delta = 0
    loss, g, gz, resid = O.flowrl_tb_loss(lp, lr, rew, beta * rew + sr - st, lens, R, 1, T, beta)
    assert np.allclose(resid, 0, atol=1e-12) and loss < 1e-24 and np.allclose(g, 0, atol=1e-13)
    # (ii) per prompt: logZ*_p = -mean_g a, a = sbar_theta - beta r - sbar_ref: mean residual and g_logZ vanish,
    #      and the loss is the mean within-group variance of a
    a = (st - beta * rew - sr).reshape(P, G)
    loss, g, gz, resid = O.flowrl_tb_loss(lp, lr, rew, -a.mean(1), lens, P, G, T, beta)
    assert np.allclose(resid.reshape(P, G).sum(1), 0, atol=1e-12)
    assert np.allclose(gz, 0, atol=1e-13)
    assert abs(loss - a.var(axis=1).mean()) < 1e-12


def test_tb_gradient_structure_and_fd():
    lp, lr, rew, lz, lens, P, G, T = _tb_case(3)
    beta = 15.0
    R = P * G
    loss, g, gz, resid = O.flowrl_tb_loss(lp, lr, rew, lz, lens, P, G, T, beta)
    g2 = g.reshape(R, T)
    for r in range(R):
        n = int(lens[r])
        assert np.all(g2[r, :n] == g2[r, 0]) and np.all(g2[r, n:] == 0)
        assert abs(g2[r].sum() - 2 * resid[r] / R) < 1e-13
    h = 1e-6
    for i in np.nonzero(O.index_build(lens, T)[0])[0][:8]:
        a = lp.copy(); a[i] += h
        b = lp.copy(); b[i] -= h
        fd = (O.flowrl_tb_loss(a, lr, rew, lz, lens, P, G, T, beta)[0]
              - O.flowrl_tb_loss(b, lr, rew, lz, lens, P, G, T, beta)[0]) / (2 * h)
        assert abs(fd - g[i]) < 1e-6
    for p in range(P):
        a = lz.copy(); a[p] += h
        b = lz.copy(); b[p] -= h
        fd = (O.flowrl_tb_loss(lp, lr, rew, a, lens, P, G, T, beta)[0]
              - O.flowrl_tb_loss(lp, lr, rew, b, lens, P, G, T, beta)[0]) / (2 * h)
        assert abs(fd - gz[p]) < 1e-6


def test_tb_zero_length_response():
    lp, lr, rew, lz, lens, P, G, T = _tb_case(4)
    lens = lens.copy(); lens[2] = 0
    loss, g, gz, resid = O.flowrl_tb_loss(lp, lr, rew, lz, lens, P, G, T, 1.0)
    assert abs(resid[2] - (lz[0] - rew[2])) < 1e-15
    assert np.all(g.reshape(P * G, T)[2] == 0)
