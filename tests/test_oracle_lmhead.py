"""Pins for the oracle's LM-head part: logits, log-sum-exp, target log-prob, entropy, merge rule.

Each test checks the oracle against something other than itself: a closed form,
a brute-force loop written with ``math`` only, an invariant, or an independent
library routine (torch / scipy).
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import lmhead_oracle as O


def _rand(n, d, V, seed=0, scale=1.0):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((n, d))
    W = rng.standard_normal((V, d)) * scale
    tok = rng.integers(0, V, size=n)
    return H, W, tok


def test_uniform_logits_closed_form():
    # identical rows of W (or H = 0) make every logit of a row equal: logp = -ln V, ent = ln V
    rng = np.random.default_rng(1)
    V, d, n = 37, 5, 6
    H = rng.standard_normal((n, d))
    W = np.tile(rng.standard_normal((1, d)), (V, 1))
    tok = rng.integers(0, V, size=n)
    lp, lse, ent = O.logprob_rows(H, W, tok)
    assert np.allclose(lp, -math.log(V), atol=1e-12)
    assert np.allclose(ent, math.log(V), atol=1e-12)
    lp0, _, ent0 = O.logprob_rows(np.zeros((n, d)), rng.standard_normal((V, d)), tok)
    assert np.allclose(lp0, -math.log(V), atol=1e-12)
    assert np.allclose(ent0, math.log(V), atol=1e-12)


def test_bruteforce_tiny_vocab():
    # pure-Python evaluation without any max shift
    H, W, tok = _rand(4, 3, 7, seed=2)
    lp, lse, ent = O.logprob_rows(H, W, tok)
    for i in range(4):
        z = [sum(H[i, k] * W[v, k] for k in range(3)) for v in range(7)]
        total = sum(math.exp(zz) for zz in z)
        assert abs(lse[i] - math.log(total)) < 1e-12
        assert abs(lp[i] - (z[tok[i]] - math.log(total))) < 1e-12
        p = [math.exp(zz) / total for zz in z]
        assert abs(ent[i] - (-sum(pp * math.log(pp) for pp in p))) < 1e-12


def test_logits_orientation():
    # z[i, v] must be <H[i], W[v]>: a transposed operand changes a non-square example
    H = np.array([[1.0, 2.0, 3.0]])
    W = np.array([[1.0, 0.0, 0.0], [0.0, 1.0, 0.0], [0.0, 0.0, 1.0], [1.0, 1.0, 1.0]])
    assert np.array_equal(O.logits(H, W), np.array([[1.0, 2.0, 3.0, 6.0]]))


def test_shift_invariance():
    # adding u to every row of W shifts all logits of row i by H[i].u: logp and ent unchanged
    H, W, tok = _rand(5, 4, 19, seed=3)
    u = np.random.default_rng(4).standard_normal(4)
    lp, lse, ent = O.logprob_rows(H, W, tok)
    lp2, lse2, ent2 = O.logprob_rows(H, W + u[None, :], tok)
    assert np.allclose(lp, lp2, atol=1e-11)
    assert np.allclose(ent, ent2, atol=1e-11)
    assert np.allclose(lse2 - lse, H @ u, atol=1e-11)


def test_probabilities_sum_to_one():
    H, W, _ = _rand(3, 4, 11, seed=5)
    tot = np.zeros(3)
    for v in range(11):
        lp, _, _ = O.logprob_rows(H, W, np.full(3, v))
        tot += np.exp(lp)
    assert np.allclose(tot, 1.0, atol=1e-12)


def test_dominant_logit():
    # one logit far above the rest: logp -> 0, ent -> 0; exponent of 50+ must not overflow
    V, d = 16, 4
    W = np.zeros((V, d))
    W[3, 0] = 800.0
    H = np.zeros((2, d))
    H[:, 0] = 1.0
    lp, lse, ent = O.logprob_rows(H, W, np.array([3, 5]))
    assert abs(lp[0]) < 1e-12 and abs(ent[0]) < 1e-12
    assert abs(lp[1] + 800.0) < 1e-9
    assert np.all(np.isfinite(lse))


def test_against_library_routines():
    H, W, tok = _rand(9, 8, 53, seed=6, scale=0.7)
    lp, lse, ent = O.logprob_rows(H, W, tok)
    z = H @ W.T
    assert np.allclose(lse, scipy.special.logsumexp(z, axis=1), atol=1e-12)
    tz = torch.from_numpy(z)
    ce = torch.nn.functional.cross_entropy(tz, torch.from_numpy(tok), reduction="none").numpy()
    assert np.allclose(-lp, ce, atol=1e-12)
    ent_t = torch.distributions.Categorical(logits=tz).entropy().numpy()
    assert np.allclose(ent, ent_t, atol=1e-12)


def test_entropy_bounds():
    H, W, tok = _rand(20, 6, 33, seed=7, scale=2.0)
    _, _, ent = O.logprob_rows(H, W, tok)
    assert np.all(ent >= 0) and np.all(ent <= math.log(33) + 1e-12)


def test_fwd_padding_and_rows():
    # padded slots give 0; valid slots equal the row-wise routine; garbage ids on padding are ignored
    rng = np.random.default_rng(8)
    R, T, d, V = 3, 5, 4, 13
    lens = np.array([5, 0, 2])
    H = rng.standard_normal((R * T, d))
    W = rng.standard_normal((V, d))
    tok = rng.integers(0, V, size=R * T)
    mask, cu, rs, rr = O.index_build(lens, T)
    tok_bad = tok.copy()
    tok_bad[mask == 0] = -12345
    lp, lse, ent = O.lmhead_logprob_fwd(H, W, tok_bad, lens, T, block=3)
    assert np.all(lp[mask == 0] == 0) and np.all(lse[mask == 0] == 0) and np.all(ent[mask == 0] == 0)
    lp2, lse2, ent2 = O.logprob_rows(H[rs], W, tok[rs])
    assert np.array_equal(lp[rs], lp2) and np.array_equal(lse[rs], lse2) and np.array_equal(ent[rs], ent2)


def test_index_build_bruteforce():
    rng = np.random.default_rng(9)
    T = 7
    lens = rng.integers(0, T + 1, size=11)
    mask, cu, rs, rr = O.index_build(lens, T)
    exp_mask, exp_rs, exp_rr, exp_cu = [], [], [], [0]
    for r, n in enumerate(lens):
        for t in range(T):
            exp_mask.append(1 if t < n else 0)
            if t < n:
                exp_rs.append(r * T + t)
                exp_rr.append(r)
        exp_cu.append(exp_cu[-1] + int(n))
    assert mask.dtype == np.uint8 and mask.tolist() == exp_mask
    assert cu.tolist() == exp_cu and rs.tolist() == exp_rs and rr.tolist() == exp_rr
    with pytest.raises(ValueError):
        O.index_build([T + 1], T)
    with pytest.raises(ValueError):
        O.index_build([-1], T)


def test_token_range_checked():
    H, W, tok = _rand(2, 3, 5, seed=10)
    with pytest.raises(ValueError):
        O.logprob_rows(H, W, np.array([0, 5]))


def test_merge_rule_on_random_splits():
    # statistics of a row split into arbitrary column ranges merge to the unsplit statistics
    rng = np.random.default_rng(11)
    for trial in range(20):
        V = int(rng.integers(2, 40))
        z = rng.standard_normal(V) * 5
        cuts = np.sort(rng.choice(np.arange(1, V), size=min(V - 1, int(rng.integers(0, 5))), replace=False))
        parts = []
        for seg in np.split(z, cuts):
            m = seg.max()
            parts.append((m, np.exp(seg - m).sum(), (np.exp(seg - m) * seg).sum()))
        parts.insert(int(rng.integers(0, len(parts) + 1)), (-np.inf, 0.0, 0.0))  # an empty range
        m, s, t = O.lse_merge(parts)
        total = sum(math.exp(v) for v in z)
        assert abs((m + math.log(s)) - math.log(total)) < 1e-12
        assert abs(t / s - sum(math.exp(v) * v for v in z) / total) < 1e-12
    assert O.lse_merge([(-np.inf, 0.0, 0.0)]) == (-np.inf, 0.0, 0.0)


def test_ce_loss_matches_library():
    # L_CE of the training objective = mean token cross-entropy over valid targets
    rng = np.random.default_rng(12)
    R, T, d, V = 4, 6, 5, 17
    lens = np.array([6, 3, 1, 4])
    H = rng.standard_normal((R * T, d))
    W = rng.standard_normal((V, d))
    tok = rng.integers(0, V, size=R * T)
    lp, _, _ = O.lmhead_logprob_fwd(H, W, tok, lens, T)
    loss, g = O.ce_loss(lp, lens, T)
    mask, *_ = O.index_build(lens, T)
    z = torch.from_numpy(H @ W.T)
    target = torch.from_numpy(np.where(mask == 1, tok, -100))
    ref = torch.nn.functional.cross_entropy(z, target, ignore_index=-100, reduction="mean").item()
    assert abs(loss - ref) < 1e-12
    assert np.allclose(g[mask == 1], -1.0 / lens.sum()) and np.all(g[mask == 0] == 0)


def test_e4m3_rounding_matches_torch_and_the_format():
    import torch
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-4, 3, 20000),
                        [0.0, 1.0, 1.0625, 1.1875, 448.0, 464.0, 2.0 ** -9, 2.0 ** -10, 1.5 * 2.0 ** -9, -0.3, 17.0, 19.0]])
    x = x[np.abs(x) < 464]                                          # beyond that the raw conversion gives NaN
    want = torch.from_numpy(x.astype(np.float32)).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = O.quantize_e4m3(x.astype(np.float32), 0)
    assert np.array_equal(got, want)
    # every result is on the grid: 3 mantissa bits, exponent in [-6, 8], subnormal step 2^-9
    nz = got[got != 0]
    m, e = np.frexp(np.abs(nz))
    assert np.all((m * 16) % 1 == 0) or np.all(np.abs(nz) < 2.0 ** -6)
    assert np.abs(got).max() <= 448
    # saturation and scaling by a power of two (exact): q(x, e) = q(x * 2^e, 0) / 2^e
    assert O.quantize_e4m3(1e9, 0) == 448 and O.quantize_e4m3(-500.0, 0) == -448
    w = rng.standard_normal(1000) * 0.02
    assert np.array_equal(O.quantize_e4m3(w, 12), O.quantize_e4m3(w * 4096, 0) / 4096)
    # relative error of a normal number is at most 2^-4
    big = w[np.abs(w) * 4096 >= 2.0 ** -6]
    assert np.all(np.abs(O.quantize_e4m3(big, 12) - big) <= np.abs(big) * 2.0 ** -4)


def test_backward_with_separate_logit_operands():
    # the 8-bit variant: logits from rounded copies, contractions with the originals; with identical
    # copies it is the ordinary backward, and dZ only depends on the logit operands
    rng = np.random.default_rng(4)
    H, W = rng.standard_normal((6, 8)), rng.standard_normal((11, 8))
    tok, g = rng.integers(0, 11, 6), rng.standard_normal(6)
    a = O.bwd_rows(H, W, tok, g)
    b = O.bwd_rows(H, W, tok, g, H.copy(), W.copy())
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    Hq, Wq = O.quantize_e4m3(H, 5), O.quantize_e4m3(W, 5)
    dH, dW = O.bwd_rows(H, W, tok, g, Hq, Wq)
    z = Hq @ Wq.T
    p = np.exp(z) / np.exp(z).sum(1, keepdims=True)
    dZ = -p * g[:, None]
    dZ[np.arange(6), tok] += g
    assert np.allclose(dH, dZ @ W, atol=1e-13) and np.allclose(dW, dZ.T @ H, atol=1e-13)
