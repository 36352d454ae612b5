"""Pins of the KV-compression oracle against what the paper and the mathematics fix
(Sec. 3, Eqs. 1-9): closed forms, invariants, brute force on tiny inputs, library routines of
independent implementation, finite differences.  None of them re-evaluates the oracle's own formula.
"""
import math

import numpy as np
import pytest

import workloads as wl
import workloads.dynakv as kv
from oracle import dynakv_oracle as O


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_bf16_rounding_matches_torch_including_ties():
    import torch
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000),
                        # exact ties between two bf16 neighbours, both parities of the kept bit
                        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(2.0 + 2.0 ** -7), 0.0, 2.0 ** -130])])
    x = x.astype(np.float32).astype(np.float64)
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_to(x, "bf16"), want)
    assert O.round_to(1.0 + 2.0 ** -8, "bf16") == 1.0 and O.round_to(1.0 + 3 * 2.0 ** -8, "bf16") == 1.0 + 2.0 ** -6
    assert np.array_equal(O.round_to(x, None), x)


def test_spectral_and_probs_brute_force_tiny():
    n, d = 3, 5
    x, U, W, b = _rand(1, n, d), _rand(2, d, d), _rand(3, d, d), _rand(4, d)
    xt = O.spectral(x, U)
    p = O.gate_probs(xt, W, b)
    for i in range(n):
        row = [sum(x[i][k] * U[k][j] for k in range(d)) for j in range(d)]
        assert np.allclose(xt[i], row, rtol=1e-13, atol=1e-13)
        z = [sum(row[k] * W[k][j] for k in range(d)) + b[j] for j in range(d)]
        den = sum(math.exp(v) for v in z)                      # no max shift: tiny values
        assert np.allclose(p[i], [math.exp(v) / den for v in z], rtol=1e-12)
    # an operand passed transposed or a dropped bias changes the result
    assert not np.allclose(O.spectral(x, U.T), xt)
    assert not np.allclose(O.gate_probs(xt, W, 0 * b), p)


def test_probs_match_scipy_softmax_and_survive_large_logits():
    from scipy.special import softmax
    xt, W, b = _rand(5, 40, 24) * 30, _rand(6, 24, 24), _rand(7, 24) * 5
    p = O.gate_probs(xt, W, b)
    assert np.allclose(p, softmax(xt @ W + b, axis=1), rtol=1e-12, atol=0)
    assert np.all(np.isfinite(p)) and np.allclose(p.sum(1), 1.0, rtol=1e-13)


@pytest.mark.parametrize("order", ["suffix", "literal"])
def test_soft_mask_invariants(order):
    p = O.gate_probs(_rand(8, 50, 33), _rand(9, 33, 33), _rand(10, 33))
    m = O.soft_mask(p, order)
    assert np.allclose(m[:, 0], 1.0, rtol=1e-13)                # the whole distribution
    assert np.all(np.diff(m, axis=1) <= 1e-15)                  # non-increasing
    assert np.all(m >= 0) and np.all(m <= 1 + 1e-13)
    for tau in (0.0, 0.1, 0.5, 0.999):
        h = O.hard_mask(m, tau)
        k = O.retained(m, tau)
        for i in range(h.shape[0]):                             # a block of ones, then zeros
            assert np.all(h[i, : k[i]] == 1) and np.all(h[i, k[i]:] == 0)
        assert np.all(k >= 1)                                   # m_0 = 1 > tau
    assert np.all(O.retained(m, 0.0) == 33)                     # every m_i > 0: nothing is pruned


def test_soft_mask_brute_force_and_the_two_readings():
    p = O.gate_probs(_rand(11, 4, 7), _rand(12, 7, 7), _rand(13, 7))
    ms, ml = O.soft_mask(p, "suffix"), O.soft_mask(p, "literal")
    d = 7
    for i in range(4):
        for j in range(d):
            assert abs(ms[i, j] - sum(p[i, l] for l in range(j, d))) < 1e-14
            assert abs(ml[i, j] - sum(p[i, l] for l in range(0, d - j))) < 1e-14
    # the literal reading is the suffix reading of the column-reversed distribution
    assert np.allclose(ml, O.soft_mask(p[:, ::-1], "suffix"), rtol=1e-14)
    # differences of the mask give the distribution back (suffix: p_j = m_j - m_{j+1})
    ext = np.concatenate([ms, np.zeros((4, 1))], axis=1)
    assert np.allclose(ext[:, :-1] - ext[:, 1:], p, atol=1e-14)


def test_one_hot_cutoff_closed_form():
    # a bias spike at position c makes p one-hot: the mask is 1 up to and including c (suffix
    # reading: "about 1 for i < k, 0 for i > k"), so c + 1 components stay; the printed formula
    # keeps d - c of them
    d = 16
    for c in (0, 5, 15):
        b = np.zeros(d)
        b[c] = 200.0
        g = O.gate(np.zeros((2, d)), np.eye(d), np.zeros((d, d)), b, 0.1)
        assert np.all(g["k"] == c + 1)
        assert np.array_equal(g["m"][0] > 0.5, np.arange(d) <= c)
        g = O.gate(np.zeros((2, d)), np.eye(d), np.zeros((d, d)), b, 0.1, order="literal")
        assert np.all(g["k"] == d - c)


def test_uniform_cutoff_closed_form():
    # W = 0, b = 0: p = 1/d, m_i = (d - i)/d, k = #{i : (d - i)/d > tau}
    d = 16
    g = O.gate(_rand(14, 3, d), _rand(15, d, d), np.zeros((d, d)), np.zeros(d), 0.25)
    assert np.allclose(g["m"], (d - np.arange(d)) / d, rtol=1e-14)
    assert np.all(g["k"] == 12)
    assert O.retain_rate_hard(g["k"], d) == 12 / 16
    assert abs(O.retain_rate_soft(g["m"]) - (d + 1) / (2 * d)) < 1e-14


def test_soft_gating_is_elementwise_product():
    n, d = 6, 9
    x, U, W, b = _rand(16, n, d), _rand(17, d, d), _rand(18, d, d), _rand(19, d)
    g = O.gate(x, U, W, b, 0.1)
    for i in range(n):
        for j in range(d):
            assert abs(g["xhat"][i, j] - g["xt"][i, j] * g["m"][i, j]) < 1e-15
    gb = O.gate(x, U, W, b, 0.1, store_dtype="bf16")
    assert np.array_equal(gb["xt"], O.round_to(x @ U, "bf16"))
    assert np.array_equal(gb["xhat"], O.round_to(gb["xt"] * gb["m"], "bf16"))


def test_store_layout():
    xt = _rand(20, 7, 20)
    k = np.array([20, 1, 8, 9, 0, 16, 3], dtype=np.int32)
    off, packed = O.store(xt, k, granule=8)
    assert off.tolist() == [0, 24, 32, 40, 56, 56, 72, 80] and packed.size == 80
    for i in range(7):
        assert np.array_equal(packed[off[i]: off[i] + k[i]], xt[i, : k[i]])
        assert np.all(packed[off[i] + k[i]: off[i + 1]] == 0)
    off1, packed1 = O.store(xt, k, granule=1)                    # tight packing
    assert off1[-1] == k.sum() and np.array_equal(packed1, np.concatenate([xt[i, : k[i]] for i in range(7)]))


def test_round_trip_is_exact_when_nothing_is_pruned():
    # orthogonal U (the PCA initialisation), tau = 0: every component is kept and x_bar = x
    n, d = 9, 24
    q, _ = np.linalg.qr(_rand(21, d, d))
    x = _rand(22, n, d)
    g = O.gate(x, q, _rand(23, d, d), _rand(24, d), 0.0)
    assert np.all(g["k"] == d)
    off, packed = O.store(g["xt"], g["k"])
    assert np.allclose(O.reconstruct(packed, off, g["k"], q.T), x, atol=1e-13)


def test_truncation_is_an_orthogonal_projection():
    # orthogonal U: the reconstruction error is exactly the discarded spectral energy (Parseval),
    # and x_bar is the projection of x on the first k basis vectors
    n, d = 12, 20
    q, _ = np.linalg.qr(_rand(25, d, d))
    x = _rand(26, n, d)
    g = O.gate(x, q, _rand(27, d, d), 3 * _rand(28, d), 0.3)
    assert 1 < g["k"].min() and len(set(g["k"].tolist())) > 2
    off, packed = O.store(g["xt"], g["k"])
    xb = O.reconstruct(packed, off, g["k"], q.T)
    for i in range(n):
        k = g["k"][i]
        assert abs(((x[i] - xb[i]) ** 2).sum() - (g["xt"][i, k:] ** 2).sum()) < 1e-12
        proj = q[:, :k] @ (q[:, :k].T @ x[i])
        assert np.allclose(xb[i], proj, atol=1e-13)


def test_reconstruct_equals_masked_dense_product_for_a_general_basis():
    # Eq. 2 then Eq. 3 with the zeros left in: (x~ * m_hard) U^-1, a plain dense product
    n, d = 10, 16
    U = _rand(29, d, d) + 4 * np.eye(d)
    Ui = np.linalg.inv(U)
    x = _rand(30, n, d)
    g = O.gate(x, U, _rand(31, d, d), _rand(32, d), 0.2)
    off, packed = O.store(g["xt"], g["k"], granule=4)
    xb = O.reconstruct(packed, off, g["k"], Ui)
    dense = (g["xt"] * O.hard_mask(g["m"], 0.2)) @ Ui
    assert np.allclose(xb, dense, atol=1e-12)
    assert not np.allclose(xb, (g["xt"] * O.hard_mask(g["m"], 0.2)) @ Ui.T, atol=1e-6)   # transposed operand


def test_retain_rate_bounds_and_penalty_gradient():
    p = O.gate_probs(_rand(33, 30, 12), _rand(34, 12, 12), _rand(35, 12))
    m = O.soft_mask(p)
    k = O.retained(m, 0.1)
    R = O.retain_rate_hard(k, 12)
    assert 1 / 12 <= R <= 1
    assert R == sum(int(v) for v in k) / (30 * 12)
    pen, Rs, grad = O.retain_penalty(m, 0.7)
    assert abs(Rs - sum(m.ravel()) / m.size) < 1e-14 and abs(pen - 0.7 * Rs * Rs) < 1e-15
    h = 1e-6
    for (i, j) in ((0, 0), (7, 5), (29, 11)):
        a, bm = m.copy(), m.copy()
        a[i, j] += h
        bm[i, j] -= h
        fd = (O.retain_penalty(a, 0.7)[0] - O.retain_penalty(bm, 0.7)[0]) / (2 * h)
        assert abs(fd - grad[i, j]) < 1e-9
    assert O.retain_rate_hard(np.zeros(0, dtype=np.int32), 12) == 0.0


def test_synthetic_workload_is_token_adaptive():
    cfg = kv.KV_CONFIGS[1].scaled(n=256)
    inp = kv.kv_inputs(cfg)
    assert inp["x"].dtype == np.uint16 and inp["x"].shape == (256, cfg.d)
    again = kv.kv_inputs(cfg)
    assert all(np.array_equal(inp[key], again[key]) for key in inp)
    U, Ui = wl.as_f64(inp["U"]), wl.as_f64(inp["U_inv"])
    assert np.abs(U @ Ui - np.eye(cfg.d)).max() < 0.05              # inverse up to storage rounding
    g = O.gate(wl.as_f64(inp["x"]), U, wl.as_f64(inp["W"]), inp["b"], cfg.tau, store_dtype="bf16")
    R = O.retain_rate_hard(g["k"], cfg.d)
    assert 0.25 < R < 0.7 and g["k"].std() > 0.03 * cfg.d           # cut-offs differ token by token
    e = (g["xt"] ** 2).sum(0)
    assert e[: cfg.d // 4].sum() > 0.6 * e.sum()                    # energy sits in the leading components


@pytest.mark.parametrize("order", ["suffix", "literal"])
def test_gate_backward_matches_finite_differences(order):
    n, d = 4, 6
    x, U, W, b = _rand(40, n, d), _rand(41, d, d), 0.7 * _rand(42, d, d), _rand(43, d)
    G, Gm = _rand(44, n, d), _rand(45, n, d)

    def loss(x, U, W, b):
        g = O.gate(x, U, W, b, 0.1, order=order)
        return float((G * g["xhat"]).sum() + (Gm * g["m"]).sum())

    got = O.gate_bwd(x, U, W, b, G, Gm, order=order)
    h = 1e-6
    for name, arr, key in (("x", x, "dx"), ("U", U, "dU"), ("W", W, "dW"), ("b", b, "db")):
        fd = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += h
            lo[idx] -= h
            args = {"x": x, "U": U, "W": W, "b": b}
            fd[idx] = (loss(**{**args, name: hi}) - loss(**{**args, name: lo})) / (2 * h)
        assert np.abs(fd - got[key]).max() <= 1e-6 * max(1.0, np.abs(fd).max()), name


def test_gate_backward_identities():
    n, d = 7, 9
    x, U, W, b = _rand(46, n, d), _rand(47, d, d), _rand(48, d, d), _rand(49, d)
    G = _rand(50, n, d)
    got = O.gate_bwd(x, U, W, b, G)
    assert np.abs(got["g_l"].sum(axis=1)).max() < 1e-13             # softmax Jacobian annihilates constants
    assert np.allclose(got["db"], got["g_l"].sum(axis=0))
    # a mask gradient that is constant over a token's positions and over tokens, c, adds c * (j + 1) to
    # dL/dp_j: the regulariser of Eq. 9 pushes probability mass towards early cut-offs
    c = 0.37
    plus = O.gate_bwd(x, U, W, b, G, np.full((n, d), c))
    p = O.gate_probs(x @ U, W, b)
    r = c * (np.arange(d) + 1.0)
    extra = p * (r - (p * r).sum(axis=1, keepdims=True))
    assert np.allclose(plus["g_l"] - got["g_l"], extra, atol=1e-12)
    # with no gate dependence (W = 0) only the direct path x^ = x~ * m remains for x and U, and W's
    # gradient still sees the mask
    z = O.gate_bwd(x, U, 0 * W, b, G)
    m = O.soft_mask(O.gate_probs(x @ U, 0 * W, b))
    assert np.allclose(z["dx"], (G * m) @ U.T, atol=1e-12) and np.allclose(z["dU"], x.T @ (G * m), atol=1e-12)
