"""GPU parity of dynakv_gate_bwd (include/dynakv.h) against the fp64 oracle's chain rule on the same
seeded inputs, through the C ABI.

Tolerance: relative Frobenius error <= 1e-2 for every gradient (dx, dU, dW, db), the bound used for
the other matrix outputs of this library.  The kernel rounds the two token-major gradients (g_l and
g_x~) to the storage type before they enter the matrix cores (2^-9 relative per element for bf16)
and accumulates in fp32; the oracle rounds nothing but x~.  Observed errors are a few 1e-3 for bf16
and below 1e-5 for fp32 (asserted at 1e-4).
"""
import numpy as np
import pytest

import workloads as wl
import workloads.dynakv as kv
from oracle import dynakv_oracle as O
from tests.harness import KvProblem, np64, rel_fro, to_device

pytestmark = pytest.mark.gpu


def _tol(cfg):
    return 1e-2 if cfg.dtype == "bf16" else 1e-4


def _oracle_bwd(cfg, inp, g_xhat, g_m, g_m_const, order):
    f = wl.as_f64
    gm = None if g_m is None else g_m.astype(np.float64)
    if g_m_const:
        gm = (0.0 if gm is None else gm) + np.full((cfg.n, cfg.d), g_m_const)
    return O.gate_bwd(f(inp["x"]), f(inp["U"]), f(inp["W"]), inp["b"], f(g_xhat), gm, order=order,
                      store_dtype=cfg.dtype)


def _bwd_parity(cfg, inp, with_g_m=True, g_m_const=0.0, literal=False, ldx=None):
    order = "literal" if literal else "suffix"
    g_xhat, g_m = kv.upstream(cfg, with_g_m=with_g_m)
    o = _oracle_bwd(cfg, inp, g_xhat, g_m, g_m_const, order)
    kp = KvProblem(cfg, inp, flags=1 if literal else 0, ldx=ldx)
    xt, _, _, _ = kp.gate(cfg.tau, soft=False)
    dx, dU, dW, db = kp.gate_bwd(xt, to_device(g_xhat), None if g_m is None else to_device(g_m), g_m_const)
    assert kp.check() == 0
    tol = _tol(cfg)
    errs = {name: rel_fro(np64(got), o[name]) for name, got in (("dx", dx), ("dU", dU), ("dW", dW), ("db", db))}
    assert all(e <= tol for e in errs.values()), errs
    return kp, o, xt, (dx, dU, dW, db), errs


@pytest.mark.parametrize("literal", [False, True])
def test_tiny_fp32_backward(literal):
    cfg = kv.KV_CONFIGS[0]
    _bwd_parity(cfg, kv.kv_inputs(cfg), with_g_m=True, g_m_const=1e-3, literal=literal)


@pytest.mark.parametrize("literal", [False, True])
def test_small_bf16_backward(literal):
    cfg = kv.KV_CONFIGS[1]
    inp = kv.kv_inputs(cfg)
    kp, o, xt, (dx, dU, dW, db), errs = _bwd_parity(cfg, inp, with_g_m=True, literal=literal)
    # a transposed or swapped operand would not pass: the gradients are far from their transposes
    assert rel_fro(np64(dW).T, o["dW"]) > 0.5 and rel_fro(np64(dU).T, o["dU"]) > 0.5
    # every row of g_l sums to 0 (softmax Jacobian), so db and the rows of dW sum to ~0
    assert abs(np64(db).sum()) <= 1e-3 * np.abs(np64(db)).sum()


def test_backward_with_the_regulariser_gradient_only_as_a_constant():
    # dL/dm = 2 alpha R / (n d) for every element (Eq. 9), no other gradient on the mask, strided x
    cfg = kv.KV_CONFIGS[1].scaled(n=777, d=320)
    _bwd_parity(cfg, kv.kv_inputs(cfg), with_g_m=False, g_m_const=2 * 0.5 * 0.44 / (777 * 320), ldx=384)


def test_backward_accumulates_parameter_gradients_on_request():
    import torch
    cfg = kv.KV_CONFIGS[1].scaled(n=600, d=256)
    inp = kv.kv_inputs(cfg)
    kp, o, xt, (dx, dU, dW, db), _ = _bwd_parity(cfg, inp, with_g_m=False)
    g_xhat, _ = kv.upstream(cfg)
    base = [torch.full_like(t, 0.25) for t in (dU, dW, db)]
    dx2, dU2, dW2, db2 = kp.gate_bwd(xt, to_device(g_xhat), accumulate_into=base)
    assert kp.check() == 0
    assert bool((dx2 == dx).all())
    for acc, plain in ((dU2, dU), (dW2, dW), (db2, db)):
        assert torch.equal(acc, plain + 0.25)
    # and the plain call is bit-reproducible
    dx3, dU3, dW3, db3 = kp.gate_bwd(xt, to_device(g_xhat))
    assert torch.equal(dU3, dU) and torch.equal(dW3, dW) and torch.equal(db3, db) and torch.equal(dx3, dx)


def test_wide_state_backward_uses_the_multi_pass_kernel():
    cfg = kv.KV_CONFIGS[1].scaled(n=70, d=2304)
    _bwd_parity(cfg, kv.kv_inputs(cfg), with_g_m=True)


@pytest.mark.parametrize("n,d", [(1, 64), (3, 64), (257, 64), (5, 1024)])
def test_smallest_streams_backward(n, d):
    cfg = kv.KV_CONFIGS[1].scaled(n=n, d=d)
    _bwd_parity(cfg, kv.kv_inputs(cfg), with_g_m=True)


def test_backward_argument_errors_come_before_any_launch():
    import torch
    import paper_2603_04411_amd as L
    cfg = kv.KV_CONFIGS[0]
    kp = KvProblem(cfg, kv.kv_inputs(cfg))
    xt, _, _, _ = kp.gate(cfg.tau, soft=False)
    g = torch.zeros_like(xt)
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    dx = torch.full_like(xt, 7.0)
    dU = torch.full((cfg.d, cfg.d), 7.0, device="cuda")
    dW, db = dU.clone(), torch.full((cfg.d,), 7.0, device="cuda")
    with pytest.raises(L.LmheadError):
        L.dynakv_gate_bwd(kp.desc, kp.x, kp.U, kp.W, kp.b, xt, g, None, 0.0, dx, dU, dW, db, small)
    ws = torch.empty(L.dynakv_bwd_workspace_bytes(kp.desc), dtype=torch.uint8, device="cuda")
    with pytest.raises(L.LmheadError):
        L.dynakv_gate_bwd(kp.desc, kp.x, kp.U, kp.W, kp.b, xt, None, None, 0.0, dx, dU, dW, db, ws)
    torch.cuda.synchronize()
    assert bool((dx == 7).all()) and bool((dU == 7).all()) and bool((db == 7).all())


def test_full_size_stream_backward_sampled_against_the_oracle():
    """The benchmark stream (262144 x 1024, bf16) in the launch configuration the benchmark times.
    (1) Upstream gradients that are non-zero on a seeded sample of tokens only: every output is then a
    function of the sample alone, which the oracle evaluates exactly (the contractions still run over
    all tokens).  (2) Dense upstream gradients: dx on sampled rows (tokens are independent) and the
    zero-sum property of the softmax Jacobian for db and dW."""
    import torch
    cfg = kv.KV_CONFIGS[2]
    inp = kv.kv_inputs(cfg)
    n, d = cfg.n, cfg.d
    rows = np.unique(np.concatenate([np.arange(0, 200), np.random.default_rng(11).integers(0, n, 800), [n - 1]]))
    kp = KvProblem(cfg, inp)
    xt, _, _, _ = kp.gate(cfg.tau, soft=False)
    g_xhat, _ = kv.upstream(cfg, rows=rows)
    dx, dU, dW, db = kp.gate_bwd(xt, to_device(g_xhat), None, 0.0)
    assert kp.check() == 0
    sub = {key: (inp[key][rows] if key == "x" else inp[key]) for key in inp}
    o = _oracle_bwd(cfg.scaled(n=rows.size), sub, g_xhat[rows], None, 0.0, "suffix")
    idx = torch.from_numpy(rows).cuda()
    assert rel_fro(np64(dx[idx]), o["dx"]) <= 1e-2
    other = torch.ones(n, dtype=torch.bool, device="cuda")
    other[idx] = False
    assert bool((dx[other] == 0).all())
    for name, got in (("dU", dU), ("dW", dW), ("db", db)):
        assert rel_fro(np64(got), o[name]) <= 1e-2, name
    del dx, dU, dW, db
    # dense upstream gradients, with the constant of the regulariser on the mask
    g_xhat, _ = kv.upstream(cfg)
    c = 2 * 0.5 * 0.44 / (n * d)
    dx, dU, dW, db = kp.gate_bwd(xt, to_device(g_xhat), None, c)
    assert kp.check() == 0
    o = _oracle_bwd(cfg.scaled(n=rows.size), sub, g_xhat[rows], None, c, "suffix")
    assert rel_fro(np64(dx[idx]), o["dx"]) <= 1e-2
    dbh, dWh = np64(db), np64(dW)
    assert abs(dbh.sum()) <= 1e-3 * np.abs(dbh).sum()
    assert np.abs(dWh.sum(1)).max() <= 1e-3 * np.abs(dWh).sum(1).max()
    assert np.isfinite(np64(dU)).all() and np.isfinite(dWh).all()
