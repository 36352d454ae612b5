"""GPU parity of the KV-compression path (include/dynakv.h) against the fp64 oracle on the same seeded
inputs, through the C ABI.

Tolerances.  Integer and byte work (segment offsets, the packed layout, zero fill) is compared
bit-exactly on inputs the oracle also sees.  The spectral state is rounded to the storage type from
an fp32 accumulator here and from fp64 in the oracle, so single elements may land on the neighbouring
bf16 value (|d| <= one unit in the last place); such a flip moves that token's gate logits by up to
~1e-2 and its mask by a few 1e-3.  Hence: x~ within one ulp of the storage type (plus the fp32
accumulation error, 1e-6 of the largest entry) and, for bf16, equal on > 99 % of the elements; |dm| <= 5e-3 (bf16) / 1e-4 (fp32); the retained count k must be a valid threshold
crossing of the oracle's mask under that tolerance everywhere, and equal to the oracle's wherever
the oracle's mask clears tau by more than the tolerance; reconstruction within 1e-2 relative
Frobenius error (the bound used for the other matrix outputs of this library).
"""
import numpy as np
import pytest

import workloads as wl
import workloads.dynakv as kv
from oracle import dynakv_oracle as O
from tests.harness import KvProblem, np64, rel_fro, to_device

pytestmark = pytest.mark.gpu


def _tols(cfg):
    return (2.0 ** -7, 5e-3) if cfg.dtype == "bf16" else (2.0 ** -22, 1e-4)


def _oracle_chain(cfg, inp, tau, order="suffix"):
    f = wl.as_f64
    g = O.gate(f(inp["x"]), f(inp["U"]), f(inp["W"]), inp["b"], tau, order=order, store_dtype=cfg.dtype)
    off, packed = O.store(g["xt"], g["k"])
    g["off"], g["packed"] = off, packed
    g["xbar"] = O.reconstruct(packed, off, g["k"], f(inp["U_inv"]), store_dtype=cfg.dtype)
    return g


def _check_k(k_gpu, o, tau, tol, d):
    """k_gpu is a valid crossing of the oracle's mask, and the oracle's own wherever that is unambiguous."""
    m = o["m"]
    n = m.shape[0]
    rows = np.arange(n)
    assert np.all((k_gpu >= 1) & (k_gpu <= d))
    last_kept = m[rows, k_gpu - 1]
    first_cut = np.where(k_gpu < d, m[rows, np.minimum(k_gpu, d - 1)], -1.0)
    assert np.all(last_kept > tau - tol) and np.all(first_cut <= tau + tol)
    ko = o["k"].astype(np.int64)
    margin = np.minimum(m[rows, ko - 1] - tau, np.where(ko < d, tau - m[rows, np.minimum(ko, d - 1)], 1.0))
    clear = margin > tol
    assert np.array_equal(k_gpu[clear], ko[clear])
    return float(np.mean(k_gpu == ko)), float(np.mean(clear))


def _gate_parity(cfg, inp, tau, flags=0, order="suffix", ldx=None):
    ulp, tol_m = _tols(cfg)
    o = _oracle_chain(cfg, inp, tau, order)
    kp = KvProblem(cfg, inp, flags=flags, ldx=ldx)
    xt, k, m, xhat = kp.gate(tau)
    assert kp.check() == 0
    g_xt, g_m, g_xhat = np64(xt), np64(m), np64(xhat)
    acc = 1e-6 * np.abs(o["xt"]).max()          # fp32 accumulation error scales with the row, not the element
    assert np.all(np.abs(g_xt - o["xt"]) <= ulp * np.abs(o["xt"]) + acc)
    if cfg.dtype == "bf16":
        assert np.mean(g_xt == o["xt"]) > 0.99
    assert np.abs(g_m - o["m"]).max() <= tol_m
    assert np.all(np.diff(g_m, axis=1) <= 1e-6) and np.abs(g_m[:, 0] - 1).max() <= 1e-5
    assert np.all(np.abs(g_xhat - o["xhat"]) <= ulp * np.abs(o["xhat"]) + tol_m * np.abs(o["xt"]) + acc)
    k_gpu = k.cpu().numpy().astype(np.int64)
    same, clear = _check_k(k_gpu, o, tau, tol_m, cfg.d)
    # without the training outputs the same counts come back
    xt2, k2, _, _ = kp.gate(tau, soft=False)
    assert np.array_equal(k2.cpu().numpy(), k.cpu().numpy()) and bool((xt2 == xt).all())
    return kp, o, (xt, k, m, xhat), same, clear


def test_tiny_fp32_chain_end_to_end():
    cfg = kv.KV_CONFIGS[0]
    inp = kv.kv_inputs(cfg)
    kp, o, (xt, k, m, xhat), same, clear = _gate_parity(cfg, inp, cfg.tau)
    assert same > 0.99 and clear > 0.95
    off, packed = kp.store(xt, k)
    total = int(off[-1].item())
    xbar = kp.reconstruct(packed, total, off, k)
    assert kp.check() == 0
    assert rel_fro(np64(xbar), o["xbar"]) <= 1e-4
    out, g = kp.retain(k, m, 0.5)
    pen, Rs, grad = O.retain_penalty(o["m"], 0.5)
    got = np64(out)
    assert abs(got[0] - O.retain_rate_hard(o["k"], cfg.d)) <= 2e-3       # a few counts may differ by one
    assert abs(got[1] - Rs) <= 1e-5 and abs(got[2] - pen) <= 1e-5
    assert np.abs(np64(g) - grad).max() <= 1e-6 * np.abs(grad).max()


@pytest.mark.parametrize("literal", [False, True])
def test_small_bf16_gate_both_mask_orders(literal):
    cfg = kv.KV_CONFIGS[1]
    inp = kv.kv_inputs(cfg)
    flags = 1 if literal else 0
    kp, o, outs, same, clear = _gate_parity(cfg, inp, cfg.tau, flags=flags, order="literal" if literal else "suffix")
    assert same > 0.9
    if literal:
        # the two readings differ: the printed formula keeps the complement count on a one-hot gate
        o2 = _oracle_chain(cfg, inp, cfg.tau, "suffix")
        assert np.mean(o2["k"] == o["k"]) < 0.5


def test_small_bf16_chain_end_to_end_with_strided_input():
    cfg = kv.KV_CONFIGS[1].scaled(n=777, d=320)       # d with a ragged last tile and last position group
    inp = kv.kv_inputs(cfg)
    kp, o, (xt, k, m, xhat), same, clear = _gate_parity(cfg, inp, cfg.tau, ldx=cfg.d + 24)
    off, packed = kp.store(xt, k)
    xbar = kp.reconstruct(packed, int(off[-1].item()), off, k)
    assert kp.check() == 0
    assert rel_fro(np64(xbar), o["xbar"]) <= 1e-2
    out, _ = kp.retain(k, m, 0.3, want_grad=False)
    assert abs(np64(out)[0] - O.retain_rate_hard(o["k"], cfg.d)) <= 2e-3
    assert abs(np64(out)[1] - O.retain_rate_soft(o["m"])) <= 1e-3


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_store_and_reconstruct_from_oracle_inputs_are_exact(dtype):
    """The store is byte work: fed with the oracle's own (rounded) x~ and k it must reproduce the oracle's
    offsets and packed array bit for bit, including counts 0 and d; the reconstruction of that store
    matches the oracle's to rounding."""
    cfg = kv.KV_CONFIGS[1].scaled(n=613, d=256, dtype=dtype)
    inp = kv.kv_inputs(cfg)
    o = _oracle_chain(cfg, inp, cfg.tau)
    k = o["k"].copy()
    k[[0, 5, 612]] = 0
    k[[1, 300]] = cfg.d
    k[2], k[3], k[4] = 1, 8, 9
    off, packed = O.store(o["xt"], k)
    xbar = O.reconstruct(packed, off, k, wl.as_f64(inp["U_inv"]), store_dtype=dtype)
    kp = KvProblem(cfg, inp)
    as_store = (lambda a: wl.bf16_bits_from_f32(a.astype(np.float32))) if dtype == "bf16" else (lambda a: a.astype(np.float32))
    d_xt, d_k = to_device(as_store(o["xt"])), to_device(k.astype(np.int32))
    g_off, g_packed = kp.store(d_xt, d_k)
    assert kp.check() == 0
    assert np.array_equal(g_off.cpu().numpy(), off)
    assert np.array_equal(np64(g_packed)[: off[-1]], packed)
    assert bool((g_packed[off[-1]:] == 5.0).all())                  # nothing written past the end
    g_xbar = kp.reconstruct(g_packed, int(off[-1]), g_off, d_k)
    assert kp.check() == 0
    got = np64(g_xbar)
    assert np.all(got[k == 0] == 0)
    assert rel_fro(got, xbar) <= (2e-3 if dtype == "bf16" else 1e-5)
    # segments laid out in reverse token order: offsets need not increase with the token index
    seg = np.diff(off)
    rev_off = np.zeros(cfg.n + 1, dtype=np.int64)
    rev_packed = np.zeros(int(off[-1]), dtype=np.float64)
    pos = 0
    for i in range(cfg.n - 1, -1, -1):
        rev_off[i] = pos
        rev_packed[pos: pos + seg[i]] = packed[off[i]: off[i + 1]]
        pos += seg[i]
    rev_off[cfg.n] = pos
    g_xbar2 = kp.reconstruct(to_device(as_store(rev_packed)), pos, to_device(rev_off), d_k)
    assert kp.check() == 0 and bool((g_xbar2 == g_xbar).all())


def test_nothing_pruned_round_trip_and_everything_pruned():
    cfg = kv.KV_CONFIGS[0].scaled(n=130, d=64)
    inp = kv.kv_inputs(cfg)
    kp = KvProblem(cfg, inp)
    xt, k, m, _ = kp.gate(0.0)                                      # tau = 0 keeps every component
    assert bool((k == cfg.d).all())
    off, packed = kp.store(xt, k)
    xbar = kp.reconstruct(packed, int(off[-1].item()), off, k)
    # U_inv is the inverse of U up to fp32 rounding, so the round trip returns x
    assert rel_fro(np64(xbar), wl.as_f64(inp["x"])) <= 1e-4
    xt, k, m, _ = kp.gate(1.001)                                    # no mask value exceeds 1 (up to rounding)
    assert bool((k == 0).all())
    off, packed = kp.store(xt, k)
    assert bool((off == 0).all()) and kp.check() == 0
    xbar = kp.reconstruct(packed, 0, off, k)                        # an empty store reconstructs to zeros
    assert kp.check() == 0 and bool((xbar == 0).all())


def test_device_side_errors_are_reported():
    import torch
    cfg = kv.KV_CONFIGS[0].scaled(n=40, d=64)
    inp = kv.kv_inputs(cfg)
    kp = KvProblem(cfg, inp)
    xt, k, _, _ = kp.gate(cfg.tau, soft=False)
    off, packed = kp.store(xt, k)
    assert kp.check() == 0
    total = int(off[-1].item())
    off2, packed2 = kp.store(xt, k, capacity=total - 8)             # the last segment does not fit
    assert kp.check() == -6
    assert bool((off2 == off).all())
    bad_k = k.clone()
    bad_k[3] = cfg.d + 1
    kp.store(xt, bad_k)
    assert kp.check() == -6
    kp.reconstruct(packed, total - 8, off, k)                       # offsets point past the readable part
    assert kp.check() == -6
    kp.reconstruct(packed, total, off, k)
    assert kp.check() == 0


def test_full_size_stream_sampled_against_the_oracle():
    """One layer's key stream at benchmark size (262144 tokens, d_kv = 1024), in the launch
    configuration the benchmark times: a seeded sample of tokens is checked against the oracle row by
    row, and the whole result against properties that hold at any size."""
    import torch
    cfg = kv.KV_CONFIGS[2]
    inp = kv.kv_inputs(cfg)
    kp = KvProblem(cfg, inp)
    xt, k, _, _ = kp.gate(cfg.tau, soft=False)
    off, packed = kp.store(xt, k)
    total = int(off[-1].item())
    xbar = kp.reconstruct(packed, total, off, k)
    assert kp.check() == 0
    n, d = cfg.n, cfg.d
    k_h, off_h = k.cpu().numpy().astype(np.int64), off.cpu().numpy()
    # integer structure of the whole store
    assert k_h.min() >= 1 and k_h.max() <= d
    seg = (k_h + 7) // 8 * 8
    assert off_h[0] == 0 and np.array_equal(np.diff(off_h), seg) and total == seg.sum()
    rows = np.unique(np.concatenate([np.arange(0, 300), np.random.default_rng(7).integers(0, n, 700), [n - 1]]))
    # packed segments are the leading components of the spectral state, zero padded
    xt_h = np64(xt[torch.from_numpy(rows).cuda()])
    for r, i in enumerate(rows):
        segv = np64(packed[off_h[i]: off_h[i + 1]])
        assert np.array_equal(segv[: k_h[i]], xt_h[r, : k_h[i]]) and np.all(segv[k_h[i]:] == 0)
    # sampled tokens against the oracle (every token is independent of the others)
    sub = {key: (inp[key][rows] if key == "x" else inp[key]) for key in inp}
    o = _oracle_chain(cfg.scaled(n=rows.size), sub, cfg.tau)
    ulp, tol_m = _tols(cfg)
    assert np.all(np.abs(xt_h - o["xt"]) <= ulp * np.abs(o["xt"]) + 1e-6 * np.abs(o["xt"]).max())
    same, clear = _check_k(k_h[rows], o, cfg.tau, tol_m, d)
    assert same > 0.9
    got = np64(xbar[torch.from_numpy(rows).cuda()])
    assert rel_fro(got, o["xbar"]) <= 1e-2
    # the reconstruction error of every token is the energy it discarded, up to rounding: U is close to
    # orthogonal here, so ||x - x_bar||^2 ~ sum_{j >= k} x~_j^2 (checked in aggregate over the sample)
    x_s = wl.as_f64(inp["x"][rows])
    tail = np.array([(o["xt"][r, k_h[i]:] ** 2).sum() for r, i in enumerate(rows)])
    err = ((x_s - got) ** 2).sum(1)
    assert abs(err.sum() - tail.sum()) <= 0.1 * tail.sum() + 1e-3 * (x_s ** 2).sum()


def test_wide_state_uses_the_multi_pass_mask_kernel():
    # d_kv beyond 2048 takes the mask kernel's generic (three-pass) path; 9 tiles along d
    cfg = kv.KV_CONFIGS[1].scaled(n=70, d=2304)
    inp = kv.kv_inputs(cfg)
    kp, o, (xt, k, m, xhat), same, clear = _gate_parity(cfg, inp, cfg.tau)
    off, packed = kp.store(xt, k)
    xbar = kp.reconstruct(packed, int(off[-1].item()), off, k)
    assert kp.check() == 0
    assert rel_fro(np64(xbar), o["xbar"]) <= 1e-2


def test_append_to_an_existing_store():
    """Decoding appends: a prefill of 500 tokens is stored, then two steps of 40 and 1 tokens are
    appended with off_base = the cache's end; offsets, packed bytes and the reconstruction of the whole
    cache must equal those of storing all 541 tokens at once."""
    import torch
    cfg = kv.KV_CONFIGS[1].scaled(n=541, d=192)
    inp = kv.kv_inputs(cfg)
    whole = KvProblem(cfg, inp)
    xt, k, _, _ = whole.gate(cfg.tau, soft=False)
    off_all, packed_all = whole.store(xt, k)
    total = int(off_all[-1].item())
    cache_off = torch.full((cfg.n + 1,), -1, dtype=torch.int64, device="cuda")
    cache = torch.full((cfg.n * cfg.d,), 5.0, dtype=whole.tdt, device="cuda")
    start, end_off = 0, 0
    for count in (500, 40, 1):
        part = KvProblem(cfg.scaled(n=count), {**inp, "x": inp["x"][start:start + count]})
        part.store(xt[start:start + count], k[start:start + count], capacity=cfg.n * cfg.d, off_base=end_off,
                   off=cache_off[start:], packed=cache)
        assert part.check() == 0
        start += count
        end_off = int(cache_off[start].item())
    assert bool((cache_off == off_all).all()) and end_off == total
    assert bool((cache[:total] == packed_all[:total]).all()) and bool((cache[total:] == 5.0).all())
    xbar = whole.reconstruct(cache, total, cache_off, k)
    ref = whole.reconstruct(packed_all, total, off_all, k)
    assert whole.check() == 0 and bool((xbar == ref).all())


@pytest.mark.parametrize("n,d", [(1, 64), (3, 64), (257, 64), (5, 1024)])
def test_smallest_streams(n, d):
    """One token, fewer tokens than a lane group, one token past a tile, the smallest d_kv."""
    cfg = kv.KV_CONFIGS[0].scaled(n=n, d=d)
    inp = kv.kv_inputs(cfg)
    kp, o, (xt, k, m, xhat), same, clear = _gate_parity(cfg, inp, cfg.tau)
    off, packed = kp.store(xt, k)
    xbar = kp.reconstruct(packed, int(off[-1].item()), off, k)
    assert kp.check() == 0
    assert rel_fro(np64(xbar), o["xbar"]) <= 1e-3
    out, _ = kp.retain(k, m, 1.0, want_grad=False)
    assert abs(np64(out)[1] - O.retain_rate_soft(o["m"])) <= 1e-5
