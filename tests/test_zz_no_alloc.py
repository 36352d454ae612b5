"""grpo_loss_noalloc (block partials in the library's static device array) against grpo_loss (caller's
workspace) through the C ABI: the same kernels run, so every output must be bit-identical.  Two calls in
a row, the second on a smaller input, so that the first call's leftovers in the shared array are there to
be (wrongly) picked up; then the size limit and an oracle check of the result itself."""
import ctypes as C

import numpy as np
import pytest

import workloads as wl
from oracle import lmhead_oracle as O
from tests.harness import np64, rel_fro, to_device

pytestmark = pytest.mark.gpu


def _both(cfg, agg):
    import torch
    import paper_2603_04411_amd as L
    lens = wl.lengths(cfg)
    lp, lo, lr = wl.synthetic_logprobs(cfg)
    adv = O.group_advantage(wl.rewards(cfg), cfg.P, cfg.G, 1e-6, 0).astype(np.float32)
    d = [to_device(a) for a in (lp, lo, lr, adv)] + [to_device(np.ascontiguousarray(lens, dtype=np.int32))]
    ws = torch.empty(L.loss_workspace_bytes(cfg.P, cfg.G, cfg.T), dtype=torch.uint8, device="cuda")
    outs = []
    for use_static in (False, True):
        loss = torch.full((1,), 7.0, dtype=torch.float32, device="cuda")
        g = torch.full((cfg.N,), 5.0, dtype=torch.float32, device="cuda")
        stats = torch.full((4,), 9.0, dtype=torch.float32, device="cuda")
        args = (d[0], d[1], d[2], d[3], d[4], cfg.P, cfg.G, cfg.T, 0.2, 0.28, 0.04, agg, loss, g, stats)
        if use_static:
            L.grpo_loss_noalloc(*args)
        else:
            L.grpo_loss(*args, ws)
        torch.cuda.synchronize()
        outs.append((loss, g, stats))
    (l0, g0, s0), (l1, g1, s1) = outs
    assert torch.equal(l0, l1) and torch.equal(g0, g1) and torch.equal(s0, s1)
    o_loss, o_g, o_stats = O.grpo_loss(lp, lo, lr, adv, lens, cfg.P, cfg.G, cfg.T, 0.2, 0.28, 0.04, agg)
    scale = max(abs(o_loss), O.grpo_abs_scale(lp, lo, lr, adv, lens, cfg.P, cfg.G, cfg.T, 0.2, 0.28, 0.04, agg))
    assert abs(float(l1.item()) - o_loss) <= 1e-3 * scale
    assert rel_fro(np64(g1), o_g) <= 1e-3 and float(s1[3].item()) == o_stats[3]


def test_static_scratch_variant_matches_workspace_variant_twice_in_a_row():
    big = wl.CONFIGS[1].scaled(P=6, G=8, T=5000, d=64, V=512)      # 48 responses x 3 blocks of partials
    small = wl.CONFIGS[1].scaled(P=2, G=3, T=300, d=64, V=512)     # 6 x 1: a prefix of the array just used
    _both(big, 0)
    _both(small, 0)
    _both(small, 1)


def test_static_scratch_size_limit_and_argument_errors():
    import paper_2603_04411_amd as L
    lib = L.load_library()
    p = 0x10000   # never dereferenced: these calls fail in host-side validation
    f = lib.grpo_loss_noalloc
    # 65535 responses x 2 blocks > 65536 partial blocks
    assert f(p, p, None, p, p, 65535, 1, 4096, 0.2, 0.2, 0.04, 0, p, p, None, None) == -5
    assert f(p, p, None, p, p, 2, 4, 32, 0.2, 0.2, 0.04, 0, None, p, None, None) == -1
    assert f(p, p, None, p, p, 2, 4, 32, 0.2, 0.2, 0.04, 2, p, p, None, None) == -2
    assert f(p, p, None, p, p, 0, 4, 32, 0.2, 0.2, 0.04, 0, p, p, None, None) == -2
