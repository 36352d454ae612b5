"""GPU parity at the benchmark's full sizes (configs 1-4), in the launch configuration bench.py times.

The oracle cannot evaluate N_v x V logits at these sizes, so each stage is checked on what it
can afford, always from seeded inputs (never from HIP outputs):
  (A) forward: integer indexing exactly; logp / lse / entropy on a stratified sample of rows;
  (B) loss kernels: full size, on seeded stand-ins for the log-prob arrays;
  (C) backward with a seeded upstream gradient: dH on the sampled rows; dW through the library
      run on the sampled rows as a problem of their own against the full oracle of that
      sub-problem; and the identities that tie the complete dH, dW to the forward outputs:
      sum_v dW[v,:] = 0 and <dW,W> = <dH,H> = sum_i g_i (logp_i + entropy_i).
"""
import sys

import numpy as np
import pytest

import workloads as wl
from oracle import lmhead_oracle as O
from tests.harness import GpuProblem, assert_index_parity, np64, rel_fro, to_device

pytestmark = pytest.mark.gpu

SAMPLE = 384


def say(msg):
    print(msg, file=sys.stderr, flush=True)


@pytest.mark.parametrize("ci", [1, 2, 3, 4])
def test_full_size(ci):
    import torch
    cfg = wl.CONFIGS[ci]
    say(f"[full] config {ci}: generating {cfg.name}")
    lens, tok = wl.lengths(cfg), wl.tokens(cfg)
    H_host, W_host = wl.hidden(cfg), wl.weight(cfg)
    gp = GpuProblem(cfg, H_host, W_host, tok, lens)
    T = cfg.T

    # ---- (A) forward ---------------------------------------------------------------------
    say("[full] forward")
    logp, lse, ent, mask, cu = gp.fwd()
    assert gp.check() == 0
    o_mask, o_cu, o_rs, _ = O.index_build(lens, T)
    assert np.array_equal(mask.cpu().numpy(), o_mask)
    assert np.array_equal(cu.cpu().numpy(), o_cu)
    assert_index_parity(gp, o_rs, tok)   # compaction map, compacted ids, gathered vocabulary columns: ==
    pad = torch.from_numpy(o_mask == 0).cuda()
    for t in (logp, lse, ent):
        assert torch.count_nonzero(t[pad]) == 0
    rows = wl.sample_valid_rows(cfg, lens, tok, SAMPLE)
    Hs, W64 = wl.as_f64(H_host[rows]), wl.as_f64(W_host)
    o_lp, o_lse, o_ent = O.logprob_rows(Hs, W64, tok[rows])
    ridx = torch.from_numpy(rows).cuda()
    for got, want, name in ((logp, o_lp, "logp"), (lse, o_lse, "lse"), (ent, o_ent, "entropy")):
        err = np.abs(np64(got[ridx]) - want).max()
        say(f"[full]   {name}: max abs err on {rows.size} rows {err:.2e}")
        assert err <= 1e-2

    # ---- (B) loss kernels at full size on seeded stand-in log-probs --------------------------------
    say("[full] loss kernels")
    s_lp, s_old, s_ref = wl.synthetic_logprobs(cfg)
    rewards, logZ = wl.rewards(cfg), wl.log_z(cfg)
    d_lp, d_old, d_ref = to_device(s_lp), to_device(s_old), to_device(s_ref)
    adv = gp.advantage(rewards)
    o_adv = O.group_advantage(rewards, cfg.P, cfg.G, 1e-6, 0)
    assert np.abs(np64(adv) - o_adv).max() <= 1e-4
    args = (s_lp, s_old, s_ref, o_adv, lens, cfg.P, cfg.G, T, cfg.clip_eps, cfg.clip_eps, cfg.kl_coef)
    for agg in (0, 1):
        loss, g, stats = gp.grpo(d_lp, d_old, d_ref, to_device(o_adv.astype(np.float32)), cfg.clip_eps,
                                 cfg.clip_eps, cfg.kl_coef, agg)
        o_loss, o_g, o_stats = O.grpo_loss(*args, agg)
        scale = max(abs(o_loss), O.grpo_abs_scale(*args, agg))
        assert abs(float(loss.item()) - o_loss) <= 1e-3 * scale
        if abs(o_loss) > 1e-3:   # the plain relative bound wherever the loss is not itself near zero
            assert abs(float(loss.item()) - o_loss) <= 1e-3 * abs(o_loss), (float(loss.item()), o_loss)
        assert rel_fro(np64(g), o_g) <= 1e-3 and torch.count_nonzero(g[pad]) == 0
        assert np.abs(np64(stats)[:3] - o_stats[:3]).max() <= 1e-3 and float(stats[3].item()) == o_stats[3]
    loss, g, gz, resid = gp.flowrl(d_lp, d_ref, rewards, logZ, cfg.beta)
    o_loss, o_g, o_gz, o_resid = O.flowrl_tb_loss(s_lp, s_ref, rewards, logZ, lens, cfg.P, cfg.G, T, cfg.beta)
    assert abs(float(loss.item()) - o_loss) <= 1e-3 * abs(o_loss)
    assert rel_fro(np64(g), o_g) <= 1e-3 and rel_fro(np64(gz), o_gz) <= 1e-3
    assert np.abs(np64(resid) - o_resid).max() <= 1e-3 * max(1.0, np.abs(o_resid).max())

    # ---- (C) backward with a seeded upstream gradient ---------------------------------------------------
    say("[full] backward")
    g_host = wl.synthetic_upstream_grad(cfg, lens)
    g_dev = to_device(g_host)
    dH, dW = gp.bwd(lse, g_dev)
    assert gp.check() == 0
    o_dH_rows, _ = O.bwd_rows(Hs, W64, tok[rows], g_host[rows].astype(np.float64))
    e_h = rel_fro(np64(dH[ridx]), o_dH_rows)
    say(f"[full]   dH on sampled rows: rel Frobenius err {e_h:.2e}")
    assert e_h <= 1e-2
    # padded rows exactly zero (checked on a sample of padded slots to bound the host copy)
    pad_idx = np.nonzero(o_mask == 0)[0]
    if pad_idx.size:
        sel = torch.from_numpy(pad_idx[:: max(1, pad_idx.size // 4096)]).cuda()
        assert torch.count_nonzero(dH[sel]) == 0
    # identities over the complete gradients (device-side reductions in fp64)
    colsum = dW.double().sum(dim=0)
    dw_scale = dW.double().abs().sum(dim=0)
    assert float((colsum.abs() / (dw_scale + 1e-30)).max()) <= 1e-3, "sum_v dW[v,:] must vanish"
    rhs = float((g_dev.double() * (logp.double() + ent.double())).sum())
    Wd = gp.W
    lhs_w = 0.0
    for v0 in range(0, cfg.V, 16384):
        lhs_w += float((dW[v0:v0 + 16384].double() * Wd[v0:v0 + 16384].double()).sum())
    lhs_h = 0.0
    for n0 in range(0, cfg.N, 32768):
        lhs_h += float((dH[n0:n0 + 32768].double() * gp.H[n0:n0 + 32768].double()).sum())
    scale = float((g_dev.double().abs() * (logp.double() + ent.double()).abs()).sum())
    say(f"[full]   <dW,W> {lhs_w:.6e}  <dH,H> {lhs_h:.6e}  sum g(logp+ent) {rhs:.6e}  (scale {scale:.3e})")
    assert abs(lhs_w - rhs) <= 1e-2 * scale and abs(lhs_h - rhs) <= 1e-2 * scale
    del dH, dW, gp
    torch.cuda.empty_cache()

    # dW against the oracle on the sampled rows run as their own problem (all rows valid)
    say("[full] dW on the sampled sub-problem")
    sub = cfg.scaled(P=1, G=1, T=int(rows.size), len_lo=int(rows.size), len_hi=int(rows.size))
    sub_lens = np.array([rows.size], dtype=np.int32)
    gs = GpuProblem(sub, H_host[rows], W_host, tok[rows], sub_lens)
    s_logp, s_lse, *_ = gs.fwd()
    g_sub = g_host[rows]
    s_dH, s_dW = gs.bwd(s_lse, to_device(g_sub))
    _, o_dW = O.bwd_rows(Hs, W64, tok[rows], g_sub.astype(np.float64))
    e_w = rel_fro(np64(s_dW), o_dW)
    e_h2 = rel_fro(np64(s_dH), o_dH_rows)
    say(f"[full]   sub-problem: dW rel err {e_w:.2e}, dH rel err {e_h2:.2e}")
    assert e_w <= 1e-2 and e_h2 <= 1e-2


def test_full_size_fp8_logits_variant():
    """configs[2] with the logits kernels on e4m3 copies: sampled rows against the oracle evaluated on the
    same rounded copies, and the identities that still tie the complete dH and dW together."""
    import torch
    cfg = wl.CONFIGS[2]
    lens, tok = wl.lengths(cfg), wl.tokens(cfg)
    H_host, W_host = wl.hidden(cfg), wl.weight(cfg)
    eh = int(np.floor(np.log2(448.0 / np.abs(wl.as_f64(H_host[:65536])).max()))) - 1
    ew = int(np.floor(np.log2(448.0 / np.abs(wl.as_f64(W_host[:65536])).max()))) - 1
    gp = GpuProblem(cfg, H_host, W_host, tok, lens, flags=4, fp8_exp_h=eh, fp8_exp_w=ew)
    logp, lse, ent, _, _ = gp.fwd()
    assert gp.check() == 0
    rows = wl.sample_valid_rows(cfg, lens, tok, SAMPLE)
    Hs, W64 = wl.as_f64(H_host[rows]), wl.as_f64(W_host)
    Hq, Wq = O.quantize_e4m3(Hs, eh), O.quantize_e4m3(W64, ew)
    assert np.abs(Hq).max() * 2.0 ** eh <= 448 and np.abs(Wq).max() * 2.0 ** ew <= 448
    o_lp, o_lse, o_ent = O.logprob_rows(Hq, Wq, tok[rows])
    ridx = torch.from_numpy(rows).cuda()
    for got, want, name in ((logp, o_lp, "logp"), (lse, o_lse, "lse"), (ent, o_ent, "entropy")):
        err = np.abs(np64(got[ridx]) - want).max()
        say(f"[full fp8]   {name}: max abs err on {rows.size} rows {err:.2e}")
        assert err <= 1e-2
    g_host = wl.synthetic_upstream_grad(cfg, lens)
    dH, dW = gp.bwd(lse, to_device(g_host))
    assert gp.check() == 0
    o_dH_rows, _ = O.bwd_rows(Hs, W64, tok[rows], g_host[rows].astype(np.float64), Hq, Wq)
    e_h = rel_fro(np64(dH[ridx]), o_dH_rows)
    say(f"[full fp8]   dH on sampled rows: rel Frobenius err {e_h:.2e}")
    assert e_h <= 1e-2
    colsum = dW.double().sum(dim=0)
    dw_scale = dW.double().abs().sum(dim=0)
    assert float((colsum.abs() / (dw_scale + 1e-30)).max()) <= 1e-3
    lhs_w = sum(float((dW[v0:v0 + 16384].double() * gp.W[v0:v0 + 16384].double()).sum()) for v0 in range(0, cfg.V, 16384))
    lhs_h = sum(float((dH[n0:n0 + 32768].double() * gp.H[n0:n0 + 32768].double()).sum()) for n0 in range(0, cfg.N, 32768))
    scale = float((dH.double().abs() * gp.H.double().abs()).sum())
    say(f"[full fp8]   <dW,W> {lhs_w:.6e}  <dH,H> {lhs_h:.6e}  (scale {scale:.3e})")
    assert abs(lhs_w - lhs_h) <= 1e-3 * scale
