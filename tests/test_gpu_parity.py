"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the same seeded inputs.

Tolerances are the benchmark's: integers bit-exact; |dlogp| <= 1e-2; loss relative
error <= 1e-3 (relative to max(|L|, sum w|l|) when L is near zero); relative
Frobenius error of dH and dW <= 1e-2.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import lmhead_oracle as O
from tests.harness import GpuProblem, assert_index_parity, np64, rel_fro, small_inputs, to_device, widen_rows

pytestmark = pytest.mark.gpu

TOL_LOGP = 1e-2
TOL_LOSS = 1e-3
TOL_GRAD = 1e-2


def _fwd_parity(cfg, inp, W_key="W", vocab_chunk=0, ldH=None, ldW=None):
    gp = GpuProblem(cfg, inp["H"], inp[W_key], inp["tok"], inp["lens"], vocab_chunk=vocab_chunk, ldH=ldH, ldW=ldW)
    logp, lse, ent, mask, cu = gp.fwd()
    assert gp.check() == 0
    o_mask, o_cu, o_rs, _ = O.index_build(inp["lens"], cfg.T)
    assert np.array_equal(mask.cpu().numpy(), o_mask)
    assert np.array_equal(cu.cpu().numpy(), o_cu)
    assert_index_parity(gp, o_rs, inp["tok"])
    o_lp, o_lse, o_ent = O.lmhead_logprob_fwd(wl.as_f64(inp["H"]), wl.as_f64(inp[W_key]), inp["tok"], inp["lens"], cfg.T)
    for got, want, name in ((logp, o_lp, "logp"), (lse, o_lse, "lse"), (ent, o_ent, "entropy")):
        g = np64(got)
        assert np.all(g[o_mask == 0] == 0), f"{name}: padded slots must be exactly 0"
        err = np.abs(g - want).max()
        assert err <= TOL_LOGP, f"{name}: max abs err {err}"
    return gp, (logp, lse, ent), (o_lp, o_lse, o_ent)


def _grpo_chain(cfg, inp, vocab_chunk=0, W_old_key="W_old", ldH=None, ldW=None):
    """fwd(theta, old, ref) -> advantages -> GRPO loss -> bwd, on GPU and in the oracle."""
    gp, (logp, lse, ent), (o_lp, o_lse, o_ent) = _fwd_parity(cfg, inp, vocab_chunk=vocab_chunk, ldH=ldH, ldW=ldW)
    lp_old, *_ = gp.fwd(W=to_device(widen_rows(inp[W_old_key], ldW)), want_entropy=False, want_index=False)
    lp_ref, *_ = gp.fwd(W=to_device(widen_rows(inp["W_ref"], ldW)), want_entropy=False, want_index=False)
    adv = gp.advantage(inp["rewards"])
    loss, g, stats = gp.grpo(logp, lp_old, lp_ref, adv, cfg.clip_eps, cfg.clip_eps, cfg.kl_coef, 0)
    dH, dW = gp.bwd(lse, g)
    assert gp.check() == 0

    H64, T = wl.as_f64(inp["H"]), cfg.T
    o_old, _, _ = O.lmhead_logprob_fwd(H64, wl.as_f64(inp[W_old_key]), inp["tok"], inp["lens"], T)
    o_ref, _, _ = O.lmhead_logprob_fwd(H64, wl.as_f64(inp["W_ref"]), inp["tok"], inp["lens"], T)
    o_adv = O.group_advantage(inp["rewards"], cfg.P, cfg.G, 1e-6, 0)
    args = (o_lp, o_old, o_ref, o_adv, inp["lens"], cfg.P, cfg.G, T, cfg.clip_eps, cfg.clip_eps, cfg.kl_coef, 0)
    o_loss, o_g, o_stats = O.grpo_loss(*args)
    scale = max(abs(o_loss), O.grpo_abs_scale(*args))
    o_dH, o_dW = O.lmhead_logprob_bwd(H64, wl.as_f64(inp["W"]), inp["tok"], inp["lens"], T, o_g)

    assert np.abs(np64(adv) - o_adv).max() <= 1e-4
    assert abs(float(loss.item()) - o_loss) <= TOL_LOSS * scale, (float(loss.item()), o_loss, scale)
    if abs(o_loss) > 1e-3:   # the plain relative bound wherever the loss is not itself near zero
        assert abs(float(loss.item()) - o_loss) <= TOL_LOSS * abs(o_loss), (float(loss.item()), o_loss)
    mask = O.index_build(inp["lens"], T)[0]
    gh = np64(dH)
    assert np.all(gh[mask == 0] == 0), "padded rows of dH must be exactly 0"
    e_h, e_w = rel_fro(gh, o_dH), rel_fro(np64(dW), o_dW)
    assert e_h <= TOL_GRAD and e_w <= TOL_GRAD, (e_h, e_w)
    return dict(err_dH=e_h, err_dW=e_w, stats=np64(stats), o_stats=o_stats)


def test_config0_fp32_grpo_end_to_end():
    cfg = wl.CONFIGS[0]
    r = _grpo_chain(cfg, small_inputs(cfg))
    assert r["err_dH"] < 1e-4 and r["err_dW"] < 1e-4     # fp32 path: far inside the bf16 tolerances
    assert abs(r["stats"][3] - r["o_stats"][3]) == 0     # N_v
    assert np.abs(r["stats"][:3] - r["o_stats"][:3]).max() < 1e-3


def test_config0_fp32_flowrl():
    cfg = wl.CONFIGS[0]
    inp = small_inputs(cfg)
    gp, (logp, lse, ent), (o_lp, o_lse, o_ent) = _fwd_parity(cfg, inp)
    lp_ref, *_ = gp.fwd(W=to_device(inp["W_ref"]), want_entropy=False, want_index=False)
    o_ref, _, _ = O.lmhead_logprob_fwd(wl.as_f64(inp["H"]), wl.as_f64(inp["W_ref"]), inp["tok"], inp["lens"], cfg.T)
    loss, g, gz, resid = gp.flowrl(logp, lp_ref, inp["rewards"], inp["logZ"], 1.0)
    o_loss, o_g, o_gz, o_resid = O.flowrl_tb_loss(o_lp, o_ref, inp["rewards"], inp["logZ"], inp["lens"],
                                                  cfg.P, cfg.G, cfg.T, 1.0)
    assert abs(float(loss.item()) - o_loss) <= TOL_LOSS * abs(o_loss)
    assert np.abs(np64(resid) - o_resid).max() <= 1e-3
    assert rel_fro(np64(gz), o_gz) <= 1e-3 and rel_fro(np64(g), o_g) <= 1e-3
    dH, dW = gp.bwd(lse, g)
    o_dH, o_dW = O.lmhead_logprob_bwd(wl.as_f64(inp["H"]), wl.as_f64(inp["W"]), inp["tok"], inp["lens"], cfg.T, o_g)
    assert rel_fro(np64(dH), o_dH) <= TOL_GRAD and rel_fro(np64(dW), o_dW) <= TOL_GRAD


@pytest.mark.parametrize("vocab_chunk", [0, 2048])
def test_bf16_small_grpo_several_tiles_and_ragged_tails(vocab_chunk):
    # config 1's distributions at a size the oracle finishes in seconds: N_v spans two token tiles with a
    # ragged tail, V spans 33 vocabulary tiles with a ragged last tile and (chunk 2048) five chunks
    cfg = wl.CONFIGS[1].scaled(P=2, G=4, T=96, d=256, V=8192 + 100)
    _grpo_chain(cfg, small_inputs(cfg), vocab_chunk=vocab_chunk)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_strided_rows_of_H_and_W(dtype):
    # ldH = d + 64 and ldW = d + 8 are part of the ABI: forward (all three policies), loss and backward
    # through row-strided inputs whose gaps hold non-zero filler; dH and dW stay dense
    cfg = wl.CONFIGS[1].scaled(P=2, G=3, T=80, d=192, V=2048 + 77, dtype=dtype)
    _grpo_chain(cfg, small_inputs(cfg), vocab_chunk=1024, ldH=cfg.d + 64, ldW=cfg.d + 8)


def test_bf16_small_near_policy_unclipped_branch():
    cfg = wl.CONFIGS[1].scaled(P=2, G=4, T=64, d=128, V=3000)
    inp = small_inputs(cfg)
    inp["W_near"] = wl.perturbed_weight(cfg, inp["W"])
    r = _grpo_chain(cfg, inp, W_old_key="W_near")
    assert r["o_stats"][0] < 0.5     # most tokens are on the unclipped branch here


def test_bf16_small_flowrl_loguniform_lengths():
    cfg = wl.CONFIGS[3].scaled(P=3, G=4, T=128, d=192, V=5000, len_lo=1, len_hi=128)
    inp = small_inputs(cfg)
    gp, (logp, lse, ent), (o_lp, o_lse, o_ent) = _fwd_parity(cfg, inp)
    lp_ref, *_ = gp.fwd(W=to_device(inp["W_ref"]), want_entropy=False, want_index=False)
    o_ref, _, _ = O.lmhead_logprob_fwd(wl.as_f64(inp["H"]), wl.as_f64(inp["W_ref"]), inp["tok"], inp["lens"], cfg.T)
    loss, g, gz, resid = gp.flowrl(logp, lp_ref, inp["rewards"], inp["logZ"], cfg.beta)
    o_loss, o_g, o_gz, o_resid = O.flowrl_tb_loss(o_lp, o_ref, inp["rewards"], inp["logZ"], inp["lens"],
                                                  cfg.P, cfg.G, cfg.T, cfg.beta)
    assert abs(float(loss.item()) - o_loss) <= TOL_LOSS * abs(o_loss)
    dH, dW = gp.bwd(lse, g)
    o_dH, o_dW = O.lmhead_logprob_bwd(wl.as_f64(inp["H"]), wl.as_f64(inp["W"]), inp["tok"], inp["lens"], cfg.T, o_g)
    assert rel_fro(np64(dH), o_dH) <= TOL_GRAD and rel_fro(np64(dW), o_dW) <= TOL_GRAD


def test_edge_lengths_zero_full_and_empty_batch():
    import torch
    cfg = wl.CONFIGS[1].scaled(P=2, G=2, T=40, d=64, V=700)
    inp = small_inputs(cfg)
    for lens in ([0, 40, 1, 0], [40, 40, 40, 40], [0, 0, 0, 0]):
        inp["lens"] = np.array(lens, dtype=np.int32)
        gp, (logp, lse, ent), (o_lp, _, _) = _fwd_parity(cfg, inp)
        o_g = np.where(O.index_build(inp["lens"], cfg.T)[0] == 1, 0.01, 0.0)
        dH, dW = gp.bwd(lse, to_device(o_g.astype(np.float32)))
        o_dH, o_dW = O.lmhead_logprob_bwd(wl.as_f64(inp["H"]), wl.as_f64(inp["W"]), inp["tok"], inp["lens"], cfg.T, o_g)
        if sum(lens) == 0:
            assert torch.count_nonzero(dH) == 0 and torch.count_nonzero(dW) == 0
        else:
            assert rel_fro(np64(dH), o_dH) <= TOL_GRAD and rel_fro(np64(dW), o_dW) <= TOL_GRAD


def test_device_side_range_errors_are_reported():
    cfg = wl.CONFIGS[1].scaled(P=1, G=2, T=16, d=64, V=300)
    inp = small_inputs(cfg)
    gp = GpuProblem(cfg, inp["H"], inp["W"], inp["tok"], inp["lens"])
    gp.fwd()
    assert gp.check() == 0
    bad_tok = inp["tok"].copy()
    bad_tok[0] = cfg.V          # slot 0 is valid (every length >= 1 here)
    gp2 = GpuProblem(cfg, inp["H"], inp["W"], bad_tok, inp["lens"])
    gp2.fwd()
    assert gp2.check() == -6
    pad_tok = inp["tok"].copy()
    pad_tok[cfg.T - 1] = -5     # padded slot: ignored
    lens = inp["lens"].copy(); lens[0] = cfg.T - 1
    gp3 = GpuProblem(cfg, inp["H"], inp["W"], pad_tok, lens)
    gp3.fwd()
    assert gp3.check() == 0
    gp4 = GpuProblem(cfg, inp["H"], inp["W"], inp["tok"], np.array([cfg.T + 1, 3], dtype=np.int32))
    gp4.fwd()
    assert gp4.check() == -6


def test_accumulate_dw_flag_and_reproducibility():
    import torch
    from paper_2603_04411_amd.binding import FLAG_ACCUM_DW
    cfg = wl.CONFIGS[1].scaled(P=1, G=4, T=80, d=128, V=1500)
    inp = small_inputs(cfg)
    gp = GpuProblem(cfg, inp["H"], inp["W"], inp["tok"], inp["lens"])
    logp, lse, *_ = gp.fwd()
    g = to_device(np.where(O.index_build(inp["lens"], cfg.T)[0] == 1, -0.003, 0.0).astype(np.float32))
    dH1, dW1 = gp.bwd(lse, g)
    dH2, dW2 = gp.bwd(lse, g)
    assert torch.equal(dH1, dH2) and torch.equal(dW1, dW2)      # no float atomics: bit-reproducible
    gp_acc = GpuProblem(cfg, inp["H"], inp["W"], inp["tok"], inp["lens"], flags=FLAG_ACCUM_DW)
    base = torch.full((cfg.V, cfg.d), 0.5, dtype=torch.float32, device="cuda")
    _, dW3 = gp_acc.bwd(lse, g, dW_init=base.clone())
    assert torch.allclose(dW3, dW1 + 0.5, atol=1e-6)


def test_cross_entropy_objective_end_to_end():
    # the paper's L_CE (Eq. 9) through the same kernels: forward -> ce_loss -> backward
    cfg = wl.CONFIGS[1].scaled(P=2, G=3, T=80, d=192, V=6000 + 37)
    inp = small_inputs(cfg)
    gp, (logp, lse, ent), (o_lp, o_lse, o_ent) = _fwd_parity(cfg, inp)
    loss, g = gp.ce(logp)
    o_loss, o_g = O.ce_loss(o_lp, inp["lens"], cfg.T)
    assert abs(float(loss.item()) - o_loss) <= TOL_LOSS * abs(o_loss)
    assert rel_fro(np64(g), o_g) <= 1e-6
    dH, dW = gp.bwd(lse, g)
    o_dH, o_dW = O.lmhead_logprob_bwd(wl.as_f64(inp["H"]), wl.as_f64(inp["W"]), inp["tok"], inp["lens"], cfg.T, o_g)
    assert rel_fro(np64(dH), o_dH) <= TOL_GRAD and rel_fro(np64(dW), o_dW) <= TOL_GRAD


def test_objective_variants_asymmetric_clip_token_mean_per_response_logz():
    """The objective variants next to the two headline losses, each against the oracle on the same fp32
    log-probabilities: clip_lo != clip_hi with the global token mean, FlowRL with one logZ per response
    (a P' = R, G' = 1 call) and FlowRL on group-normalised rewards."""
    cfg = wl.CONFIGS[1].scaled(P=6, G=8, T=300, d=64, V=512)
    lens = wl.lengths(cfg)
    lp, lo, lr = wl.synthetic_logprobs(cfg)
    mask = O.index_build(lens, cfg.T)[0]
    dummy = np.zeros((8, cfg.d), dtype=np.uint16)
    gp = GpuProblem(cfg, dummy, dummy, np.zeros(cfg.N, dtype=np.int32), lens)
    d_lp, d_lo, d_lr = (to_device(a) for a in (lp, lo, lr))
    adv = gp.advantage(wl.rewards(cfg), ddof=1)
    o_adv = O.group_advantage(wl.rewards(cfg), cfg.P, cfg.G, 1e-6, 1)
    assert np.abs(np64(adv) - o_adv).max() <= 1e-4
    for clip_lo, clip_hi, kl, agg in ((0.2, 0.28, 0.04, 1), (0.1, 0.4, 0.0, 0), (0.3, 0.2, 0.1, 1)):
        loss, g, stats = gp.grpo(d_lp, d_lo, d_lr, adv, clip_lo, clip_hi, kl, agg)
        args = (np64(d_lp), np64(d_lo), np64(d_lr), o_adv, lens, cfg.P, cfg.G, cfg.T, clip_lo, clip_hi, kl, agg)
        o_loss, o_g, o_stats = O.grpo_loss(*args)
        scale = max(abs(o_loss), O.grpo_abs_scale(*args))
        assert abs(float(loss.item()) - o_loss) <= TOL_LOSS * scale
        assert np.all(np64(g)[mask == 0] == 0) and rel_fro(np64(g), o_g) <= 1e-3

    # one logZ per response: the same entry point with P' = R, G' = 1
    per = cfg.scaled(P=cfg.R, G=1)
    gpr = GpuProblem(per, dummy, dummy, np.zeros(cfg.N, dtype=np.int32), lens)
    rng = np.random.default_rng(5)
    logz_r = rng.standard_normal(cfg.R).astype(np.float32)
    rewards = rng.random(cfg.R).astype(np.float32)
    loss, g, gz, resid = gpr.flowrl(d_lp, d_lr, rewards, logz_r, 15.0)
    o = O.flowrl_tb_loss(np64(d_lp), np64(d_lr), rewards, logz_r, lens, cfg.R, 1, cfg.T, 15.0)
    assert abs(float(loss.item()) - o[0]) <= TOL_LOSS * abs(o[0])
    assert rel_fro(np64(g), o[1]) <= 1e-3 and rel_fro(np64(gz), o[2]) <= 1e-3
    assert np.abs(np64(resid) - o[3]).max() <= 1e-3 * np.abs(o[3]).max()

    # rewards normalised by the caller (here: the group-relative advantages) are used as passed
    loss, g, gz, resid = gp.flowrl(d_lp, d_lr, np64(adv).astype(np.float32), wl.log_z(cfg), 1.0)
    o = O.flowrl_tb_loss(np64(d_lp), np64(d_lr), np64(adv), wl.log_z(cfg), lens, cfg.P, cfg.G, cfg.T, 1.0)
    assert abs(float(loss.item()) - o[0]) <= TOL_LOSS * abs(o[0])
    assert rel_fro(np64(g), o[1]) <= 1e-3 and rel_fro(np64(gz), o[2]) <= 1e-3


def test_multi_policy_forward_matches_separate_passes_and_the_oracle():
    """Current, old and reference policy over the same hidden states in one pass: bit-identical to three
    separate forward calls, and within tolerance of the oracle."""
    cfg = wl.CONFIGS[1].scaled(P=3, G=4, T=80, d=192, V=2 * 256 + 77)
    inp = small_inputs(cfg)
    gp = GpuProblem(cfg, inp["H"], inp["W"], inp["tok"], inp["lens"])
    Ws = [gp.W, to_device(inp["W_old"]), to_device(inp["W_ref"])]
    logps, lse, ent = gp.fwd_multi(Ws)
    # every policy's gather picked the sampled token's column
    assert_index_parity(gp, O.index_build(inp["lens"], cfg.T)[2], inp["tok"], ws=gp.ws_multi, npol=3)
    for p, key in enumerate(("W", "W_old", "W_ref")):
        lp1, lse1, ent1, _, _ = gp.fwd(W=Ws[p])
        assert bool((logps[p] == lp1).all())
        if p == 0:
            assert bool((lse == lse1).all()) and bool((ent == ent1).all())
        o_lp, o_lse, o_ent = O.lmhead_logprob_fwd(wl.as_f64(inp["H"]), wl.as_f64(inp[key]), inp["tok"], inp["lens"], cfg.T)
        assert np.abs(np64(logps[p]) - o_lp).max() <= TOL_LOGP
    two, _, _ = gp.fwd_multi(Ws[:2], want_entropy=False)
    assert bool((two[0] == logps[0]).all()) and bool((two[1] == logps[1]).all())


def _fp8_exponent(a):
    """Largest power of two that keeps max|a| * 2^e inside the e4m3 range."""
    return int(np.floor(np.log2(448.0 / np.abs(wl.as_f64(a)).max())))


@pytest.mark.parametrize("vocab_chunk", [0, 1024])
def test_fp8_logits_variant(vocab_chunk):
    """Logits from e4m3 copies of H and W (forward and the backward's recompute), dH / dW contracted with the
    bf16 operands: against the oracle evaluated on the same rounded copies."""
    cfg = wl.CONFIGS[1].scaled(P=2, G=4, T=96, d=384, V=4096 + 100)
    inp = small_inputs(cfg)
    eh, ew = _fp8_exponent(inp["H"]), _fp8_exponent(inp["W"])
    assert eh >= 5 and ew >= 10                      # H ~ N(0,1), W ~ N(0, 0.02^2)
    H64, W64 = wl.as_f64(inp["H"]), wl.as_f64(inp["W"])
    Hq, Wq = O.quantize_e4m3(H64, eh), O.quantize_e4m3(W64, ew)
    gp = GpuProblem(cfg, inp["H"], inp["W"], inp["tok"], inp["lens"], vocab_chunk=vocab_chunk, flags=4,
                    fp8_exp_h=eh, fp8_exp_w=ew)
    logp, lse, ent, _, _ = gp.fwd()
    assert gp.check() == 0
    o_lp, o_lse, o_ent = O.lmhead_logprob_fwd(Hq, Wq, inp["tok"], inp["lens"], cfg.T)
    for got, want in ((logp, o_lp), (lse, o_lse), (ent, o_ent)):
        assert np.abs(np64(got) - want).max() <= TOL_LOGP
    # it is a different function of the inputs than the bf16 path: the two disagree by far more than that
    b_lp, _, _ = O.lmhead_logprob_fwd(H64, W64, inp["tok"], inp["lens"], cfg.T)
    assert np.abs(o_lp - b_lp).max() > 2 * TOL_LOGP
    g = wl.synthetic_upstream_grad(cfg, inp["lens"])
    dH, dW = gp.bwd(lse, to_device(g))
    o_dH, o_dW = O.lmhead_logprob_bwd(H64, W64, inp["tok"], inp["lens"], cfg.T, g, H_logits=Hq, W_logits=Wq)
    e_h, e_w = rel_fro(np64(dH), o_dH), rel_fro(np64(dW), o_dW)
    assert e_h <= TOL_GRAD and e_w <= TOL_GRAD, (e_h, e_w)
    # the multi-policy pass takes the same route
    logps, lse2, _ = GpuProblem.fwd_multi(gp, [gp.W, to_device(inp["W_ref"])], want_entropy=False)
    assert bool((logps[0] == logp).all()) and bool((lse2 == lse).all())
    o_ref, _, _ = O.lmhead_logprob_fwd(Hq, O.quantize_e4m3(wl.as_f64(inp["W_ref"]), ew), inp["tok"], inp["lens"], cfg.T)
    assert np.abs(np64(logps[1]) - o_ref).max() <= TOL_LOGP


@pytest.mark.parametrize("d,dtype", [(128, "bf16"), (256, "bf16"), (512, "f32"), (1152, "bf16"), (1664, "f32")])
def test_fp8_logits_contraction_lengths(d, dtype):
    """The e4m3 main loop over 1, 2, 4, 9 and 13 K-steps of 128 values (its prologue, the loop unrolled by the
    ring's period, the variable-slot loop and the last three steps each taken or skipped), for both storage
    types of H, W and dZ."""
    cfg = wl.CONFIGS[1].scaled(P=2, G=3, T=112, d=d, V=1024 + 300, dtype=dtype)
    inp = small_inputs(cfg)
    eh, ew = _fp8_exponent(inp["H"]), _fp8_exponent(inp["W"])
    H64, W64 = wl.as_f64(inp["H"]), wl.as_f64(inp["W"])
    Hq, Wq = O.quantize_e4m3(H64, eh), O.quantize_e4m3(W64, ew)
    gp = GpuProblem(cfg, inp["H"], inp["W"], inp["tok"], inp["lens"], flags=4, fp8_exp_h=eh, fp8_exp_w=ew)
    logp, lse, ent, _, _ = gp.fwd()
    assert gp.check() == 0
    o_lp, o_lse, o_ent = O.lmhead_logprob_fwd(Hq, Wq, inp["tok"], inp["lens"], cfg.T)
    for got, want in ((logp, o_lp), (lse, o_lse), (ent, o_ent)):
        assert np.abs(np64(got) - want).max() <= TOL_LOGP
    g = wl.synthetic_upstream_grad(cfg, inp["lens"])
    dH, dW = gp.bwd(lse, to_device(g))
    o_dH, o_dW = O.lmhead_logprob_bwd(H64, W64, inp["tok"], inp["lens"], cfg.T, g, H_logits=Hq, W_logits=Wq)
    e_h, e_w = rel_fro(np64(dH), o_dH), rel_fro(np64(dW), o_dW)
    assert e_h <= TOL_GRAD and e_w <= TOL_GRAD, (e_h, e_w)


@pytest.mark.parametrize("vocab_chunk", [0, 2048])
def test_bf16_dh_output_flag(vocab_chunk):
    """dH written as bf16: the fp32 sums over the vocabulary chunks rounded once at the end."""
    cfg = wl.CONFIGS[1].scaled(P=2, G=4, T=96, d=256, V=8192 + 100)
    inp = small_inputs(cfg)
    g = wl.synthetic_upstream_grad(cfg, inp["lens"])
    ref = GpuProblem(cfg, inp["H"], inp["W"], inp["tok"], inp["lens"], vocab_chunk=vocab_chunk)
    _, lse, _, _, _ = ref.fwd()
    dH32, dW32 = ref.bwd(lse, to_device(g))
    gp = GpuProblem(cfg, inp["H"], inp["W"], inp["tok"], inp["lens"], vocab_chunk=vocab_chunk, flags=8)
    dH16, dW16 = gp.bwd(lse, to_device(g))
    assert gp.check() == 0 and dH16.dtype.itemsize == 2
    assert bool((dW16 == dW32).all())
    a, b = np64(dH16), np64(dH32)
    assert np.all(np.abs(a - b) <= 2.0 ** -8 * np.abs(b) + 1e-12)
    mask = O.index_build(inp["lens"], cfg.T)[0]
    assert np.all(a[mask == 0] == 0)
    o_dH, _ = O.lmhead_logprob_bwd(wl.as_f64(inp["H"]), wl.as_f64(inp["W"]), inp["tok"], inp["lens"], cfg.T, g)
    assert rel_fro(a, o_dH) <= TOL_GRAD


@pytest.mark.parametrize("shape", [(1, 1, 1, 64, 5), (1, 2, 3, 64, 257), (3, 1, 7, 128, 256), (1, 1, 300, 64, 1000)])
def test_smallest_shapes(shape):
    """Degenerate sizes: one slot, a vocabulary smaller than a tile or exactly one tile, one response,
    a group of one (advantage 0), a response longer than a token tile."""
    P, G, T, d, V = shape
    cfg = wl.CONFIGS[1].scaled(P=P, G=G, T=T, d=d, V=V, len_lo=1, len_hi=T)
    inp = small_inputs(cfg)
    r = _grpo_chain(cfg, inp)
    assert r["o_stats"][3] == inp["lens"].sum()


def test_fp32_hidden_size_multiple_of_32():
    """fp32 rows need d to be a multiple of 32 only (one 128-byte K-step); d = 96 also leaves the dH / dW tiles
    ragged along d."""
    cfg = wl.CONFIGS[0].scaled(P=2, G=2, T=24, d=96, V=777)
    r = _grpo_chain(cfg, small_inputs(cfg))
    assert r["err_dH"] < 1e-4 and r["err_dW"] < 1e-4


def test_mfma_probe_does_the_flops_it_reports():
    """The measurement aid behind the benchmark's `ceiling` figures: with all-ones operands every accumulator
    element grows by K = 32 per MFMA, so a thread's 64 blocks x 4 elements sum to 8192 x iters."""
    import torch
    import paper_2603_04411_amd as L
    wgs, iters = 3, 5
    ops = torch.ones(wgs * 256 * 128, dtype=torch.bfloat16, device="cuda")
    sink = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
    L.lmhead_probe_mfma(ops, sink, wgs, iters)
    torch.cuda.synchronize()
    assert bool((sink == 8192.0 * iters).all())
