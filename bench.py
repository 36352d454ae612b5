#!/usr/bin/env python3
"""Benchmark of the fused LM-head log-prob + policy-loss step (forward + backward) on one MI355X.

One step = one pass of the whole hot path over one batch of seeded synthetic input, all
tensors already resident in HBM:
    lmhead_logprob_fwd(theta) [lmhead_logprob_fwd_multi(theta, old, ref) where the workload recomputes them]
    -> group_advantage -> grpo_loss | flowrl_tb_loss -> lmhead_logprob_bwd (dH, dW).
Prints ONE JSON line (metric: valid tokens/s of the step) with a `roofline` object for the
dominant matrix-core kernel (timed with HIP events inside the library, on the launch stream)
and a `cpu_baseline` object (the fp64 oracle timed on the host cores on a bounded row sample).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_MFMA_TFLOPS = 157.3
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense fp8 MFMA
KERNEL_NAMES = ["fwd_kernel (logits + online softmax)", "dz_kernel (logits recompute -> dZ)",
                "gemm_t_kernel<dH>", "gemm_t_kernel<dW>"]


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def to_device(a: np.ndarray):
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


TRAFFIC_KEYS = ["fwd_kernel", "dz_kernel", "gemm_t_kernel<dH>", "gemm_t_kernel<dW>"]


def kernel_sources_sha() -> str:
    """Digest of the HIP sources the library is built from (identifies the kernels a profile was taken on)."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2603_04411_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(kind: int, cfg_index: int, vocab_chunk: int):
    """(bytes per launch, source) of one kernel kind: the scaled FETCH_SIZE + WRITE_SIZE that two
    rocprofv3 --pmc runs of this same command recorded under profiles/.  rocprofv3 cannot run inside the
    timed process, so the figure is taken from the summary -- but only if the summary says it was measured
    for THIS workload, THIS chunking and THESE kernel sources; otherwise (None, reason)."""
    name = f"hbm_traffic_bench_config{cfg_index}.md"
    path = os.path.join(ROOT, "profiles", name)
    want = f"config={cfg_index} vocab_chunk={vocab_chunk or 'default'} csrc_sha={kernel_sources_sha()}"
    value, valid_for = None, None
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == TRAFFIC_KEYS[kind]:
                value = float(parts[2])
            if parts and parts[0] == "measured_for":
                valid_for = " ".join(parts[1:])
    except OSError:
        return None, f"no profiles/{name}"
    if valid_for != want:
        return None, f"profiles/{name} was measured for [{valid_for}], this run is [{want}]"
    return value, f"profiles/{name}"


def cpu_baseline(cfg, H_host, W_host, tok, lens, sample_rows: int, gpu_logp=None):
    """Times the oracle (as it stands) on a seeded subset of valid rows: fwd + CE-style bwd."""
    import workloads as wl
    from oracle import lmhead_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    rows = wl.sample_valid_rows(cfg, lens, tok, sample_rows)
    Hs = wl.as_f64(H_host[rows])
    W64 = wl.as_f64(W_host)
    t0 = time.perf_counter()
    lp, lse, ent = O.logprob_rows(Hs, W64, tok[rows])
    g = np.full(rows.size, -1.0 / rows.size)
    dH, dW = O.bwd_rows(Hs, W64, tok[rows], g)
    dt = time.perf_counter() - t0
    out = {"value": rows.size / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
           "sample": f"{rows.size} seeded valid rows of the same workload, full V and d: "
                     f"fp64 logits+lse+entropy forward, then dZ, dH rows and the rows' dW ({dt:.1f} s)"}
    if gpu_logp is not None:
        out["gpu_vs_oracle_max_abs_logp_err_on_sample"] = float(np.abs(gpu_logp[rows] - lp).max())
    return out


def matrix_core_ceiling(L, torch, workgroups: int = 1024, iters: int = 20000):
    """Rate of a bare v_mfma_f32_16x16x32_bf16 loop on register operands (lmhead_probe_mfma), measured here
    and now: on zeros and on N(0,1) bf16 values.  No data moves during the loop, so this is what the matrix
    cores of this machine sustain under the part's power management -- the practical ceiling next to the nominal
    2.5 PFLOP/s peak -- and it shows how much of the gap to the nominal peak is operand content alone."""
    threads = workgroups * 256
    sink = torch.empty(threads, dtype=torch.float32, device="cuda")
    flops = workgroups * 4 * iters * float(1 << 20)
    out = {}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20260304)
    for name in ("zeros", "random"):
        if name == "zeros":
            ops = torch.zeros(threads * 128, dtype=torch.bfloat16, device="cuda")
        else:
            ops = torch.randn(threads * 128, dtype=torch.float32, device="cuda", generator=gen).to(torch.bfloat16)
        times = []
        for rep in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            L.lmhead_probe_mfma(ops, sink, workgroups, iters)
            e1.record()
            e1.synchronize()
            times.append(e0.elapsed_time(e1))
        out[f"mfma_loop_{name}_tflops"] = flops / (min(times[1:]) * 1e-3) / 1e12   # first repetition warms up
    out["what"] = ("bare v_mfma_f32_16x16x32_bf16 loop on register operands, no data movement, "
                   f"{workgroups} workgroups x 4 wavefronts x {iters} x 2^20 flop, measured in this run")
    return out


def main() -> int:
    if "--workload" in sys.argv:
        # the widened path has its own step, metric and roofline: bench.py --workload dynakv [...]
        i = sys.argv.index("--workload")
        which = sys.argv[i + 1] if i + 1 < len(sys.argv) else ""
        rest = sys.argv[1:i] + sys.argv[i + 2:]
        if which == "dynakv":
            import bench_dynakv
            return bench_dynakv.main(rest)
        if which != "lmhead":
            print(f"bench.py: unknown workload {which!r} (lmhead | dynakv)", file=sys.stderr)
            return 2
        sys.argv = [sys.argv[0]] + rest
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=2, help="index into the workload list (default: the target config)")
    ap.add_argument("--vocab-chunk", type=int, default=0)
    ap.add_argument("--cpu-rows", type=int, default=4096, help="rows of the oracle sample (0 = skip)")
    ap.add_argument("--separate-forwards", action="store_true",
                    help="where the step recomputes old/reference log-probs, use one forward call per policy "
                         "instead of the single multi-policy pass (for comparison)")
    ap.add_argument("--fp8-logits", action="store_true",
                    help="variant: logits (forward and recompute) from e4m3 copies of H and W; NOT the headline "
                         "configuration (it changes the numerics), reported for comparison")
    ap.add_argument("--no-ceiling", action="store_true",
                    help="skip the bare matrix-core loop that is reported next to the nominal peak")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one 1 GiB device-to-device copy first (reference point for FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import workloads as wl
    import paper_2603_04411_amd as L

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    cfg = wl.CONFIGS[args.config]
    torch.cuda.set_device(0)
    f32 = dict(dtype=torch.float32, device="cuda")

    t_gen = time.perf_counter()
    log(f"generating workload {cfg.name}: N={cfg.N} d={cfg.d} V={cfg.V} ({cfg.dtype})")
    lens, tok = wl.lengths(cfg), wl.tokens(cfg)
    rewards, logZ = wl.rewards(cfg), wl.log_z(cfg)
    H_host = wl.hidden(cfg)
    log(f"H done ({time.perf_counter() - t_gen:.1f} s)")
    W_host = wl.weight(cfg)
    H, W = to_device(H_host), to_device(W_host)
    W_old = to_device(wl.weight(cfg, "old")) if cfg.loss == "grpo" else None
    W_ref = to_device(wl.weight(cfg, "ref"))
    log(f"weights done ({time.perf_counter() - t_gen:.1f} s)")
    tok_d, lens_d = to_device(tok), to_device(lens)
    rew_d, logZ_d = to_device(rewards), to_device(logZ)
    nv = int(lens.sum())

    fp8 = {}
    if args.fp8_logits:
        # power-of-two scales that bring the largest magnitude of each operand just inside the e4m3 range
        amax_h = float(np.abs(wl.as_f64(H_host[: 1 << 16])).max())
        amax_w = max(float(np.abs(wl.as_f64(m[: 1 << 16])).max()) for m in (W_host,))
        fp8 = dict(flags=4, fp8_exp_h=int(np.floor(np.log2(448.0 / amax_h))) - 1,
                   fp8_exp_w=int(np.floor(np.log2(448.0 / amax_w))) - 1)
    desc = L.make_desc(cfg.P, cfg.G, cfg.T, cfg.d, cfg.V, cfg.dtype, vocab_chunk=args.vocab_chunk, **fp8)
    assert L.validate_desc(desc) == 0
    n_pol = (3 if cfg.loss == "grpo" else 2) if cfg.recompute_old_ref else 1
    ws = torch.empty(max(L.workspace_bytes(desc), L.multi_workspace_bytes(desc, n_pol)), dtype=torch.uint8,
                     device="cuda")
    loss_ws = torch.empty(L.loss_workspace_bytes(cfg.P, cfg.G, cfg.T), dtype=torch.uint8, device="cuda")
    N = cfg.N
    logp, lse = torch.empty(N, **f32), torch.empty(N, **f32)
    ent = torch.empty(N, **f32) if cfg.want_entropy else None
    lp_old, lp_ref = torch.empty(N, **f32), torch.empty(N, **f32)
    scratch_lse = torch.empty(N, **f32)
    adv = torch.empty(cfg.R, **f32)
    loss = torch.zeros(1, **f32)
    g_logp = torch.empty(N, **f32)
    g_logZ = torch.empty(cfg.P, **f32)
    stats = torch.zeros(4, **f32)
    dH = torch.empty(N, cfg.d, **f32)
    dW = torch.empty(cfg.V, cfg.d, **f32)

    def fwd_other():
        if W_old is not None:
            L.lmhead_logprob_fwd(desc, H, W_old, tok_d, lens_d, lp_old, scratch_lse, None, None, None, ws)
        L.lmhead_logprob_fwd(desc, H, W_ref, tok_d, lens_d, lp_ref, scratch_lse, None, None, None, ws)

    def step():
        if cfg.recompute_old_ref and args.separate_forwards:
            L.lmhead_logprob_fwd(desc, H, W, tok_d, lens_d, logp, lse, ent, None, None, ws)
            fwd_other()
        elif cfg.recompute_old_ref:
            # current, old and reference policy share the hidden states: one pass over all of them
            mats = [W, W_old, W_ref] if W_old is not None else [W, W_ref]
            outs = [logp, lp_old, lp_ref] if W_old is not None else [logp, lp_ref]
            L.lmhead_logprob_fwd_multi(desc, H, mats, tok_d, lens_d, outs, lse, ent, None, None, ws)
        else:
            L.lmhead_logprob_fwd(desc, H, W, tok_d, lens_d, logp, lse, ent, None, None, ws)
        if cfg.loss == "grpo":
            L.group_advantage(rew_d, cfg.P, cfg.G, 1e-6, 0, adv)
            L.grpo_loss(logp, lp_old, lp_ref, adv, lens_d, cfg.P, cfg.G, cfg.T, cfg.clip_eps, cfg.clip_eps,
                        cfg.kl_coef, 0, loss, g_logp, stats, loss_ws)
        else:
            L.flowrl_tb_loss(logp, lp_ref, rew_d, logZ_d, lens_d, cfg.P, cfg.G, cfg.T, cfg.beta, loss, g_logp,
                             g_logZ, None, loss_ws)
        L.lmhead_logprob_bwd(desc, H, W, tok_d, lens_d, lse, g_logp, dH, dW, ws)

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not cfg.recompute_old_ref:
        fwd_other()      # old / reference log-probs are inputs of the step here: computed once, untimed
    torch.cuda.synchronize()
    log(f"setup done ({time.perf_counter() - t_gen:.1f} s); warmup x{args.warmup}")
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if L.lmhead_check(ws) != 0:
        print("bench.py: device-side range error in the synthetic inputs", file=sys.stderr)
        return 4

    L.lmhead_timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern = [L.lmhead_timing_read(k) for k in range(4)]
    L.lmhead_timing_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    log(f"{ms_per_step:.1f} ms/step, loss {float(loss.item()):.6f}")

    # roofline of the dominant matrix-core kernel: algorithmic flops per launch = 2 * N_v * d * (vocabulary
    # columns the launch covers); summed over a pass that is 2 * N_v * V * d per kernel kind.
    n_fwd_passes = 1 + ((2 if W_old is not None else 1) if cfg.recompute_old_ref else 0)
    flops_per_pass = 2.0 * nv * cfg.V * cfg.d
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_MFMA_TFLOPS
    kinds = []
    for k, (ms, n) in enumerate(kern):
        passes = args.steps * (n_fwd_passes if k == 0 else 1)
        tf = flops_per_pass * passes / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
        kpeak = PEAK_FP8_TFLOPS if (args.fp8_logits and k < 2) else peak     # the two logits kernels run in e4m3
        kinds.append({"kernel": KERNEL_NAMES[k], "launches": int(n), "avg_ms": ms / n if n else 0.0,
                      "total_ms": ms, "tflops": tf, "peak": kpeak, "frac": tf / kpeak})
    dom = max(range(4), key=lambda k: kern[k][0])
    dms, dn = kern[dom]
    dom_passes = args.steps * (n_fwd_passes if dom == 0 else 1)
    flops_per_launch = flops_per_pass * dom_passes / dn
    achieved = flops_per_launch / (dms / dn * 1e-3) / 1e12
    dpeak = kinds[dom]["peak"]
    traffic, traffic_source = (None, "not recorded for the 8-bit logits variant") if args.fp8_logits else \
        recorded_traffic(dom, cfg.index, args.vocab_chunk)
    roofline = {"bound": "mfma", "kernel": KERNEL_NAMES[dom], "achieved": achieved, "peak": dpeak,
                "unit": "TFLOP/s", "frac": achieved / dpeak,
                "traffic": traffic, "traffic_source": traffic_source,
                "flops_per_launch": flops_per_launch, "avg_launch_ms": dms / dn}
    step_flops_hw = flops_per_pass * (3 + n_fwd_passes)       # executed, including the dZ recompute
    step_flops_model = flops_per_pass * 3                      # logits + dH + dW

    ceiling = None
    if cfg.dtype == "bf16" and not args.fp8_logits and not args.no_ceiling:      # the probe is a bf16 loop
        ceiling = matrix_core_ceiling(L, torch)
        log(f"bare MFMA loop: {ceiling['mfma_loop_zeros_tflops']:.0f} TFLOP/s on zeros, "
            f"{ceiling['mfma_loop_random_tflops']:.0f} on random bf16")
        roofline["frac_of_mfma_loop_on_random_operands"] = achieved / ceiling["mfma_loop_random_tflops"]
    gpu_logp = logp.double().cpu().numpy()
    cpu = None
    if args.cpu_rows > 0:
        log(f"timing the oracle on {args.cpu_rows} rows")
        cpu = cpu_baseline(cfg, H_host, W_host, tok, lens, args.cpu_rows, None if args.fp8_logits else gpu_logp)

    out = {
        "metric": "tokens/s fused LM-head logprob+loss fwd+bwd (1 GPU)",
        "value": nv / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype + ("+e4m3 logits" if args.fp8_logits else ""), "data": "synthetic",
        "config": {"workload": f"configs[{cfg.index}] {cfg.name}", "P": cfg.P, "G": cfg.G, "T": cfg.T,
                   "d": cfg.d, "V": cfg.V, "token_slots": cfg.N, "valid_tokens": nv, "loss": cfg.loss,
                   "vocab_chunk": int(args.vocab_chunk) or "library default",
                   "tokens_counted": "valid (unpadded) tokens", "slots_per_s": cfg.N / (ms_per_step * 1e-3)},
        # executed = 2 N_v V d per matrix-core pass (logits, logits recompute, dH, dW: 8 N_v V d per step
        # plus the extra forwards where old / reference log-probs are recomputed): what the matrix cores
        # do and what the 60 % target refers to.  model = 6 N_v V d (logits + dH + dW), no recompute.
        "step_tflops_executed": step_flops_hw / (ms_per_step * 1e-3) / 1e12,
        # one peak does not fit a step whose logits kernels run in e4m3 and whose dH / dW run in bf16
        "step_frac_of_peak_executed": None if args.fp8_logits else step_flops_hw / (ms_per_step * 1e-3) / 1e12 / peak,
        "step_tflops_model": step_flops_model / (ms_per_step * 1e-3) / 1e12,
        "step_frac_of_peak_model": None if args.fp8_logits else step_flops_model / (ms_per_step * 1e-3) / 1e12 / peak,
        "step_flops": {"executed": step_flops_hw, "model": step_flops_model},
        "loss": float(loss.item()),
        "roofline": roofline,
        "ceiling": ceiling,
        "kernels": kinds,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
