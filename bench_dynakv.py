#!/usr/bin/env python3
"""Benchmark of the token-adaptive KV compression path on one MI355X (also reachable as
``bench.py --workload dynakv``).

One step = one pass over one layer's key (or value) stream of n tokens, all tensors resident in HBM:
    dynakv_gate (x~ = xU, gate logits, mask, retained counts k) -> dynakv_store (offsets + packed
    segments) -> dynakv_reconstruct (x_bar = x^[0:k] U^-1[0:k, :] for every token).
Prints ONE JSON line: tokens/s of the step, a `roofline` object for the kernel that takes the most
time (timed with HIP events inside the library, on the launch stream) and a `cpu_baseline` object
(the fp64 oracle on a bounded token sample).
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

PEAK_BF16_TFLOPS = 2500.0
PEAK_F32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
KINDS = {4: "kv_gemm_kernel<spectral projection>", 5: "kv_gemm_kernel<gate logits>",
         6: "kv_mask_kernel (softmax + cumulative mask + threshold)", 7: "kv_gemm_kernel<reconstruction>"}
# --backward: one step = dynakv_gate (training outputs off) + dynakv_gate_bwd
BWD_KINDS = {4: "kv_gemm_kernel<spectral projection>", 5: "kv_gemm_kernel<gate logits> (forward + recompute)",
             6: "kv_mask_kernel", 8: "kv_mask_bwd_kernel", 9: "kv_gemm_kernel<g_x~ = g_l W^T + g_xhat m>",
             10: "kv_gemm_kernel<dx = g_x~ U^T>", 11: "gemm_t_kernel<dW>", 12: "gemm_t_kernel<dU>",
             13: "transpose_kernel (two operand copies per parameter gradient)"}


TRAFFIC_KEYS = {4: "spectral_projection", 5: "gate_logits", 6: "kv_mask_kernel", 7: "reconstruction"}


def recorded_traffic(kind: int, config: int):
    """(bytes per launch, source) of one kernel kind: scaled FETCH_SIZE + WRITE_SIZE from the two rocprofv3
    --pmc runs summarised under profiles/ -- used only if that summary says it was measured for this
    workload and these kernel sources (rocprofv3 cannot run inside the timed process); else (None, reason)."""
    from bench import kernel_sources_sha
    name = "hbm_traffic_bench_dynakv.md"
    want = f"kv_config={config} csrc_sha={kernel_sources_sha()}"
    value, valid_for = None, None
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
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


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def to_device(a: np.ndarray):
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def cpu_baseline(cfg, inp, sample: int):
    """The oracle chain (gate, store, reconstruction) on the first `sample` tokens."""
    import workloads as wl
    from oracle import dynakv_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    f = wl.as_f64
    x, U, W, Ui = f(inp["x"][:sample]), f(inp["U"]), f(inp["W"]), f(inp["U_inv"])
    t0 = time.perf_counter()
    g = O.gate(x, U, W, inp["b"], cfg.tau, store_dtype=cfg.dtype)
    off, packed = O.store(g["xt"], g["k"])
    xbar = O.reconstruct(packed, off, g["k"], Ui, store_dtype=cfg.dtype)
    dt = time.perf_counter() - t0
    return ({"value": sample / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
             "sample": f"the first {sample} tokens of the same workload: fp64 gate, store and reconstruction ({dt:.1f} s)"},
            g["k"], xbar)


def backward_main(args, cfg, inp, L, desc, params, ws, xt, k) -> int:
    """Training pair: the gate's forward (x~, k) and its backward (dx, dU, dW, db)."""
    import torch
    import workloads.dynakv as kv
    x, U, W, b = params
    n, d = cfg.n, cfg.d
    tdt = xt.dtype
    g_np, _ = kv.upstream(cfg)
    g_xhat = to_device(g_np)
    g_const = 2 * 0.5 * 0.44 / (n * d)
    ws_b = torch.empty(L.dynakv_bwd_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    dx = torch.empty(n, d, dtype=tdt, device="cuda")
    dU = torch.empty(d, d, dtype=torch.float32, device="cuda")
    dW = torch.empty(d, d, dtype=torch.float32, device="cuda")
    db = torch.empty(d, dtype=torch.float32, device="cuda")

    def step():
        L.dynakv_gate(desc, x, U, W, b, cfg.tau, xt, k, None, None, ws)
        L.dynakv_gate_bwd(desc, x, U, W, b, xt, g_xhat, None, g_const, dx, dU, dW, db, ws_b)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if L.dynakv_check(ws_b) != 0:
        print("bench_dynakv.py: device-side range error", file=sys.stderr)
        return 4
    L.lmhead_timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern = {kind: L.lmhead_timing_read(kind) for kind in BWD_KINDS}
    L.lmhead_timing_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    log(f"{ms_per_step:.3f} ms/step (gate forward + backward)")
    esz = 2 if cfg.dtype == "bf16" else 4
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_MFMA_TFLOPS
    dense = 2.0 * n * d * d
    # algorithmic bytes per launch: mask backward reads logits (4), x~ and g_xhat (esz each) and writes
    # g_l and g_xhat*m (esz each); a transpose pair reads and writes two [n x d] operands
    byts = {6: n * d * 4.0, 8: n * d * (4.0 + 4 * esz), 13: 4.0 * n * d * esz}
    kinds = []
    for kind, name in BWD_KINDS.items():
        ms, cnt = kern[kind]
        avg = ms / cnt if cnt else 0.0
        if kind in byts:
            rate = byts[kind] / (avg * 1e-3) / 1e9 if avg else 0.0
            kinds.append({"kernel": name, "kind": kind, "launches": int(cnt), "avg_ms": avg, "bound": "hbm",
                          "gbs": rate, "frac": rate / PEAK_HBM_GBS})
        else:
            rate = dense / (avg * 1e-3) / 1e12 if avg else 0.0
            kinds.append({"kernel": name, "kind": kind, "launches": int(cnt), "avg_ms": avg, "bound": "mfma",
                          "tflops": rate, "frac": rate / peak})
    per_step = {e["kernel"]: e["avg_ms"] * e["launches"] / args.steps for e in kinds}
    dom = max(kinds, key=lambda e: e["avg_ms"] * e["launches"])
    if dom["bound"] == "mfma":
        roofline = {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom["tflops"], "peak": peak,
                    "unit": "TFLOP/s", "frac": dom["frac"], "traffic": None, "avg_launch_ms": dom["avg_ms"]}
    else:
        roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["gbs"], "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": dom["frac"], "traffic": None, "avg_launch_ms": dom["avg_ms"]}
    cpu = None
    if args.cpu_rows > 0:
        import workloads as wl
        from oracle import dynakv_oracle as O
        m = min(args.cpu_rows, n)
        log(f"timing the oracle's forward + backward on {m} tokens")
        f = wl.as_f64
        xs, gs = f(inp["x"][:m]), f(g_np[:m])
        t0 = time.perf_counter()
        O.gate(xs, f(inp["U"]), f(inp["W"]), inp["b"], cfg.tau, store_dtype=cfg.dtype)
        o = O.gate_bwd(xs, f(inp["U"]), f(inp["W"]), inp["b"], gs, np.full((m, d), g_const), store_dtype=cfg.dtype)
        dt = time.perf_counter() - t0
        got = dx[:m].double().cpu().numpy()
        cpu = {"value": m / dt, "unit": "tokens/s", "cores": os.cpu_count() or 1, "kind": "oracle",
               "sample": f"the first {m} tokens of the same workload: fp64 gate forward and backward ({dt:.1f} s)",
               "gpu_vs_oracle_rel_fro_dx_on_sample": float(np.linalg.norm(got - o["dx"]) / np.linalg.norm(o["dx"]))}
    out = {
        "metric": "tokens/s KV gate forward + backward (training, 1 GPU)",
        "value": n / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"kv_configs[{args.config}] {cfg.name} (gate forward + backward)", "n": n, "d_kv": d},
        "step_tflops": 7 * dense / (ms_per_step * 1e-3) / 1e12,
        "roofline": roofline, "kernels": kinds, "ms_per_step_by_kernel": per_step, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="index into workloads.dynakv.KV_CONFIGS")
    ap.add_argument("--cpu-rows", type=int, default=32768, help="tokens of the oracle sample (0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--backward", action="store_true",
                    help="time the training pair dynakv_gate + dynakv_gate_bwd instead of gate + store + reconstruction")
    args = ap.parse_args(argv)
    if args.gpus != 1:
        print("bench_dynakv.py: this build runs on ONE GPU only; use --gpus 1", file=sys.stderr)
        return 2

    import torch
    import workloads.dynakv as kv
    import paper_2603_04411_amd as L

    if not torch.cuda.is_available():
        print("bench_dynakv.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    cfg = kv.KV_CONFIGS[args.config]
    torch.cuda.set_device(0)
    t_gen = time.perf_counter()
    log(f"generating workload {cfg.name}: n={cfg.n} d={cfg.d} ({cfg.dtype})")
    inp = kv.kv_inputs(cfg)
    log(f"inputs done ({time.perf_counter() - t_gen:.1f} s)")
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    x, U, W, Ui, b = (to_device(inp[key]) for key in ("x", "U", "W", "U_inv", "b"))
    desc = L.make_kv_desc(cfg.n, cfg.d, cfg.dtype)
    assert L.dynakv_validate_desc(desc) == 0
    ws = torch.empty(L.dynakv_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    n, d = cfg.n, cfg.d
    xt = torch.empty(n, d, dtype=tdt, device="cuda")
    k = torch.empty(n, dtype=torch.int32, device="cuda")
    off = torch.empty(n + 1, dtype=torch.int64, device="cuda")
    packed = torch.empty(n * d, dtype=tdt, device="cuda")
    xbar = torch.empty(n, d, dtype=tdt, device="cuda")

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.backward:
        return backward_main(args, cfg, inp, L, desc, (x, U, W, b), ws, xt, k)

    def step():
        L.dynakv_gate(desc, x, U, W, b, cfg.tau, xt, k, None, None, ws)
        L.dynakv_store(desc, xt, k, 0, off, packed, n * d, ws)
        L.dynakv_reconstruct(desc, packed, n * d, off, k, Ui, xbar, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if L.dynakv_check(ws) != 0:
        print("bench_dynakv.py: device-side range error", file=sys.stderr)
        return 4
    L.lmhead_timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern = {kind: L.lmhead_timing_read(kind) for kind in KINDS}
    L.lmhead_timing_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    k_host = k.cpu().numpy().astype(np.int64)
    retain = float(k_host.mean() / d)
    log(f"{ms_per_step:.3f} ms/step, retain rate {retain:.4f}")

    # algorithmic work per launch: the two dense products are 2 n d^2 flops each; the reconstruction
    # is 2 d sum_i k_i; the mask kernel reads the fp32 logits and the bias once and writes k
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_MFMA_TFLOPS
    work = {4: 2.0 * n * d * d, 5: 2.0 * n * d * d, 7: 2.0 * d * float(k_host.sum())}
    mask_bytes = n * d * 4.0 + n * 4.0 + d * 4.0
    kinds = []
    for kind, name in KINDS.items():
        ms, cnt = kern[kind]
        avg = ms / cnt if cnt else 0.0
        if kind == 6:
            rate = mask_bytes / (avg * 1e-3) / 1e9 if avg else 0.0
            kinds.append({"kernel": name, "kind": kind, "launches": int(cnt), "avg_ms": avg, "bound": "hbm",
                          "gbs": rate, "frac": rate / PEAK_HBM_GBS})
        else:
            rate = work[kind] / (avg * 1e-3) / 1e12 if avg else 0.0
            kinds.append({"kernel": name, "kind": kind, "launches": int(cnt), "avg_ms": avg, "bound": "mfma",
                          "tflops": rate, "frac": rate / peak})
    dom = max(kinds, key=lambda e: e["avg_ms"])
    traffic, traffic_source = recorded_traffic(dom["kind"], args.config)
    if dom["bound"] == "mfma":
        roofline = {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom["tflops"], "peak": peak,
                    "unit": "TFLOP/s", "frac": dom["frac"], "traffic": traffic, "traffic_source": traffic_source,
                    "avg_launch_ms": dom["avg_ms"]}
    else:
        roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["gbs"], "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": dom["frac"], "traffic": traffic, "traffic_source": traffic_source,
                    "avg_launch_ms": dom["avg_ms"]}

    cpu = None
    if args.cpu_rows > 0:
        m = min(args.cpu_rows, n)
        log(f"timing the oracle on {m} tokens")
        cpu, o_k, o_xbar = cpu_baseline(cfg, inp, m)
        cpu["gpu_vs_oracle_fraction_of_equal_k_on_sample"] = float(np.mean(k_host[:m] == o_k))
        got = xbar[:m].double().cpu().numpy()
        cpu["gpu_vs_oracle_rel_fro_xbar_on_sample"] = float(np.linalg.norm(got - o_xbar) / np.linalg.norm(o_xbar))

    step_flops = work[4] + work[5] + work[7]
    out = {
        "metric": "tokens/s KV gate + ragged store + low-rank reconstruction (1 GPU)",
        "value": n / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"kv_configs[{args.config}] {cfg.name}", "n": n, "d_kv": d, "tau": cfg.tau,
                   "retain_rate": retain},
        "step_tflops": step_flops / (ms_per_step * 1e-3) / 1e12,
        "roofline": roofline, "kernels": kinds, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
