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


TRAFFIC_KEYS = {4: "spectral_projection", 5: "gate_logits", 6: "kv_mask_kernel", 7: "reconstruction"}


def recorded_traffic(kind: int):
    """HBM-side bytes per launch of one kernel kind for kv_configs[2], as recorded from two rocprofv3
    --pmc runs (FETCH_SIZE, WRITE_SIZE; scaling stated in the file).  None if absent."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_bench_dynakv.md")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == TRAFFIC_KEYS[kind]:
                return float(parts[2])
    except OSError:
        pass
    return None


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


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="index into workloads.dynakv.KV_CONFIGS")
    ap.add_argument("--cpu-rows", type=int, default=32768, help="tokens of the oracle sample (0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true")
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

    def step():
        L.dynakv_gate(desc, x, U, W, b, cfg.tau, xt, k, None, None, ws)
        L.dynakv_store(desc, xt, k, 0, off, packed, n * d, ws)
        L.dynakv_reconstruct(desc, packed, n * d, off, k, Ui, xbar, ws)

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
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
    traffic = recorded_traffic(dom["kind"]) if args.config == 2 else None
    if dom["bound"] == "mfma":
        roofline = {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom["tflops"], "peak": peak,
                    "unit": "TFLOP/s", "frac": dom["frac"], "traffic": traffic, "avg_launch_ms": dom["avg_ms"]}
    else:
        roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["gbs"], "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": dom["frac"], "traffic": traffic, "avg_launch_ms": dom["avg_ms"]}

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
