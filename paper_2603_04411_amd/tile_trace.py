"""Where a tile's time goes: per-workgroup time stamps of ``fwd_kernel`` or ``dz_kernel`` from the trace build.

    python -m paper_2603_04411_amd.build --trace            # liblmhead_trace.so (same sources, -DLMHEAD_TRACE)
    python -m paper_2603_04411_amd.tile_trace fwd c2 c1     # on the GPU; `dz` instead of `fwd` for the dZ kernel

The trace build writes, for each of the first 2^19 workgroups, the 100 MHz real-time counter at fourteen points of
the tile (kernel entry, main-loop entry, first data landed, after 5 / 10 / 15 K-steps, end of the unrolled loop,
end of the drain, epilogue start, three points inside it, and its end) and the shader clock counter at six of them, which gives the clock
frequency inside the loop and inside the epilogue separately.  Inputs are seeded and synthetic (N(0,1) hidden
states, N(0, 0.02^2) weights, uniform lengths in [T/4, T]).  A diagnostic: it loads the trace library directly
and is not used by the binding, the tests or the benchmark.
"""
from __future__ import annotations

import ctypes as C
import os
import sys

import numpy as np
import torch

from . import binding

SHAPES = {"c2": (32, 8, 2048, 4096, 151936), "c1": (8, 8, 256, 2048, 151936)}   # P, G, T, d, V of configs[2], configs[1]
NWG = 1 << 19
TICK_US = 0.01     # the real-time counter runs at 100 MHz


EPILOGUE = {
    "fwd": [("epilogue: target-logit capture", 2, 11), ("epilogue: softmax statistics of 256 values per lane", 11, 12),
            ("epilogue: lane-group merges, partials to LDS", 12, 13), ("epilogue: barrier, cross-wave merge, stores", 13, 3)],
    "dz": [("epilogue: per-token scalars fetched (one round trip)", 2, 11),
           ("epilogue: dZ formed, stored from registers, staged in LDS", 11, 12), ("epilogue: barrier", 12, 13),
           ("epilogue: vocabulary-major copy streamed out of LDS", 13, 3)],
}


def main(argv):
    kernel = "fwd"
    if argv and argv[0] in ("fwd", "dz"):
        kernel, argv = argv[0], argv[1:]
    names = argv or ["c2", "c1"]
    kind = {"fwd": 1, "dz": 2}[kernel]
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblmhead_trace.so")
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2603_04411_amd.build --trace`")
    binding.library_path = lambda: path          # this process works on the trace build
    lib = binding.load_library()
    lib.lmhead_debug_set_trace.argtypes = [C.c_void_p, C.c_int]
    lib.lmhead_debug_set_trace.restype = C.c_int
    tbuf = torch.zeros(2 * NWG * 16, dtype=torch.int64, device="cuda")
    for name in names:
        P, G, T, d, V = SHAPES[name]
        torch.manual_seed(0)
        N = P * G * T
        H = torch.randn(N, d, device="cuda").bfloat16()
        W = (torch.randn(V, d, device="cuda") * 0.02).bfloat16()
        tok = torch.randint(0, V, (N,), device="cuda", dtype=torch.int32)
        lens = torch.randint(T // 4, T + 1, (P * G,), device="cuda", dtype=torch.int32)
        desc = binding.make_desc(P, G, T, d, V, "bf16")
        ws = torch.empty(binding.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
        logp = torch.empty(N, dtype=torch.float32, device="cuda")
        lse = torch.empty_like(logp)
        if kernel == "dz":
            g = torch.randn(N, dtype=torch.float32, device="cuda") * 1e-4
            dH = torch.empty(N, d, dtype=torch.float32, device="cuda")
            dW = torch.empty(V, d, dtype=torch.float32, device="cuda")
        for _ in range(2):       # the second pass is the one that is read
            assert lib.lmhead_debug_set_trace(tbuf.data_ptr(), kind) == 0
            tbuf.zero_()
            binding.lmhead_logprob_fwd(desc, H, W, tok, lens, logp, lse, None, None, None, ws)
            if kernel == "dz":   # every vocabulary chunk's launch writes its workgroups' records; the last full-width one stays
                binding.lmhead_logprob_bwd(desc, H, W, tok, lens, lse, g, dH, dW, ws)
            torch.cuda.synchronize()
        full = tbuf.cpu().numpy().astype(np.uint64).reshape(2 * NWG, 16)
        t, cy = full[:NWG].astype(np.int64), full[NWG:].astype(np.int64)
        ok = (t[:, 3] > t[:, 0]) & (t[:, 0] > 0) & (t[:, 10] > 0) & (t[:, 3] - t[:, 0] < 100000)
        t, cy = t[ok], cy[ok]
        ksteps = d * 2 // 128
        print(f"== {kernel}_kernel, {name}: P x G x T = {P} x {G} x {T}, d = {d} ({ksteps} K-steps per tile), V = {V}; "
              f"{len(t)} workgroups traced")
        unrolled_end = 5 * ((ksteps - 7) // 5 + 1) if ksteps >= 7 else 0
        segs = [("kernel entry -> main loop entry", 0, 1), ("prologue: first two K-steps requested, own loads of K-step 0 landed", 1, 4),
                ("prologue barrier (all waves' loads landed)", 4, 5), ("K-steps 0-4", 5, 6), ("K-steps 5-9", 6, 7),
                ("K-steps 10-14", 7, 8), (f"K-steps 15-{unrolled_end - 1} (steady state)", 8, 9),
                (f"K-steps {unrolled_end}-{ksteps - 1} (variable-slot loop and drain)", 9, 10), ("final barrier", 10, 2)]
        segs += EPILOGUE[kernel] + [("epilogue, all of it", 2, 3), ("whole tile", 0, 3)]
        print(f"{'section':74s} {'mean us':>8s} {'p10':>7s} {'p50':>7s} {'p90':>7s}")
        for label, a, b in segs:
            x = (t[:, b] - t[:, a]) * TICK_US
            x = x[(x > -1) & (x < 1000)]
            print(f"{label:74s} {x.mean():8.2f} {np.percentile(x, 10):7.2f} {np.percentile(x, 50):7.2f} {np.percentile(x, 90):7.2f}")
        for label, a, b, steps in (("K-steps 0-4", 5, 6, 5), ("steady-state loop", 8, 9, unrolled_end - 15), ("epilogue", 2, 3, 0)):
            us = (t[:, b] - t[:, a]) * TICK_US
            cc = (cy[:, b] - cy[:, a]).astype(np.float64)
            good = (us > 0.5) & (cc > 0)
            line = f"{label}: {us[good].mean():.2f} us = {cc[good].mean():.0f} shader clocks -> {np.median(cc[good] / us[good]):.0f} MHz"
            if steps > 0:
                line += f"; {cc[good].mean() / steps:.0f} clocks per K-step (2048 of them are MFMA issue cycles: {100 * 2048 * steps / cc[good].mean():.1f} % busy)"
            print(line)
        if kernel == "fwd":
            # do the workgroups of one XCD start together?  (sorted start times of the tiles of XCD 0)
            xcc = cy[:, 12] & 0xf
            st = np.sort(t[xcc == 0][:, 0])
            gaps = np.diff(st) * TICK_US
            print(f"XCD 0: {len(st)} tiles; gap between consecutive tile starts: p50 {np.percentile(gaps, 50):.2f} us, "
                  f"p90 {np.percentile(gaps, 90):.2f}, p99 {np.percentile(gaps, 99):.2f} (rounds of 32 tiles that start together)")
        del H, W, ws
        if kernel == "dz":
            del dH, dW
        torch.cuda.empty_cache()
    lib.lmhead_debug_set_trace(None, 0)


if __name__ == "__main__":
    main(sys.argv[1:])
