#!/usr/bin/env python3
"""Writes tests/golden/oracle_regression.json: a handful of oracle outputs on tiny seeded inputs.

The paper prints no worked numerical example for any of the computations built here (its tables are
benchmark scores of trained models), so there are no paper values to store.  This file is instead a
regression guard for the oracles themselves: the values are produced by this script, which calls only
``oracle/`` and the seeded generators, and ``tests/test_golden.py`` recomputes them.  A deliberate change
of an oracle's arithmetic has to regenerate the file (``python tests/golden/make_golden.py``) and say why
in its commit message.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads as wl                      # noqa: E402
import workloads.dynakv as kv               # noqa: E402
from oracle import dynakv_oracle as K       # noqa: E402
from oracle import lmhead_oracle as O       # noqa: E402


def compute() -> dict:
    out = {}
    # LM head + GRPO on the benchmark's tiny fp32 configuration (Eq. 9's L_CE term and the losses on top)
    cfg = wl.CONFIGS[0]
    H, W = wl.as_f64(wl.hidden(cfg)), wl.as_f64(wl.weight(cfg))
    tok, lens = wl.tokens(cfg), wl.lengths(cfg)
    lp, lse, ent = O.lmhead_logprob_fwd(H, W, tok, lens, cfg.T)
    lp_old, _, _ = O.lmhead_logprob_fwd(H, wl.as_f64(wl.weight(cfg, "old")), tok, lens, cfg.T)
    lp_ref, _, _ = O.lmhead_logprob_fwd(H, wl.as_f64(wl.weight(cfg, "ref")), tok, lens, cfg.T)
    adv = O.group_advantage(wl.rewards(cfg), cfg.P, cfg.G)
    loss, g, stats = O.grpo_loss(lp, lp_old, lp_ref, adv, lens, cfg.P, cfg.G, cfg.T, cfg.clip_eps, cfg.clip_eps,
                                 cfg.kl_coef, 0)
    dH, dW = O.lmhead_logprob_bwd(H, W, tok, lens, cfg.T, g)
    ce, _ = O.ce_loss(lp, lens, cfg.T)
    tb, _, gz, resid = O.flowrl_tb_loss(lp, lp_ref, wl.rewards(cfg), wl.log_z(cfg), lens, cfg.P, cfg.G, cfg.T, 1.0)
    out["lmhead_config0"] = {
        "lengths": [int(v) for v in lens], "sum_logp": float(lp.sum()), "sum_lse": float(lse.sum()),
        "sum_entropy": float(ent.sum()), "advantages": [float(v) for v in adv], "grpo_loss": float(loss),
        "grpo_clip_fraction": float(stats[0]), "ce_loss": float(ce), "flowrl_loss": float(tb),
        "flowrl_resid": [float(v) for v in resid], "dH_fro": float(np.linalg.norm(dH)),
        "dW_fro": float(np.linalg.norm(dW)), "dW_colsum_max": float(np.abs(dW.sum(0)).max()),
    }
    # token-adaptive KV compression on the tiny fp32 stream (Sec. 3, Eqs. 1-8)
    kc = kv.KV_CONFIGS[0].scaled(n=40, d=64)
    inp = kv.kv_inputs(kc)
    f = wl.as_f64
    res = K.gate(f(inp["x"]), f(inp["U"]), f(inp["W"]), inp["b"], kc.tau, store_dtype="f32")
    off, packed = K.store(res["xt"], res["k"])
    xbar = K.reconstruct(packed, off, res["k"], f(inp["U_inv"]), store_dtype="f32")
    lit = K.gate(f(inp["x"]), f(inp["U"]), f(inp["W"]), inp["b"], kc.tau, order="literal", store_dtype="f32")
    pen, Rs, _ = K.retain_penalty(res["m"], 0.5)
    out["dynakv_tiny"] = {
        "k": [int(v) for v in res["k"]], "k_literal": [int(v) for v in lit["k"]], "store_elems": int(off[-1]),
        "retain_hard": K.retain_rate_hard(res["k"], kc.d), "retain_soft": Rs, "penalty": pen,
        "xbar_fro": float(np.linalg.norm(xbar)), "recon_err_fro": float(np.linalg.norm(xbar - f(inp["x"]))),
        "sum_mask": float(res["m"].sum()),
    }
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_regression.json")
    with open(path, "w") as fh:
        json.dump(compute(), fh, indent=1, sort_keys=True)
        fh.write("\n")
    print("wrote", path)
