"""Test-side plumbing: upload seeded inputs, run the HIP path through the C ABI, run the oracle chain."""
from __future__ import annotations

import numpy as np

import workloads as wl


def to_device(a: np.ndarray):
    """numpy -> torch device tensor; uint16 arrays are bf16 bit patterns."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


class GpuProblem:
    """Device-resident tensors of one workload plus its workspace."""

    def __init__(self, cfg, H, W, tok, lens, vocab_chunk=0, flags=0, fp8_exp_h=0, fp8_exp_w=0, ldH=None, ldW=None):
        import torch
        import paper_2603_04411_amd as L
        self.L = L
        self.cfg = cfg
        self.desc = L.make_desc(cfg.P, cfg.G, cfg.T, cfg.d, cfg.V, cfg.dtype, vocab_chunk=vocab_chunk, flags=flags,
                                fp8_exp_h=fp8_exp_h, fp8_exp_w=fp8_exp_w, ldH=ldH, ldW=ldW)
        assert L.validate_desc(self.desc) == 0
        self.H = to_device(widen_rows(H, ldH))
        self.W = to_device(widen_rows(W, ldW))
        self.tok = to_device(np.ascontiguousarray(tok, dtype=np.int32))
        self.lens = to_device(np.ascontiguousarray(lens, dtype=np.int32))
        self.ws = torch.empty(L.workspace_bytes(self.desc), dtype=torch.uint8, device="cuda")
        self.loss_ws = torch.empty(L.loss_workspace_bytes(cfg.P, cfg.G, cfg.T), dtype=torch.uint8, device="cuda")

    def fwd(self, W=None, want_entropy=True, want_index=True):
        import torch
        cfg = self.cfg
        N, R = cfg.N, cfg.R
        f = dict(dtype=torch.float32, device="cuda")
        logp = torch.full((N,), 7.0, **f)
        lse = torch.full((N,), 7.0, **f)
        ent = torch.full((N,), 7.0, **f) if want_entropy else None
        mask = torch.full((N,), 9, dtype=torch.uint8, device="cuda") if want_index else None
        cu = torch.full((R + 1,), -9, dtype=torch.int32, device="cuda") if want_index else None
        self.L.lmhead_logprob_fwd(self.desc, self.H, self.W if W is None else W, self.tok, self.lens,
                                  logp, lse, ent, mask, cu, self.ws)
        return logp, lse, ent, mask, cu

    def fwd_multi(self, Ws, want_entropy=True):
        """One pass over several weight matrices (device tensors); returns ([logp...], lse, entropy)."""
        import torch
        cfg = self.cfg
        f = dict(dtype=torch.float32, device="cuda")
        logps = [torch.full((cfg.N,), 7.0, **f) for _ in Ws]
        lse = torch.full((cfg.N,), 7.0, **f)
        ent = torch.full((cfg.N,), 7.0, **f) if want_entropy else None
        ws = torch.empty(self.L.multi_workspace_bytes(self.desc, len(Ws)), dtype=torch.uint8, device="cuda")
        self.ws_multi = ws
        self.L.lmhead_logprob_fwd_multi(self.desc, self.H, Ws, self.tok, self.lens, logps, lse, ent, None, None, ws)
        assert self.L.lmhead_check(ws) == 0
        return logps, lse, ent

    def bwd(self, lse, g_logp, dW_init=None):
        import torch
        cfg = self.cfg
        dh_type = torch.bfloat16 if (self.desc.flags & 8) else torch.float32
        dH = torch.full((cfg.N, cfg.d), 3.0, dtype=dh_type, device="cuda")
        dW = torch.full((cfg.V, cfg.d), 3.0, dtype=torch.float32, device="cuda") if dW_init is None else dW_init
        self.L.lmhead_logprob_bwd(self.desc, self.H, self.W, self.tok, self.lens, lse, g_logp, dH, dW, self.ws)
        return dH, dW

    def advantage(self, rewards, eps=1e-6, ddof=0):
        import torch
        r = to_device(np.ascontiguousarray(rewards, dtype=np.float32))
        adv = torch.empty_like(r)
        self.L.group_advantage(r, self.cfg.P, self.cfg.G, eps, ddof, adv)
        return adv

    def grpo(self, logp, logp_old, logp_ref, adv, clip_lo=0.2, clip_hi=0.2, kl=0.04, agg=0):
        import torch
        cfg = self.cfg
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        g = torch.full((cfg.N,), 5.0, dtype=torch.float32, device="cuda")
        stats = torch.zeros(4, dtype=torch.float32, device="cuda")
        self.L.grpo_loss(logp, logp_old, logp_ref, adv, self.lens, cfg.P, cfg.G, cfg.T, clip_lo, clip_hi, kl, agg,
                         loss, g, stats, self.loss_ws)
        return loss, g, stats

    def flowrl(self, logp, logp_ref, rewards, logZ, beta):
        import torch
        cfg = self.cfg
        r = to_device(np.ascontiguousarray(rewards, dtype=np.float32))
        z = to_device(np.ascontiguousarray(logZ, dtype=np.float32))
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        g = torch.full((cfg.N,), 5.0, dtype=torch.float32, device="cuda")
        gz = torch.zeros(cfg.P, dtype=torch.float32, device="cuda")
        resid = torch.zeros(cfg.R, dtype=torch.float32, device="cuda")
        self.L.flowrl_tb_loss(logp, logp_ref, r, z, self.lens, cfg.P, cfg.G, cfg.T, beta, loss, g, gz, resid,
                              self.loss_ws)
        return loss, g, gz, resid

    def ce(self, logp):
        import torch
        cfg = self.cfg
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        g = torch.full((cfg.N,), 5.0, dtype=torch.float32, device="cuda")
        self.L.ce_loss(logp, self.lens, cfg.R, cfg.T, loss, g, self.loss_ws)
        return loss, g

    def index_regions(self, ws=None, npol=1):
        """(N_v, row_slot[Ncap], tok_c[Ncap], gathered_id[npol][Ncap]) as the last forward left them in `ws`."""
        import torch
        ws = self.ws if ws is None else ws
        torch.cuda.synchronize()
        out = []
        for which in (self.L.WS_NV, self.L.WS_ROW_SLOT, self.L.WS_TOK_C, self.L.WS_GATHERED_ID):
            off, nbytes = self.L.workspace_region(self.desc, npol, which)
            out.append(ws[off:off + nbytes].cpu().numpy().view(np.int32).copy())
        ncap = out[1].size
        return int(out[0][0]), out[1], out[2], out[3].reshape(npol, ncap)

    def check(self):
        return self.L.lmhead_check(self.ws)


def widen_rows(a: np.ndarray, ld):
    """Rows of `a` embedded in a buffer with row stride `ld` elements; the gap holds a non-zero filler
    (bf16 / fp32 2.0) so that a kernel that ignored the stride would not pass by reading zeros."""
    if ld is None or ld == a.shape[1]:
        return a
    fill = 0x4000 if a.dtype == np.uint16 else 2.0
    wide = np.full((a.shape[0], ld), fill, dtype=a.dtype)
    wide[:, : a.shape[1]] = a
    return wide


def assert_index_parity(gp, o_row_slot, tok, ws=None, npol=1):
    """Bit-exact check of the compaction map, the compacted token ids and the gathered vocabulary columns
    against the oracle's index_build (integers: ==)."""
    nv, row_slot, tok_c, gid = gp.index_regions(ws, npol)
    assert nv == o_row_slot.size
    assert np.array_equal(row_slot[:nv], o_row_slot), "compaction map"
    pad_end = (nv + 255) // 256 * 256
    assert np.all(row_slot[nv:pad_end] == -1), "compaction map is padded with -1 up to the tile multiple"
    want = np.asarray(tok, dtype=np.int32)[o_row_slot]
    assert np.array_equal(tok_c[:nv], want), "compacted token ids"
    assert np.all(tok_c[nv:pad_end] == -1)
    for p in range(npol):
        assert np.array_equal(gid[p, :nv], want), "gathered vocabulary column != sampled token id"
        assert np.all(gid[p, nv:pad_end] == -1)


def np64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_fro(a, b):
    """||a - b||_F / ||b||_F."""
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def small_inputs(cfg):
    """All inputs of a (small) workload as numpy arrays."""
    return dict(
        H=wl.hidden(cfg), W=wl.weight(cfg), W_old=wl.weight(cfg, "old"), W_ref=wl.weight(cfg, "ref"),
        tok=wl.tokens(cfg), lens=wl.lengths(cfg), rewards=wl.rewards(cfg), logZ=wl.log_z(cfg),
    )


class KvProblem:
    """Device tensors and workspace of one KV-compression workload (include/dynakv.h)."""

    def __init__(self, cfg, inp, flags=0, ldx=None):
        import torch
        import paper_2603_04411_amd as L
        self.L, self.cfg = L, cfg
        self.tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        x = inp["x"]
        if ldx is not None and ldx != cfg.d:          # rows embedded in a wider buffer
            wide = np.zeros((cfg.n, ldx), dtype=x.dtype)
            wide[:, : cfg.d] = x
            x = wide
        self.desc = L.make_kv_desc(cfg.n, cfg.d, cfg.dtype, ldx=ldx, flags=flags)
        assert L.dynakv_validate_desc(self.desc) == 0
        self.x, self.U, self.W, self.U_inv = (to_device(a) for a in (x, inp["U"], inp["W"], inp["U_inv"]))
        self.b = to_device(inp["b"])
        self.ws = torch.empty(L.dynakv_workspace_bytes(self.desc), dtype=torch.uint8, device="cuda")

    def gate(self, tau, soft=True):
        import torch
        cfg = self.cfg
        xt = torch.full((cfg.n, cfg.d), 3.0, dtype=self.tdt, device="cuda")
        k = torch.full((cfg.n,), -7, dtype=torch.int32, device="cuda")
        m = torch.full((cfg.n, cfg.d), 3.0, dtype=torch.float32, device="cuda") if soft else None
        xhat = torch.full((cfg.n, cfg.d), 3.0, dtype=self.tdt, device="cuda") if soft else None
        self.L.dynakv_gate(self.desc, self.x, self.U, self.W, self.b, tau, xt, k, m, xhat, self.ws)
        return xt, k, m, xhat

    def store(self, xt, k, capacity=None, off_base=0, off=None, packed=None):
        import torch
        cfg = self.cfg
        capacity = off_base + cfg.n * cfg.d if capacity is None else capacity
        if off is None:
            off = torch.full((cfg.n + 1,), -1, dtype=torch.int64, device="cuda")
        if packed is None:
            packed = torch.full((max(capacity, 8),), 5.0, dtype=self.tdt, device="cuda")
        self.L.dynakv_store(self.desc, xt, k, off_base, off, packed, capacity, self.ws)
        return off, packed

    def reconstruct(self, packed, packed_elems, off, k):
        import torch
        cfg = self.cfg
        xbar = torch.full((cfg.n, cfg.d), 3.0, dtype=self.tdt, device="cuda")
        self.L.dynakv_reconstruct(self.desc, packed, packed_elems, off, k, self.U_inv, xbar, self.ws)
        return xbar

    def retain(self, k, m, alpha, want_grad=True):
        import torch
        cfg = self.cfg
        out = torch.zeros(3, dtype=torch.float32, device="cuda")
        g = torch.full((cfg.n, cfg.d), 3.0, dtype=torch.float32, device="cuda") if want_grad else None
        self.L.dynakv_retain(self.desc, k, m, alpha, out, g, self.ws)
        return out, g

    def gate_bwd(self, xt, g_xhat, g_m=None, g_m_const=0.0, accumulate_into=None):
        """dx, dU, dW, db of dynakv_gate_bwd (its own, larger workspace).  `accumulate_into` = (dU, dW, db)
        tensors to add to, with DYNAKV_FLAG_ACCUM_GRAD."""
        import torch
        cfg = self.cfg
        desc = self.desc
        if accumulate_into is not None:
            desc = self.L.make_kv_desc(cfg.n, cfg.d, cfg.dtype, ldx=self.desc.ldx,
                                       flags=self.desc.flags | self.L.FLAG_ACCUM_GRAD)
        if getattr(self, "ws_bwd", None) is None:
            self.ws_bwd = torch.empty(self.L.dynakv_bwd_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
        dx = torch.full((cfg.n, cfg.d), 3.0, dtype=self.tdt, device="cuda")
        if accumulate_into is None:
            dU = torch.full((cfg.d, cfg.d), 3.0, dtype=torch.float32, device="cuda")
            dW = torch.full((cfg.d, cfg.d), 3.0, dtype=torch.float32, device="cuda")
            db = torch.full((cfg.d,), 3.0, dtype=torch.float32, device="cuda")
        else:
            dU, dW, db = accumulate_into
        self.L.dynakv_gate_bwd(desc, self.x, self.U, self.W, self.b, xt, g_xhat, g_m, g_m_const, dx, dU, dW, db,
                               self.ws_bwd)
        return dx, dU, dW, db

    def check(self):
        return self.L.dynakv_check(self.ws)
