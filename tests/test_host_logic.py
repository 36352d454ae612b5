"""CPU-only checks of the host side of the library: the shared object loads and exports every
symbol the header declares, argument validation returns the documented codes before anything
is launched, workspace sizing behaves, and the tile-walk mapping is a bijection."""
import ctypes as C
import os
import re
import subprocess
import sys

import pytest

import paper_2603_04411_amd as L
from paper_2603_04411_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(L.library_path()):
        from paper_2603_04411_amd.build import build_library
        build_library()
    return L.load_library()


def test_every_declared_symbol_is_exported(lib):
    declared = []
    for name, symbols in (("lmhead.h", L.EXPORTED_SYMBOLS), ("dynakv.h", L.DYNAKV_SYMBOLS)):
        header = open(os.path.join(ROOT, "include", name)).read()
        here = re.findall(r"LMHEAD_API\s+[\w\s\*]+?\b(\w+)\s*\(", header)
        assert len(here) >= 7
        for sym in here:
            assert hasattr(lib, sym), f"{sym} is declared in {name} but not exported"
        assert sorted(here) == sorted(symbols)
        declared += here
    assert lib.lmhead_abi_version() == 2
    # nothing but the C ABI is exported
    out = subprocess.run(["nm", "-D", "--defined-only", L.library_path()], capture_output=True, text=True).stdout
    exported = [ln.split()[-1] for ln in out.splitlines() if " T " in ln]
    assert sorted(exported) == sorted(declared)
    # the diagnostic trace build (if it has been built) is the same ABI plus its one hook; the product library
    # must not carry that hook
    assert "lmhead_debug_set_trace" not in exported
    trace = os.path.join(os.path.dirname(L.library_path()), "liblmhead_trace.so")
    if os.path.exists(trace):
        out = subprocess.run(["nm", "-D", "--defined-only", trace], capture_output=True, text=True).stdout
        texp = [ln.split()[-1] for ln in out.splitlines() if " T " in ln]
        assert sorted(texp) == sorted(declared + ["lmhead_debug_set_trace"])


def test_descriptor_matches_c_layout():
    # int32 x8, int64 x2, uint32 x2 with natural alignment
    assert C.sizeof(B.LmheadDesc) == 8 * 4 + 2 * 8 + 2 * 4
    assert B.LmheadDesc.ldH.offset == 32 and B.LmheadDesc.flags.offset == 48


def test_descriptor_validation_codes(lib):
    ok = L.make_desc(2, 4, 32, 256, 4096, "f32")
    assert L.validate_desc(ok) == 0 and L.workspace_bytes(ok) > 0
    cases = [
        (dict(P=0), -2), (dict(T=-1), -2), (dict(V=0), -2), (dict(d=250), -2), (dict(d=0), -2),
        (dict(ldH=128), -2), (dict(ldW=255), -2), (dict(dtype=7), -3), (dict(flags=1 << 9), -3), (dict(flags=16), -3),
        (dict(vocab_chunk=-5), -2), (dict(P=70000, G=70000), -2), (dict(ldH=258), -4),
        (dict(fp8_exp_h=3), -2), (dict(fp8_exp_w=-1), -2),                      # exponents without the flag
        (dict(flags=4, d=192, ldH=192, ldW=192), -2), (dict(flags=4, fp8_exp_w=99), -2),
    ]
    for change, code in cases:
        kw = dict(P=2, G=4, T=32, d=256, V=4096, dtype="f32")
        kw.update(change)
        desc = L.make_desc(**kw)
        assert L.validate_desc(desc) == code, (change, L.validate_desc(desc))
        assert L.workspace_bytes(desc) == 0
    assert lib.lmhead_validate_desc(None) == -1
    # one K-step is a 128-byte line: 32 fp32 or 64 bf16 values
    assert L.validate_desc(L.make_desc(2, 4, 32, 96, 4096, "f32")) == 0
    assert L.validate_desc(L.make_desc(2, 4, 32, 48, 4096, "f32")) == -2
    assert L.validate_desc(L.make_desc(2, 4, 32, 96, 4096, "bf16")) == -2
    fp8 = L.make_desc(2, 4, 32, 256, 4096, "bf16", flags=4, fp8_exp_h=6, fp8_exp_w=12)
    plain = L.make_desc(2, 4, 32, 256, 4096, "bf16")
    assert L.validate_desc(fp8) == 0 and L.workspace_bytes(fp8) > L.workspace_bytes(plain)


def test_sizes_beyond_the_32_bit_tile_offsets_are_rejected(lib):
    # A 256-row operand tile is addressed with 32-bit byte offsets in a 2 GiB window, so every row pitch
    # must stay below 2^31 / 256 bytes; the widest rows are N (+ padding) or V (+ padding) elements.
    def code(P, T, V, dtype, d=64, **kw):
        return L.validate_desc(L.make_desc(P, 1, T, d, V, dtype, **kw))
    assert code(16383, 256, 1000, "bf16") == 0            # N + 64 = 4194112 < 4 Mi elements of 2 bytes
    assert code(16384, 256, 1000, "bf16") == -2           # N + 64 >= 4 Mi
    assert code(8191, 256, 1000, "f32") == 0
    assert code(8192, 256, 1000, "f32") == -2
    assert code(2, 8, 16383 * 256, "bf16") == 0           # V + padding
    assert code(2, 8, 16383 * 256 + 1, "bf16") == -2
    assert code(2, 8, 1000, "bf16", ldW=1 << 22) == -2    # the caller's own row stride counts too
    assert code(2, 8, 1000, "bf16", ldW=(1 << 22) - 8) == 0
    assert L.workspace_bytes(L.make_desc(16384, 1, 256, 64, 1000, "bf16")) == 0
    # the launch of a rejected size never happens: the compute entry points return the same code
    p = 0x10000
    bad = L.make_desc(16384, 1, 256, 64, 1000, "bf16")
    assert lib.lmhead_logprob_bwd(C.byref(bad), p, p, p, p, p, p, p, p, p, 1 << 45, None) == -2


def test_workspace_region_query(lib):
    desc = L.make_desc(3, 4, 100, 128, 5000, "bf16")
    total = L.workspace_bytes(desc)
    ncap = (3 * 4 * 100 + 255) // 256 * 256
    seen = []
    for which, nbytes in ((L.WS_NV, 4), (L.WS_ROW_SLOT, 4 * ncap), (L.WS_TOK_C, 4 * ncap), (L.WS_GATHERED_ID, 4 * ncap)):
        off, got = L.workspace_region(desc, 1, which)
        assert got == nbytes and off % 4 == 0 and off + got <= total
        seen.append((off, off + got))
    seen.sort()
    assert all(a[1] <= b[0] for a, b in zip(seen, seen[1:])), "regions do not overlap"
    off3, bytes3 = L.workspace_region(desc, 3, L.WS_GATHERED_ID)
    assert bytes3 == 3 * 4 * ncap and off3 + bytes3 <= L.multi_workspace_bytes(desc, 3)
    o, b = C.c_size_t(), C.c_size_t()
    q = lib.lmhead_workspace_region
    assert q(C.byref(desc), 1, 9, C.byref(o), C.byref(b)) == -2
    assert q(C.byref(desc), 0, 1, C.byref(o), C.byref(b)) == -2
    assert q(C.byref(desc), 1, 1, None, C.byref(b)) == -1
    assert q(C.byref(L.make_desc(3, 4, 100, 100, 5000, "bf16")), 1, 1, C.byref(o), C.byref(b)) == -2


def test_compute_entry_points_reject_bad_arguments_before_any_launch(lib):
    desc = L.make_desc(2, 4, 32, 256, 4096, "bf16")
    need = L.workspace_bytes(desc)
    p = 0x10000   # never dereferenced: every call below must fail in host-side validation
    d = C.byref(desc)
    fwd, bwd = lib.lmhead_logprob_fwd, lib.lmhead_logprob_bwd
    assert fwd(d, None, p, p, p, p, p, None, None, None, p, need, None) == -1
    assert fwd(d, p, p, p, p, None, p, None, None, None, p, need, None) == -1
    assert fwd(d, p, p, p, p, p, p, None, None, None, None, need, None) == -1
    assert fwd(d, p + 8, p, p, p, p, p, None, None, None, p, need, None) == -4
    assert fwd(d, p, p, p, p, p, p, None, None, None, p + 64, need, None) == -4
    assert fwd(d, p, p, p, p, p, p, None, None, None, p, need - 1, None) == -5
    assert bwd(d, p, p, p, p, None, p, p, p, p, need, None) == -1
    assert bwd(d, p, p, p, p, p, p, p + 4, p, p, need, None) == -4
    assert bwd(d, p, p, p, p, p, p, p, p, p, 0, None) == -5
    multi = lib.lmhead_logprob_fwd_multi
    vp3 = (C.c_void_p * 3)(p, p, p)
    need3 = L.multi_workspace_bytes(desc, 3)
    assert need3 > need and L.multi_workspace_bytes(desc, 1) == need
    assert L.multi_workspace_bytes(desc, 0) == 0 and L.multi_workspace_bytes(desc, 5) == 0
    assert multi(d, p, vp3, 5, p, p, vp3, None, None, None, None, p, need3, None) == -2
    assert multi(d, p, vp3, 3, p, p, vp3, None, None, None, None, p, need, None) == -5
    assert multi(d, p, (C.c_void_p * 3)(p, None, p), 3, p, p, vp3, None, None, None, None, p, need3, None) == -1
    assert multi(d, p, (C.c_void_p * 3)(p, p + 8, p), 3, p, p, vp3, None, None, None, None, p, need3, None) == -4
    assert multi(d, p, vp3, 3, p, p, None, None, None, None, None, p, need3, None) == -1
    bad = L.make_desc(2, 4, 32, 100, 4096, "bf16")
    assert fwd(C.byref(bad), p, p, p, p, p, p, None, None, None, p, 1 << 40, None) == -2
    assert lib.group_advantage(None, 2, 4, 1e-6, 0, p, None) == -1
    assert lib.group_advantage(p, 0, 4, 1e-6, 0, p, None) == -2
    assert lib.group_advantage(p, 2, 4, 1e-6, 2, p, None) == -2
    lws = L.loss_workspace_bytes(2, 4, 32)
    assert lws > 0 and L.loss_workspace_bytes(0, 4, 32) == 0
    g = lib.grpo_loss
    assert g(p, p, None, p, p, 2, 4, 32, 0.2, 0.2, 0.04, 0, None, p, None, p, lws, None) == -1
    assert g(p, p, None, p, p, 2, 4, 32, 0.2, 0.2, 0.04, 3, p, p, None, p, lws, None) == -2
    assert g(p, p, None, p, p, 2, 4, 32, 0.2, 0.2, 0.04, 0, p, p, None, p, lws - 1, None) == -5
    f = lib.flowrl_tb_loss
    assert f(p, None, p, p, p, 2, 4, 32, 1.0, p, p, None, None, p, lws, None) == -1
    assert f(p, p, p, p, p, 2, 4, -32, 1.0, p, p, None, None, p, lws, None) == -2
    assert f(p, p, p, p, p, 2, 4, 32, 1.0, p, p, None, None, p, 8, None) == -5
    c = lib.ce_loss
    assert c(p, None, 8, 32, p, p, p, lws, None) == -1
    assert c(p, p, 0, 32, p, p, p, lws, None) == -2
    assert c(p, p, 8, 32, p, p, p, 4, None) == -5
    assert lib.lmhead_check(None, None) == -1
    probe = lib.lmhead_probe_mfma
    assert probe(None, 1 << 20, p, 1 << 20, 4, 10, None) == -1
    assert probe(p, 1 << 20, p, 1 << 20, 0, 10, None) == -2
    assert probe(p, 1 << 20, p, 1 << 20, 4, 0, None) == -2
    assert probe(p + 4, 1 << 20, p, 1 << 20, 4, 10, None) == -4
    assert probe(p, 4 * 256 * 256 - 1, p, 1 << 20, 4, 10, None) == -5
    assert probe(p, 1 << 20, p, 4 * 256 * 4 - 1, 4, 10, None) == -5
    ms, n = C.c_double(), C.c_int64()
    assert lib.lmhead_timing_read(14, C.byref(ms), C.byref(n)) == -2
    assert lib.lmhead_timing_read(0, None, C.byref(n)) == -1


def test_dynakv_descriptor_and_argument_validation(lib):
    from paper_2603_04411_amd import dynakv as K
    assert C.sizeof(K.DynakvDesc) == 4 * 4 + 2 * 8 and K.DynakvDesc.ldx.offset == 16
    ok = L.make_kv_desc(1000, 512, "bf16")
    assert L.dynakv_validate_desc(ok) == 0
    need = L.dynakv_workspace_bytes(ok)
    assert need > 1000 * 512 * 4        # holds the fp32 gate logits
    cases = [
        (dict(n=0), -2), (dict(d=0), -2), (dict(d=100), -2), (dict(d=16384), -2), (dict(dtype=5), -3),
        (dict(flags=4), -3), (dict(ldx=256), -2), (dict(ldx=516), -4), (dict(n=1 << 22), -2),
    ]
    for change, code in cases:
        kw = dict(n=1000, d=512, dtype="bf16")
        kw.update(change)
        desc = L.make_kv_desc(**kw)
        assert L.dynakv_validate_desc(desc) == code, (change, L.dynakv_validate_desc(desc))
        assert L.dynakv_workspace_bytes(desc) == 0
    assert lib.dynakv_validate_desc(None) == -1
    p = 0x10000   # never dereferenced
    d = C.byref(ok)
    gate, store, rec, ret = lib.dynakv_gate, lib.dynakv_store, lib.dynakv_reconstruct, lib.dynakv_retain
    assert gate(d, None, p, p, p, 0.1, p, p, None, None, p, need, None) == -1
    assert gate(d, p, p, p, p, 0.1, p, None, None, None, p, need, None) == -1
    assert gate(d, p, p + 2, p, p, 0.1, p, p, None, None, p, need, None) == -4
    assert gate(d, p, p, p, p, 0.1, p, p, None, None, p + 16, need, None) == -4
    assert gate(d, p, p, p, p, 0.1, p, p, None, None, p, need - 1, None) == -5
    assert gate(d, p, p, p, p, 0.1, p, p, None, None, None, need, None) == -1
    assert store(d, p, p, 0, None, p, 1 << 20, p, need, None) == -1
    assert store(d, p, p, 0, p, p, -1, p, need, None) == -2
    assert store(d, p, p, 12, p, p, 1 << 20, p, need, None) == -2       # base offset not on a granule
    assert store(d, p, p, -8, p, p, 1 << 20, p, need, None) == -2
    assert store(d, p, p, 0, p + 4, p, 1 << 20, p, need, None) == -4
    assert rec(d, p, 1 << 20, p, p, None, p, p, need, None) == -1
    assert rec(d, p, 1 << 31, p, p, p, p, p, need, None) == -2       # more than 2^31 bytes of bf16
    assert rec(d, p, 1 << 20, p, p, p, p, p, 100, None) == -5
    assert ret(d, p, p, 0.5, None, None, p, need, None) == -1
    assert ret(d, p, p + 4, 0.5, p, None, p, need, None) == -4
    # the backward: a workspace of its own size, larger than the forward's
    bneed = L.dynakv_bwd_workspace_bytes(ok)
    assert bneed > need + 2 * 1000 * 512 * 2 and L.dynakv_bwd_workspace_bytes(L.make_kv_desc(1000, 100, "bf16")) == 0
    assert L.dynakv_validate_desc(L.make_kv_desc(1000, 512, "bf16", flags=L.FLAG_ACCUM_GRAD | L.FLAG_LITERAL_FLIP)) == 0
    bwd = lib.dynakv_gate_bwd
    bwd.argtypes = [C.c_void_p] * 8 + [C.c_float] + [C.c_void_p] * 5 + [C.c_size_t, C.c_void_p]
    bwd.restype = C.c_int
    assert bwd(d, p, p, p, p, p, None, None, 0.0, p, p, p, p, p, bneed, None) == -1
    assert bwd(d, p, p, p, p, p, p, None, 0.0, p, p, p, None, p, bneed, None) == -1
    assert bwd(d, p, p, p, p, p, p, p + 4, 0.0, p, p, p, p, p, bneed, None) == -4
    assert bwd(d, p, p, p, p, p, p, None, 0.0, p, p, p, p, p + 32, bneed, None) == -4
    assert bwd(d, p, p, p, p, p, p, None, 0.0, p, p, p, p, p, bneed - 1, None) == -5
    assert bwd(d, p, p, p, p, p, p, None, 0.0, p, p, p, p, p, need, None) == -5
    assert lib.dynakv_check(None, None) == -1


def test_workspace_grows_with_the_problem_and_default_chunk_is_bounded():
    small = L.workspace_bytes(L.make_desc(8, 8, 256, 2048, 151936, "bf16"))
    big = L.workspace_bytes(L.make_desc(32, 8, 2048, 4096, 151936, "bf16"))
    huge = L.workspace_bytes(L.make_desc(8, 16, 8192, 5120, 151936, "bf16"))
    assert small < big < huge < 100 * 2 ** 30          # sized for a 288 GB part, well below it
    narrow = L.workspace_bytes(L.make_desc(32, 8, 2048, 4096, 151936, "bf16", vocab_chunk=2048))
    assert narrow < big


def test_binding_has_no_cpu_fallback():
    import torch
    desc = L.make_desc(1, 1, 8, 64, 100, "bf16")
    t = torch.zeros(8, 64)
    with pytest.raises(ValueError):
        L.lmhead_logprob_fwd(desc, t, t, t, t, t, t, None, None, None, t)


def test_tile_walk_is_a_bijection(tmp_path):
    exe = tmp_path / "tile_map_check"
    src = os.path.join(ROOT, "tests", "host", "tile_map_check.cpp")
    subprocess.run(["g++", "-O2", "-o", str(exe), src], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "bad=0" in r.stdout
