"""The seeded input generators: determinism, storage rounding, and the stated distributions."""
import numpy as np
import torch

import workloads as wl


def test_bf16_rounding_is_rne_and_widening_exact():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))).astype(np.float32)
    bits = wl.bf16_bits_from_f32(x)
    ref = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(wl.f32_from_bf16_bits(bits), ref.float().numpy())
    # exact ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert wl.bf16_bits_from_f32(np.array([1.0 + 2.0 ** -8], np.float32))[0] == 0x3F80
    assert wl.bf16_bits_from_f32(np.array([1.0 + 3 * 2.0 ** -8], np.float32))[0] == 0x3F82


def test_blocks_regenerate_independently():
    c = wl.CONFIGS[1].scaled(P=2, G=2, T=300, d=64, V=1000)
    H = wl.hidden(c)
    assert H.shape == (c.N, 64) and H.dtype == np.uint16
    rows = [0, 255, 256, 700, c.N - 1]
    assert np.array_equal(wl.matrix_rows(c, wl.STREAM_H, rows), H[rows])
    assert np.array_equal(wl.hidden(c, threads=1), H)
    W, Wo = wl.weight(c), wl.weight(c, "old")
    assert W.shape == (1000, 64) and not np.array_equal(W, Wo)
    Wp = wl.perturbed_weight(c, W)
    d = wl.as_f64(Wp) - wl.as_f64(W)
    assert 0 < np.abs(d).max() < 0.02


def test_distributions():
    c = wl.CONFIGS[1]
    ln = wl.lengths(c)
    assert ln.dtype == np.int32 and ln.min() >= 64 and ln.max() <= 256 and ln.size == 64
    r = wl.rewards(c)
    assert set(np.unique(r)) <= {0.0, 1.0}
    tok = wl.tokens(c)
    assert tok.dtype == np.int32 and tok.min() >= 0 and tok.max() < c.V
    # finite Zipf(1.1): P(id 0) = 1 / sum_k k^-1.1
    p0 = 1.0 / (np.arange(1, c.V + 1, dtype=np.float64) ** -1.1).sum()
    assert abs((tok == 0).mean() - p0) < 0.02
    H = wl.as_f64(wl.matrix_rows(c, wl.STREAM_H, np.arange(512)))
    assert abs(H.std() - 1) < 0.02 and abs(H.mean()) < 0.01
    W = wl.as_f64(wl.matrix_rows(c, wl.STREAM_W, np.arange(512)))
    assert abs(W.std() - 0.02) < 0.001
    c3 = wl.CONFIGS[3]
    l3 = wl.lengths(c3)
    assert l3.min() >= 32 and l3.max() <= 4096 and np.median(l3) < 1200   # log-uniform is bottom-heavy
    assert wl.log_z(c3).shape == (16,) and np.all(wl.log_z(wl.CONFIGS[0]) == 0)
    r3 = wl.rewards(c3)
    assert r3.min() >= 0 and r3.max() < 1 and len(np.unique(r3)) > 100
    assert wl.CONFIGS[2].len_lo == 512 and wl.CONFIGS[2].len_hi == 2048


def test_row_subset():
    c = wl.CONFIGS[1]
    ln, tok = wl.lengths(c), wl.tokens(c)
    s = wl.sample_valid_rows(c, ln, tok, 512)
    assert s.size == 512 and np.all(np.diff(s) > 0)
    assert np.all((s % c.T) < ln[s // c.T])
    assert np.array_equal(s, wl.sample_valid_rows(c, ln, tok, 512))
