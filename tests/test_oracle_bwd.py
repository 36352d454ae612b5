"""Pins for the oracle's backward (softmax Jacobian, dH, dW)."""
import numpy as np
import torch

from oracle import lmhead_oracle as O


def _case(seed, R=3, T=4, d=5, V=11):
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, T + 1, size=R)
    lens[0] = T
    H = rng.standard_normal((R * T, d))
    W = rng.standard_normal((V, d)) * 0.5
    tok = rng.integers(0, V, size=R * T)
    g = rng.standard_normal(R * T)
    mask, *_ = O.index_build(lens, T)
    return H, W, tok, lens, T, g * mask, mask


def _objective(H, W, tok, lens, T, g):
    lp, _, _ = O.lmhead_logprob_fwd(H, W, tok, lens, T)
    return float((g * lp).sum())


def test_central_differences_tiny():
    H, W, tok, lens, T, g, mask = _case(0)
    dH, dW = O.lmhead_logprob_bwd(H, W, tok, lens, T, g)
    h = 1e-6
    rng = np.random.default_rng(1)
    for _ in range(25):
        i, k = int(rng.integers(0, H.shape[0])), int(rng.integers(0, H.shape[1]))
        a = H.copy(); a[i, k] += h
        b = H.copy(); b[i, k] -= h
        fd = (_objective(a, W, tok, lens, T, g) - _objective(b, W, tok, lens, T, g)) / (2 * h)
        assert abs(fd - dH[i, k]) < 1e-7
    for _ in range(25):
        v, k = int(rng.integers(0, W.shape[0])), int(rng.integers(0, W.shape[1]))
        a = W.copy(); a[v, k] += h
        b = W.copy(); b[v, k] -= h
        fd = (_objective(H, a, tok, lens, T, g) - _objective(H, b, tok, lens, T, g)) / (2 * h)
        assert abs(fd - dW[v, k]) < 1e-7
    assert np.all(dH[mask == 0] == 0)


def test_cross_entropy_special_case_vs_autograd():
    # g = -1/N_v makes the objective the mean cross-entropy (L_CE): compare with torch autograd
    H, W, tok, lens, T, _, mask = _case(2, R=4, T=5, d=6, V=13)
    lp, _, _ = O.lmhead_logprob_fwd(H, W, tok, lens, T)
    loss, g = O.ce_loss(lp, lens, T)
    dH, dW = O.lmhead_logprob_bwd(H, W, tok, lens, T, g)
    Ht = torch.tensor(H, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    target = torch.from_numpy(np.where(mask == 1, tok, -100))
    L = torch.nn.functional.cross_entropy(Ht @ Wt.T, target, ignore_index=-100)
    L.backward()
    assert abs(L.item() - loss) < 1e-12
    assert np.allclose(Ht.grad.numpy(), dH, atol=1e-13)
    assert np.allclose(Wt.grad.numpy(), dW, atol=1e-13)


def test_gradient_identities():
    # sum_v dW[v,:] = 0 and <dW,W> = <dH,H> = sum_i g_i (logp_i + ent_i)
    H, W, tok, lens, T, g, mask = _case(3, R=5, T=6, d=7, V=29)
    dH, dW = O.lmhead_logprob_bwd(H, W, tok, lens, T, g, block=4)
    lp, _, ent = O.lmhead_logprob_fwd(H, W, tok, lens, T)
    assert np.allclose(dW.sum(axis=0), 0, atol=1e-12)
    s = float((g * (lp + ent)).sum())
    assert abs((dW * W).sum() - s) < 1e-11 and abs((dH * H).sum() - s) < 1e-11


def test_rows_routine_equals_full_on_subset():
    H, W, tok, lens, T, g, mask = _case(4)
    rows = np.nonzero(mask)[0]
    dH, dW = O.lmhead_logprob_bwd(H, W, tok, lens, T, g, block=3)
    dh, dw = O.bwd_rows(H[rows], W, tok[rows], g[rows])
    assert np.allclose(dH[rows], dh, atol=1e-14) and np.allclose(dW, dw, atol=1e-13)
