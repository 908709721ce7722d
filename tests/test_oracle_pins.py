"""Pins for the CPU oracle: closed forms, finite differences, invariants and the library routine.

None of these checks re-types the oracle's own formula: each compares it with something fixed by
the mathematics (a closed form, a brute-force derivative, an invariance) or with torch's
cross_entropy under autograd on the CPU.
"""
import math

import numpy as np
import pytest
import torch

from oracle import tiled_ce_oracle as orc

IGN = -100


def _rand(N, H, V, seed, ignore=(), wscale=0.3):
    g = np.random.default_rng(seed)
    h = g.standard_normal((N, H))
    W = g.standard_normal((V, H)) * wscale
    y = g.integers(0, V, size=N).astype(np.int32)
    for i in ignore:
        y[i] = IGN
    return h, W, y


# ---- closed forms ----------------------------------------------------------------------------
@pytest.mark.parametrize("V", [4096, 128256, 152064])
def test_zero_hidden_gives_ln_v(V):
    N, H = 6, 4
    g = np.random.default_rng(1)
    W = g.standard_normal((V, H)) * 0.02
    y = g.integers(0, V, size=N).astype(np.int32)
    y[2] = IGN
    h = np.zeros((N, H))
    out = orc.forward(h, W, y)
    assert out["n_valid"] == 5
    assert abs(out["loss"] - math.log(V)) < 1e-12
    # printed values of ln V for the three vocabularies
    assert abs(math.log(4096) - 8.317766) < 1e-6 and abs(math.log(128256) - 11.761784) < 1e-6
    assert abs(math.log(152064) - 11.932057) < 1e-6
    dH, dW = orc.backward(h, W, y)
    assert np.abs(dW).max() == 0.0
    M = 5
    wbar = W.mean(axis=0)
    for i in range(N):
        exp = np.zeros(H) if y[i] == IGN else (wbar - W[y[i]]) / M
        np.testing.assert_allclose(dH[i], exp, rtol=0, atol=1e-15)


def test_zero_weight_closed_form():
    N, H, V = 9, 5, 17
    h, _, y = _rand(N, H, V, 2, ignore=(0, 4))
    W = np.zeros((V, H))
    out = orc.forward(h, W, y)
    assert abs(out["loss"] - math.log(V)) < 1e-14
    dH, dW = orc.backward(h, W, y, grad_loss=1.7)
    assert np.abs(dH).max() == 0.0
    M = 7
    exp = np.zeros((V, H))
    for i in range(N):
        if y[i] == IGN:
            continue
        exp += (1.0 / V) * h[i][None, :]
        exp[y[i]] -= h[i]
    np.testing.assert_allclose(dW, 1.7 * exp / M, rtol=0, atol=1e-14)


def test_scaled_identity_closed_form():
    V = H = 11
    c = 2.5
    y = np.array([3, 0, 10, 7, 3], dtype=np.int32)
    h = np.eye(V)[y]
    out = orc.forward(h, c * np.eye(V), y)
    assert abs(out["loss"] - (math.log(math.exp(c) + V - 1) - c)) < 1e-14


def test_single_class_and_logistic():
    h, W, _ = _rand(5, 3, 1, 3)
    y = np.zeros(5, dtype=np.int32)
    assert orc.forward(h, W, y)["loss"] == 0.0
    dH, dW = orc.backward(h, W, y)
    assert np.abs(dH).max() == 0.0 and np.abs(dW).max() == 0.0
    # two classes: per-token loss is softplus(z_other - z_label)
    h, W, y = _rand(7, 4, 2, 4)
    out = orc.forward(h, W, y)
    z = h @ W.T
    for i in range(7):
        d = z[i, 1 - y[i]] - z[i, y[i]]
        assert abs(out["loss_rows"][i] - math.log1p(math.exp(d))) < 1e-13


# ---- brute force -----------------------------------------------------------------------------
@pytest.mark.parametrize("N,H,V,ign", [(4, 3, 5, (1,)), (8, 16, 32, (0, 5, 7))])
def test_finite_differences(N, H, V, ign):
    h, W, y = _rand(N, H, V, 5, ignore=ign)
    g = 1.3
    dH, dW = orc.backward(h, W, y, grad_loss=g)
    eps = 1e-6

    def L(hh, WW):
        return g * orc.forward(hh, WW, y)["loss"]

    for i in range(N):
        for k in range(H):
            hp, hm = h.copy(), h.copy()
            hp[i, k] += eps
            hm[i, k] -= eps
            fd = (L(hp, W) - L(hm, W)) / (2 * eps)
            assert abs(fd - dH[i, k]) < 2e-8, (i, k)
    for v in range(V):
        for k in range(H):
            Wp, Wm = W.copy(), W.copy()
            Wp[v, k] += eps
            Wm[v, k] -= eps
            fd = (L(h, Wp) - L(h, Wm)) / (2 * eps)
            assert abs(fd - dW[v, k]) < 2e-8, (v, k)


# ---- invariants ------------------------------------------------------------------------------
def test_dlogits_sum_to_zero_columns_of_dw_vanish():
    # sum_v dz[i, v] = 0 for every row  =>  sum_v dW[v, k] = sum_i (sum_v dz[i, v]) h[i, k] = 0
    h, W, y = _rand(37, 8, 29, 6, ignore=(3, 30))
    dH, dW = orc.backward(h, W, y)
    assert np.abs(dW.sum(axis=0)).max() < 1e-15
    # and with W = a single repeated row u, dH[i] = (sum_v dz[i, v]) u = 0
    Wc = np.tile(W[:1], (29, 1))
    dHc, _ = orc.backward(h, Wc, y)
    assert np.abs(dHc).max() < 1e-15


def test_ignored_rows_contribute_nothing():
    h, W, y = _rand(12, 6, 19, 7, ignore=(2, 3, 11))
    out = orc.forward(h, W, y)
    dH, dW = orc.backward(h, W, y)
    for i in (2, 3, 11):
        assert (dH[i] == 0.0).all() and out["loss_rows"][i] == 0.0
    h2 = h.copy()
    h2[[2, 3, 11]] = np.random.default_rng(8).standard_normal((3, 6)) * 50
    out2 = orc.forward(h2, W, y)
    dH2, dW2 = orc.backward(h2, W, y)
    assert out2["loss"] == out["loss"]
    assert (dW2 == dW).all()
    # dropping the ignored rows altogether gives the same loss and dW
    keep = np.array([i for i in range(12) if i not in (2, 3, 11)])
    out3 = orc.forward(h[keep], W, y[keep])
    _, dW3 = orc.backward(h[keep], W, y[keep])
    assert abs(out3["loss"] - out["loss"]) < 1e-14
    np.testing.assert_allclose(dW3, dW, rtol=0, atol=1e-15)


def test_loss_bit_identical_across_row_blocks():
    h, W, y = _rand(130, 12, 40, 9, ignore=(0, 64, 129))
    ref = orc.forward(h, W, y, row_block=None, ordered=True)
    for rb in (1, 7, 128, 130):
        o = orc.forward(h, W, y, row_block=rb, ordered=True)
        assert o["loss"] == ref["loss"]
        assert (o["lse"] == ref["lse"]).all()
    # the BLAS contraction may round differently per blocking, but only in the last bits
    for rb in (1, 7, 128):
        o = orc.forward(h, W, y, row_block=rb)
        assert abs(o["loss"] - ref["loss"]) < 1e-13
    dH0, dW0 = orc.backward(h, W, y)
    dH1, dW1 = orc.backward(h, W, y, row_block=7)
    np.testing.assert_allclose(dH1, dH0, rtol=0, atol=1e-15)
    np.testing.assert_allclose(dW1, dW0, rtol=0, atol=1e-15)


def test_shift_of_every_weight_row_changes_nothing():
    h, W, y = _rand(10, 5, 13, 10, ignore=(4,))
    c = np.random.default_rng(11).standard_normal(5)
    o0, o1 = orc.forward(h, W, y), orc.forward(h, W + c, y)
    assert abs(o0["loss"] - o1["loss"]) < 1e-13
    g0, g1 = orc.backward(h, W, y), orc.backward(h, W + c, y)
    np.testing.assert_allclose(g1[0], g0[0], rtol=0, atol=1e-14)
    np.testing.assert_allclose(g1[1], g0[1], rtol=0, atol=1e-14)


def test_permutations():
    h, W, y = _rand(14, 6, 21, 12, ignore=(1, 9))
    g = np.random.default_rng(13)
    pt = g.permutation(14)
    o0, (dH0, dW0) = orc.forward(h, W, y), orc.backward(h, W, y)
    o1, (dH1, dW1) = orc.forward(h[pt], W, y[pt]), orc.backward(h[pt], W, y[pt])
    assert abs(o0["loss"] - o1["loss"]) < 1e-14
    np.testing.assert_allclose(dH1, dH0[pt], rtol=0, atol=1e-15)
    np.testing.assert_allclose(dW1, dW0, rtol=0, atol=1e-15)
    pv = g.permutation(21)              # new id j holds old row pv[j]
    inv = np.argsort(pv)
    y2 = np.where(y == IGN, IGN, inv[np.clip(y, 0, 20)]).astype(np.int32)
    o2, (dH2, dW2) = orc.forward(h, W[pv], y2), orc.backward(h, W[pv], y2)
    assert abs(o0["loss"] - o2["loss"]) < 1e-14
    np.testing.assert_allclose(dH2, dH0, rtol=0, atol=1e-15)
    np.testing.assert_allclose(dW2, dW0[pv], rtol=0, atol=1e-15)


def test_linear_in_upstream_gradient():
    h, W, y = _rand(9, 4, 15, 14, ignore=(8,))
    a, b = orc.backward(h, W, y, grad_loss=1.0), orc.backward(h, W, y, grad_loss=2.0)
    assert (b[0] == 2.0 * a[0]).all() and (b[1] == 2.0 * a[1]).all()


def test_all_ignored_and_bad_label():
    h, W, _ = _rand(5, 4, 9, 15)
    y = np.full(5, IGN, dtype=np.int32)
    o = orc.forward(h, W, y)
    assert o["loss"] == 0.0 and o["n_valid"] == 0
    dH, dW = orc.backward(h, W, y)
    assert np.abs(dH).max() == 0.0 and np.abs(dW).max() == 0.0
    y[1] = 9
    with pytest.raises(ValueError):
        orc.forward(h, W, y)
    y[1] = -1
    with pytest.raises(ValueError):
        orc.backward(h, W, y)


def test_mean_is_global_not_mean_of_tile_means():
    # two "tiles" with different numbers of valid tokens: the loss is sum / global count
    h, W, y = _rand(8, 4, 7, 16, ignore=(0, 1, 2))
    o = orc.forward(h, W, y, row_block=4)
    a, b = orc.forward(h[:4], W, y[:4]), orc.forward(h[4:], W, y[4:])
    glob = (a["loss"] * a["n_valid"] + b["loss"] * b["n_valid"]) / 5
    assert abs(o["loss"] - glob) < 1e-14
    assert abs(o["loss"] - 0.5 * (a["loss"] + b["loss"])) > 1e-3


# ---- the library routine ---------------------------------------------------------------------
@pytest.mark.parametrize("N,H,V,seed", [(64, 32, 257, 20), (33, 24, 100, 21), (512, 256, 4096, 22)])
def test_against_torch_cross_entropy_autograd(N, H, V, seed):
    g = np.random.default_rng(seed)
    h = g.standard_normal((N, H))
    W = g.standard_normal((V, H)) * (0.02 if V == 4096 else 0.4)
    y = g.integers(0, V, size=N).astype(np.int32)
    y[g.random(N) < 0.1] = IGN
    ht = torch.tensor(h, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    loss = torch.nn.functional.cross_entropy(
        torch.nn.functional.linear(ht, Wt), torch.tensor(y, dtype=torch.long),
        ignore_index=IGN, reduction="mean")
    (1.5 * loss).backward()
    o = orc.forward(h, W, y, row_block=50)
    dH, dW = orc.backward(h, W, y, grad_loss=1.5, row_block=50)
    assert abs(o["loss"] - loss.item()) < 1e-12 * max(1.0, abs(loss.item()))
    np.testing.assert_allclose(dH, ht.grad.numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(
        o["lse"], torch.logsumexp(torch.nn.functional.linear(ht, Wt), dim=1).detach().numpy(),
        rtol=0, atol=1e-12)


# ---- the sampled forms equal the full forms ----------------------------------------------------
def test_sampled_rows_equal_full():
    h, W, y = _rand(40, 8, 50, 30, ignore=(0, 17, 39))
    full = orc.forward(h, W, y)
    dH, dW = orc.backward(h, W, y, grad_loss=0.7)
    rows = np.array([0, 1, 17, 38, 39])
    dHr, lse_r, lr = orc.dhidden_rows(h, W, y, rows, full["n_valid"], grad_loss=0.7)
    np.testing.assert_allclose(dHr, dH[rows], rtol=0, atol=1e-15)
    np.testing.assert_allclose(lse_r, full["lse"][rows], rtol=0, atol=1e-13)
    np.testing.assert_allclose(lr, full["loss_rows"][rows], rtol=0, atol=1e-13)
    ids = np.array([0, 49, int(y[1]), 7])
    dWr = orc.dw_rows(h, W, y, full["lse"], ids, grad_loss=0.7, row_block=16)
    np.testing.assert_allclose(dWr, dW[ids], rtol=0, atol=1e-15)


def test_bf16_widening_is_exact():
    bits = np.array([0x0000, 0x3F80, 0xBF80, 0x4049, 0x3C00, 0x0080, 0x8001], dtype=np.uint16)
    v = orc.bf16_bits_to_f64(bits)
    exp = [0.0, 1.0, -1.0, 3.140625, 2.0 ** -7, 2.0 ** -126, -(2.0 ** -133)]
    assert v.tolist() == exp
    t = torch.tensor(bits.astype(np.int16)).view(torch.bfloat16).double().numpy()
    assert (t == v).all()


def test_sum_and_unreduced_losses_against_torch():
    """reduction='sum' and the unreduced token losses against the library routine."""
    g = np.random.default_rng(31)
    N, H, V = 40, 16, 50
    h = g.standard_normal((N, H))
    W = g.standard_normal((V, H)) * 0.4
    y = g.integers(0, V, N).astype(np.int64)
    y[[3, 17, 18]] = IGN
    f = orc.forward(h, W, y, reduction="sum")
    ht = torch.tensor(h, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    z = torch.nn.functional.linear(ht, Wt)
    none = torch.nn.functional.cross_entropy(z, torch.tensor(y), ignore_index=IGN, reduction="none")
    tot = torch.nn.functional.cross_entropy(z, torch.tensor(y), ignore_index=IGN, reduction="sum")
    np.testing.assert_allclose(f["loss_rows"], none.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(f["loss"], float(tot.detach()), rtol=1e-13)
    (1.5 * tot).backward()
    dH, dW = orc.backward(h, W, y, grad_loss=1.5, reduction="sum")
    np.testing.assert_allclose(dH, ht.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), rtol=0, atol=1e-12)
    # the sum is M times the mean, for the loss and for both gradients
    fm = orc.forward(h, W, y)
    M = fm["n_valid"]
    assert abs(f["loss"] - M * fm["loss"]) <= 1e-12 * abs(f["loss"])
    dHm, dWm = orc.backward(h, W, y, grad_loss=1.5)
    np.testing.assert_allclose(dH, M * dHm, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(dW, M * dWm, rtol=1e-12, atol=1e-15)
