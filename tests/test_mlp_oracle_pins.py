"""Pins for oracle/tiled_mlp_oracle.py: closed forms, finite differences, invariants and torch
autograd of the same expression.  CPU only.  Each pin is chosen so that a plausible mistake (a
dropped term of silu', a transposed weight, u and g swapped, a missing factor) fails it."""
import numpy as np
import pytest
import torch

from oracle import tiled_mlp_oracle as orc


def _rand(N, H, I, seed, scale=0.5):
    g = np.random.default_rng(seed)
    x = g.standard_normal((N, H))
    Wg = g.standard_normal((I, H)) * scale
    Wu = g.standard_normal((I, H)) * scale
    Wd = g.standard_normal((H, I)) * scale
    dy = g.standard_normal((N, H))
    return x, Wg, Wu, Wd, dy


def test_silu_closed_forms():
    z = np.array([0.0, 1.0, -1.0, 30.0, -30.0, 745.0, -745.0])
    s = orc.silu(z)
    assert s[0] == 0.0
    assert abs(s[1] - 1.0 / (1.0 + np.exp(-1.0))) < 1e-15
    assert abs(s[2] + 1.0 / (1.0 + np.exp(1.0))) < 1e-15
    assert abs(s[3] - 30.0) < 1e-11 and abs(s[4]) < 1e-11
    assert np.isfinite(s).all() and s[5] == 745.0 and abs(s[6]) < 1e-300
    # silu(z) - silu(-z) = z  (from sigmoid(z) + sigmoid(-z) = 1)
    zz = np.linspace(-8, 8, 101)
    np.testing.assert_allclose(orc.silu(zz) - orc.silu(-zz), zz, atol=1e-14)
    # derivative: 1/2 at 0, and against a central difference
    assert orc.silu_grad(np.array([0.0]))[0] == 0.5
    e = 1e-6
    np.testing.assert_allclose(orc.silu_grad(zz), (orc.silu(zz + e) - orc.silu(zz - e)) / (2 * e),
                               atol=1e-9)


def test_single_unit_closed_form():
    # N = H = I = 1: y = silu(x wg) * (x wu) * wd
    x, wg, wu, wd, dy = 0.7, -1.3, 0.9, 2.0, 0.4
    y = orc.forward(np.array([[x]]), np.array([[wg]]), np.array([[wu]]), np.array([[wd]]))
    g, u = x * wg, x * wu
    sig = 1.0 / (1.0 + np.exp(-g))
    assert abs(y[0, 0] - g * sig * u * wd) < 1e-15
    dx, dWg, dWu, dWd = orc.backward(np.array([[x]]), np.array([[wg]]), np.array([[wu]]),
                                     np.array([[wd]]), np.array([[dy]]))
    da = dy * wd
    dsilu = sig * (1 + g * (1 - sig))
    assert abs(dWd[0, 0] - dy * g * sig * u) < 1e-15
    assert abs(dWg[0, 0] - da * u * dsilu * x) < 1e-15
    assert abs(dWu[0, 0] - da * g * sig * x) < 1e-15
    assert abs(dx[0, 0] - (da * u * dsilu * wg + da * g * sig * wu)) < 1e-15


def test_zero_input_and_zero_weights():
    x, Wg, Wu, Wd, dy = _rand(6, 5, 7, 1)
    # x = 0: g = u = 0, a = 0, y = 0; dg = da * 0 * 1/2 = 0, du = da * 0 = 0 -> every gradient is 0
    z = np.zeros_like(x)
    assert (orc.forward(z, Wg, Wu, Wd) == 0).all()
    for t in orc.backward(z, Wg, Wu, Wd, dy):
        assert (t == 0).all()
    # Wu = 0: y = 0, dWd = 0, dx = du Wu + dg Wg = 0 (dg has the factor u = 0), dWg = 0,
    # dWu = (da * silu(g))^T x is NOT zero
    y = orc.forward(x, Wg, np.zeros_like(Wu), Wd)
    dx, dWg, dWu, dWd = orc.backward(x, Wg, np.zeros_like(Wu), Wd, dy)
    assert (y == 0).all() and (dWd == 0).all() and (dx == 0).all() and (dWg == 0).all()
    ref = ((dy @ Wd) * orc.silu(x @ Wg.T)).T @ x
    np.testing.assert_allclose(dWu, ref, atol=1e-13)
    assert np.abs(dWu).max() > 1e-3


def test_gate_saturation_limits():
    # a very positive gate makes silu the identity: y = (g * u) Wd^T; a very negative one kills it
    g0 = np.random.default_rng(2)
    x = np.abs(g0.standard_normal((4, 3))) + 0.5
    Wg = np.full((5, 3), 40.0)
    Wu = g0.standard_normal((5, 3))
    Wd = g0.standard_normal((3, 5))
    y = orc.forward(x, Wg, Wu, Wd)
    np.testing.assert_allclose(y, ((x @ Wg.T) * (x @ Wu.T)) @ Wd.T, rtol=1e-12)
    assert np.abs(orc.forward(x, -Wg, Wu, Wd)).max() < 1e-20


@pytest.mark.parametrize("N,H,I", [(3, 4, 5), (7, 6, 9)])
def test_finite_differences(N, H, I):
    x, Wg, Wu, Wd, dy = _rand(N, H, I, 3)
    dx, dWg, dWu, dWd = orc.backward(x, Wg, Wu, Wd, dy)

    def L(x_, Wg_, Wu_, Wd_):
        return float((orc.forward(x_, Wg_, Wu_, Wd_) * dy).sum())

    e = 1e-6
    for arr, grad, which in ((x, dx, 0), (Wg, dWg, 1), (Wu, dWu, 2), (Wd, dWd, 3)):
        num = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            args = [x.copy(), Wg.copy(), Wu.copy(), Wd.copy()]
            args[which][idx] += e
            up = L(*args)
            args[which][idx] -= 2 * e
            num[idx] = (up - L(*args)) / (2 * e)
        np.testing.assert_allclose(grad, num, rtol=1e-6, atol=1e-8)


@pytest.mark.parametrize("N,H,I,seed", [(33, 24, 40, 5), (64, 32, 96, 6)])
def test_against_torch_autograd(N, H, I, seed):
    x, Wg, Wu, Wd, dy = _rand(N, H, I, seed)
    t = [torch.tensor(a, requires_grad=True) for a in (x, Wg, Wu, Wd)]
    F = torch.nn.functional
    y = F.linear(F.silu(F.linear(t[0], t[1])) * F.linear(t[0], t[2]), t[3])
    y.backward(torch.tensor(dy))
    np.testing.assert_allclose(orc.forward(x, Wg, Wu, Wd), y.detach().numpy(), rtol=0, atol=1e-12)
    for got, ref in zip(orc.backward(x, Wg, Wu, Wd, dy), t):
        np.testing.assert_allclose(got, ref.grad.numpy(), rtol=0, atol=1e-11)


def test_tiling_and_row_invariants():
    x, Wg, Wu, Wd, dy = _rand(37, 8, 12, 7)
    y = orc.forward(x, Wg, Wu, Wd)
    full = orc.backward(x, Wg, Wu, Wd, dy)
    for rb in (1, 5, 16, 37):
        # rows are independent: nothing depends on the row blocking (up to the summation order
        # inside the library matmul)
        np.testing.assert_allclose(orc.forward(x, Wg, Wu, Wd, row_block=rb), y, rtol=1e-12, atol=1e-13)
        part = orc.backward(x, Wg, Wu, Wd, dy, row_block=rb)
        for a, b in zip(part, full):
            np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    # permuting tokens permutes y and dx and leaves the weight gradients unchanged
    p = np.random.default_rng(8).permutation(37)
    np.testing.assert_allclose(orc.forward(x[p], Wg, Wu, Wd), y[p], rtol=1e-12, atol=1e-13)
    perm = orc.backward(x[p], Wg, Wu, Wd, dy[p])
    np.testing.assert_allclose(perm[0], full[0][p], rtol=1e-12, atol=1e-13)
    for a, b in zip(perm[1:], full[1:]):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    # linear in dy
    twice = orc.backward(x, Wg, Wu, Wd, 2.0 * dy)
    for a, b in zip(twice, full):
        np.testing.assert_allclose(a, 2.0 * b, rtol=1e-13, atol=0)
    # a row with dy = 0 contributes nothing to any weight gradient and has dx = 0
    dy0 = dy.copy()
    dy0[11] = 0
    z = orc.backward(x, Wg, Wu, Wd, dy0)
    x2 = x.copy()
    x2[11] += 3.0
    z2 = orc.backward(x2, Wg, Wu, Wd, dy0)
    assert (z[0][11] == 0).all()
    for a, b in zip(z[1:], z2[1:]):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)


def test_sampled_entries_equal_full():
    x, Wg, Wu, Wd, dy = _rand(50, 10, 14, 9)
    y = orc.forward(x, Wg, Wu, Wd)
    dx, dWg, dWu, dWd = orc.backward(x, Wg, Wu, Wd, dy)
    rows = np.array([0, 7, 49, 23])
    np.testing.assert_allclose(orc.forward_rows(x, Wg, Wu, Wd, rows), y[rows], atol=1e-13)
    np.testing.assert_allclose(orc.dx_rows(x, Wg, Wu, Wd, dy, rows), dx[rows], atol=1e-12)
    cols = np.array([0, 13, 5])
    np.testing.assert_allclose(orc.dwd_columns(x, Wg, Wu, dy, cols, row_block=16), dWd[:, cols], atol=1e-12)
    og, ou = orc.dwgu_rows(x, Wg, Wu, Wd, dy, cols, row_block=16)
    np.testing.assert_allclose(og, dWg[cols], atol=1e-12)
    np.testing.assert_allclose(ou, dWu[cols], atol=1e-12)


def test_bf16_inputs_are_widened_exactly():
    bits = np.array([[0x3F80, 0xBF80, 0x0000, 0x4000]], dtype=np.uint16)     # 1, -1, 0, 2
    np.testing.assert_array_equal(orc.bf16_bits_to_f64(bits), [[1.0, -1.0, 0.0, 2.0]])
    Wg = np.array([[0x3F80, 0, 0, 0]], dtype=np.uint16)       # g = x0 = 1
    Wu = np.array([[0, 0, 0, 0x3F80]], dtype=np.uint16)       # u = x3 = 2
    Wd = np.array([[0x3F80]] * 4, dtype=np.uint16)
    y = orc.forward(bits, Wg, Wu, Wd)
    np.testing.assert_allclose(y, np.full((1, 4), 2.0 / (1.0 + np.exp(-1.0))), rtol=1e-15)
