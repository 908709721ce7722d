"""Pins for oracle/tiled_linear_oracle.py: brute-force loops, closed forms, torch autograd."""
import numpy as np
import torch

from oracle import tiled_linear_oracle as orc


def test_brute_force_loops():
    g = np.random.default_rng(0)
    N, K, M = 4, 3, 5
    x, W, dy = g.standard_normal((N, K)), g.standard_normal((M, K)), g.standard_normal((N, M))
    y = np.zeros((N, M)); dx = np.zeros((N, K)); dW = np.zeros((M, K))
    for n in range(N):
        for m in range(M):
            for k in range(K):
                y[n, m] += x[n, k] * W[m, k]
                dx[n, k] += dy[n, m] * W[m, k]
                dW[m, k] += dy[n, m] * x[n, k]
    np.testing.assert_allclose(orc.forward(x, W), y, atol=1e-14)
    gx, gW = orc.backward(x, W, dy)
    np.testing.assert_allclose(gx, dx, atol=1e-14)
    np.testing.assert_allclose(gW, dW, atol=1e-14)


def test_closed_forms():
    g = np.random.default_rng(1)
    x = g.standard_normal((6, 4))
    assert (orc.forward(x, np.eye(4)) == x).all()                 # identity weight
    W = np.zeros((3, 4)); W[1, 2] = 2.0                           # one entry: y[:, 1] = 2 x[:, 2]
    y = orc.forward(x, W)
    assert (y[:, 1] == 2.0 * x[:, 2]).all() and (y[:, [0, 2]] == 0).all()
    dy = np.zeros((6, 3)); dy[4, 1] = 1.0                         # one upstream entry
    dx, dW = orc.backward(x, W, dy)
    assert (dx[4] == W[1]).all() and (np.delete(dx, 4, axis=0) == 0).all()
    assert (dW[1] == x[4]).all() and (dW[[0, 2]] == 0).all()


def test_against_torch_autograd_and_bf16_widening():
    g = np.random.default_rng(2)
    x, W, dy = g.standard_normal((33, 24)), g.standard_normal((40, 24)), g.standard_normal((33, 40))
    xt, Wt = torch.tensor(x, requires_grad=True), torch.tensor(W, requires_grad=True)
    y = torch.nn.functional.linear(xt, Wt)
    y.backward(torch.tensor(dy))
    np.testing.assert_allclose(orc.forward(x, W), y.detach().numpy(), atol=1e-12)
    dx, dW = orc.backward(x, W, dy)
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), atol=1e-12)
    bits = np.array([[0x3F80, 0xC000]], dtype=np.uint16)          # 1, -2
    assert (orc.forward(bits, np.array([[0x4000, 0x3F80]], dtype=np.uint16)) == [[0.0]]).all()
