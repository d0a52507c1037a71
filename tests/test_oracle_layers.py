"""Pins for oracle/layers.py: hand cases, library routines (torch CPU fp64), adjoint identities."""
import numpy as np
import torch

from oracle import layers as ly


def test_fc_hand_case():
    X = np.array([[1.0, 2.0, 3.0], [-1.0, 0.5, 0.0]])
    W = np.array([[1.0, -1.0], [0.0, 2.0], [2.0, 1.0]])
    # by hand: row0 = [1+0+6, -1+4+3] = [7, 6]; row1 = [-1, 1+1] = [-1, 2]
    assert np.array_equal(ly.fc_forward(X, W, False), np.array([[7.0, 6.0], [-1.0, 2.0]]))
    Y = ly.fc_forward(X, W, True)
    assert np.array_equal(Y, np.array([[7.0, 6.0], [0.0, 2.0]]))
    dY = np.array([[1.0, 1.0], [10.0, 100.0]])
    dX, dW = ly.fc_backward(dY, X, W, Y, True)
    G = np.array([[1.0, 1.0], [0.0, 100.0]])                  # gradient blocked where Y == 0
    assert np.array_equal(dX, np.array([[0.0, 2.0, 3.0], [-100.0, 200.0, 100.0]]))
    assert np.array_equal(dW, X.T @ G)
    assert np.array_equal(dW, np.array([[1.0, -99.0], [2.0, 52.0], [3.0, 3.0]]))


def test_fc_identity_and_onehot():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((5, 7))
    assert np.array_equal(ly.fc_forward(X, np.eye(7), False), X)
    W = rng.standard_normal((7, 4))
    E = np.zeros((1, 7)); E[0, 3] = 1.0
    assert np.array_equal(ly.fc_forward(E, W, False)[0], W[3])      # W[i, j]: neuron i -> neuron j (Sec. 2.1)


def test_fc_against_torch_autograd():
    rng = np.random.default_rng(1)
    X, W, dY = rng.standard_normal((6, 9)), rng.standard_normal((9, 5)), rng.standard_normal((6, 5))
    xt = torch.tensor(X, requires_grad=True); wt = torch.tensor(W, requires_grad=True)
    yt = torch.relu(xt @ wt)
    yt.backward(torch.tensor(dY))
    Y = ly.fc_forward(X, W, True)
    dX, dW = ly.fc_backward(dY, X, W, Y, True)
    np.testing.assert_allclose(Y, yt.detach().numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dX, xt.grad.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dW, wt.grad.numpy(), rtol=0, atol=1e-13)


def test_abs_product():
    A = np.array([[1.0, -2.0]]); B = np.array([[3.0], [-4.0]])
    assert ly.abs_product(A, B)[0, 0] == 11.0


def test_conv_against_torch():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((3, 4, 6, 5)); W = rng.standard_normal((7, 4, 3, 3)); pad = 1
    Y = ly.conv_forward(X, W, pad)
    xt = torch.tensor(X, requires_grad=True); wt = torch.tensor(W, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt, padding=pad)
    np.testing.assert_allclose(Y, yt.detach().numpy(), rtol=0, atol=1e-12)
    dY = rng.standard_normal(Y.shape)
    yt.backward(torch.tensor(dY))
    np.testing.assert_allclose(ly.conv_dgrad(dY, W, pad, 6, 5), xt.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(ly.conv_wgrad(X, dY, pad, 3, 3), wt.grad.numpy(), rtol=0, atol=1e-12)


def test_conv_no_pad_and_1x1_reduces_to_fc():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((2, 3, 5, 5)); W = rng.standard_normal((4, 3, 3, 3))
    yt = torch.nn.functional.conv2d(torch.tensor(X), torch.tensor(W), padding=0)
    np.testing.assert_allclose(ly.conv_forward(X, W, 0), yt.numpy(), rtol=0, atol=1e-12)
    X1 = rng.standard_normal((5, 6, 1, 1)); W1 = rng.standard_normal((4, 6, 1, 1))
    np.testing.assert_allclose(ly.conv_forward(X1, W1, 0)[:, :, 0, 0], X1[:, :, 0, 0] @ W1[:, :, 0, 0].T, atol=1e-13)


def test_conv_adjoint_identities():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((2, 3, 5, 4)); W = rng.standard_normal((5, 3, 3, 3)); pad = 1
    Y = ly.conv_forward(X, W, pad)
    dY = rng.standard_normal(Y.shape)
    lhs = np.sum(dY * Y)
    assert abs(lhs - np.sum(ly.conv_dgrad(dY, W, pad, 5, 4) * X)) < 1e-10
    assert abs(lhs - np.sum(ly.conv_wgrad(X, dY, pad, 3, 3) * W)) < 1e-10


def test_conv_point_matches_full():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((2, 3, 5, 4)); W = rng.standard_normal((5, 3, 3, 3))
    Y = ly.conv_forward(X, W, 1)
    for (n, k, y, x) in [(0, 0, 0, 0), (1, 4, 4, 3), (0, 2, 2, 1), (1, 1, 0, 3)]:
        v, mag = ly.conv_forward_point(X, W, 1, n, k, y, x)
        assert abs(v - Y[n, k, y, x]) < 1e-12 and mag >= abs(v)


# ---- the same operators as plain nested loops (oracle/layers_plain.c): the definitions written out; the numpy forms
# above must agree with them up to the order of the fp64 additions

def test_plain_loops_hand_case_and_orientation():
    from oracle import layers_plain as lp
    X = np.array([[1.0, 2.0, 3.0], [-1.0, 0.5, 0.0]])
    W = np.array([[1.0, -1.0], [0.0, 2.0], [2.0, 1.0]])
    assert np.array_equal(lp.fc_forward(X, W, False), np.array([[7.0, 6.0], [-1.0, 2.0]]))     # by hand, as above
    Y = lp.fc_forward(X, W, True)
    assert np.array_equal(Y, np.array([[7.0, 6.0], [0.0, 2.0]]))
    dX, dW = lp.fc_backward(np.array([[1.0, 1.0], [10.0, 100.0]]), X, W, Y, True)
    assert np.array_equal(dX, np.array([[0.0, 2.0, 3.0], [-100.0, 200.0, 100.0]]))
    assert np.array_equal(dW, np.array([[1.0, -99.0], [2.0, 52.0], [3.0, 3.0]]))
    # a filter with a single 1 at tap (r, s) of channel pair (ko, c) shifts channel c of the image into channel ko
    Xi = np.arange(2 * 2 * 3 * 4, dtype=np.float64).reshape(2, 2, 3, 4)
    Wt = np.zeros((3, 2, 3, 3)); Wt[2, 1, 0, 2] = 1.0          # reads X[n, 1, y + 0 - 1, x + 2 - 1]
    Yc = lp.conv_forward(Xi, Wt, 1)
    want = np.zeros((2, 3, 3, 4)); want[:, 2, 1:, :3] = Xi[:, 1, :2, 1:]
    assert np.array_equal(Yc, want)


def test_numpy_forms_agree_with_the_plain_loops():
    from oracle import layers_plain as lp
    rng = np.random.default_rng(11)
    for (b, ni, no, relu) in [(5, 7, 3, False), (9, 33, 17, True), (16, 64, 40, True)]:
        X, W, dY = rng.standard_normal((b, ni)), rng.standard_normal((ni, no)), rng.standard_normal((b, no))
        Y = ly.fc_forward(X, W, relu)
        np.testing.assert_allclose(Y, lp.fc_forward(X, W, relu), rtol=0, atol=1e-12)
        dX, dW = ly.fc_backward(dY, X, W, Y, relu)
        pX, pW = lp.fc_backward(dY, X, W, Y, relu)
        np.testing.assert_allclose(dX, pX, rtol=0, atol=1e-12)
        np.testing.assert_allclose(dW, pW, rtol=0, atol=1e-12)
    for (N, C, K, H, Wd, R, S, pad) in [(2, 3, 4, 5, 6, 3, 3, 1), (3, 2, 5, 4, 4, 1, 1, 0), (2, 4, 3, 7, 5, 5, 3, 2),
                                        (1, 2, 2, 6, 6, 3, 3, 0)]:
        X, W = rng.standard_normal((N, C, H, Wd)), rng.standard_normal((K, C, R, S))
        Y = ly.conv_forward(X, W, pad)
        np.testing.assert_allclose(Y, lp.conv_forward(X, W, pad), rtol=0, atol=1e-12)
        dY = rng.standard_normal(Y.shape)
        if R == S:      # the numpy data gradient takes one padding for both image dimensions
            np.testing.assert_allclose(ly.conv_dgrad(dY, W, pad, H, Wd), lp.conv_dgrad(dY, W, pad, H, Wd), rtol=0, atol=1e-12)
        np.testing.assert_allclose(ly.conv_wgrad(X, dY, pad, R, S), lp.conv_wgrad(X, dY, pad, R, S), rtol=0, atol=1e-12)
