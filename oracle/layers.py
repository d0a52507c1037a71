"""Untiled layer operators in fp64 (Sec. 2.1: x_{l+1} = f(x_l W_l),
dC/dx_l = df(dC/dx_{l+1}) W_l^T, dC/dW_l = x_l^T df(dC/dx_{l+1})), f = ReLU or
identity.  W is n_in x n_out.  Convolution is the textbook stride-1
cross-correlation with zero padding; its backward operators are written from
the same sum, term by term."""
import numpy as np


def fc_forward(X, W, relu):
    pre = np.matmul(X.astype(np.float64), W.astype(np.float64))
    return np.maximum(pre, 0.0) if relu else pre


def fc_backward(dY, X, W, Y, relu):
    """Returns (dX, dW).  Y is the layer's output (post-activation)."""
    G = dY.astype(np.float64)
    if relu:
        G = G * (Y > 0)
    dX = np.matmul(G, W.astype(np.float64).T)
    dW = np.matmul(X.astype(np.float64).T, G)
    return dX, dW


def abs_product(A, B):
    """(|A| |B|)_ij : the scale the contraction tolerance is stated against."""
    return np.matmul(np.abs(A.astype(np.float64)), np.abs(B.astype(np.float64)))


def _padded(X, pad):
    return np.pad(X.astype(np.float64), ((0, 0), (0, 0), (pad, pad), (pad, pad)))


def conv_forward(X, W, pad):
    """Y[n,ko,y,x] = sum_{c,r,s} X[n,c,y+r-pad,x+s-pad] W[ko,c,r,s], zero outside."""
    N, C, H, Wd = X.shape
    K, _, R, S = W.shape
    P, Q = H + 2 * pad - R + 1, Wd + 2 * pad - S + 1
    Xp = _padded(X, pad)
    Wf = W.astype(np.float64)
    Y = np.zeros((N, K, P, Q))
    for r in range(R):
        for s in range(S):
            # sum over c of X[n,c,y+r,x+s] * W[ko,c,r,s]
            Y += np.einsum("ncyx,kc->nkyx", Xp[:, :, r:r + P, s:s + Q], Wf[:, :, r, s], optimize=True)
    return Y


def conv_dgrad(dY, W, pad, H, Wd):
    """dX[n,c,h,w] = sum over every (ko,r,s,y,x) term of the forward sum that reads X[n,c,h,w]."""
    N, K, P, Q = dY.shape
    _, C, R, S = W.shape
    dXp = np.zeros((N, C, H + 2 * pad, Wd + 2 * pad))
    G = dY.astype(np.float64)
    Wf = W.astype(np.float64)
    for r in range(R):
        for s in range(S):
            dXp[:, :, r:r + P, s:s + Q] += np.einsum("nkyx,kc->ncyx", G, Wf[:, :, r, s], optimize=True)
    return dXp[:, :, pad:pad + H, pad:pad + Wd]


def conv_wgrad(X, dY, pad, R, S):
    """dW[ko,c,r,s] = sum_{n,y,x} X[n,c,y+r-pad,x+s-pad] dY[n,ko,y,x]."""
    N, K, P, Q = dY.shape
    C = X.shape[1]
    Xp = _padded(X, pad)
    G = dY.astype(np.float64)
    dW = np.zeros((K, C, R, S))
    for r in range(R):
        for s in range(S):
            dW[:, :, r, s] = np.einsum("ncyx,nkyx->kc", Xp[:, :, r:r + P, s:s + Q], G, optimize=True)
    return dW


def conv_forward_point(X, W, pad, n, ko, y, x):
    """One output of conv_forward from the definition (for sampled checks at full size)."""
    _, C, H, Wd = X.shape
    _, _, R, S = W.shape
    acc = 0.0
    mag = 0.0
    for r in range(R):
        for s in range(S):
            h, w = y + r - pad, x + s - pad
            if 0 <= h < H and 0 <= w < Wd:
                a = X[n, :, h, w].astype(np.float64)
                b = W[ko, :, r, s].astype(np.float64)
                acc += float(np.dot(a, b))
                mag += float(np.dot(np.abs(a), np.abs(b)))
    return acc, mag
