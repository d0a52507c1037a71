"""Python face of layers_plain.c: the layer operators of Sec. 2.1 (and the textbook convolution) as plain nested loops
in fp64.  TEST INFRASTRUCTURE ONLY.  Compiled on first use with gcc into oracle/_build/.

These are the definitions written out; oracle/layers.py computes the same sums through numpy (so that full-size checks
take seconds) and is pinned against these on small shapes in tests/test_oracle_layers.py.  The benchmark's
cpu_baseline times these."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "layers_plain.c")
_LIB = os.path.join(_HERE, "_build", "liboracle_layers_plain.so")
_lib = None
_dp = ctypes.POINTER(ctypes.c_double)
_i64 = ctypes.c_int64


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.plain_fc_forward.argtypes = [_dp, _dp, _dp, _i64, _i64, _i64, ctypes.c_int]
        L.plain_fc_backward.argtypes = [_dp] * 7 + [_i64, _i64, _i64, ctypes.c_int]
        for f in (L.plain_conv_forward, L.plain_conv_dgrad, L.plain_conv_wgrad):
            f.argtypes = [_dp, _dp, _dp] + [_i64] * 8
        for f in (L.plain_fc_forward, L.plain_fc_backward, L.plain_conv_forward, L.plain_conv_dgrad, L.plain_conv_wgrad):
            f.restype = None
        _lib = L
    return _lib


def threads():
    """threads the loops run on (OpenMP's default: every core the process may use, or OMP_NUM_THREADS)"""
    env = os.environ.get("OMP_NUM_THREADS", "")
    if env.isdigit() and int(env) > 0:
        return int(env)
    return len(os.sched_getaffinity(0))


def _c(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(_dp)


def fc_forward(X, W, relu):
    X, W = _c(X), _c(W)
    Y = np.empty((X.shape[0], W.shape[1]))
    lib().plain_fc_forward(_p(X), _p(W), _p(Y), X.shape[0], X.shape[1], W.shape[1], int(bool(relu)))
    return Y


def fc_backward(dY, X, W, Y, relu):
    dY, X, W, Y = _c(dY), _c(X), _c(W), _c(Y)
    b, n_in, n_out = X.shape[0], X.shape[1], W.shape[1]
    G, dX, dW = np.empty((b, n_out)), np.empty((b, n_in)), np.empty((n_in, n_out))
    lib().plain_fc_backward(_p(dY), _p(X), _p(W), _p(Y), _p(G), _p(dX), _p(dW), b, n_in, n_out, int(bool(relu)))
    return dX, dW


def conv_forward(X, W, pad):
    X, W = _c(X), _c(W)
    N, C, H, Wd = X.shape
    K, _, R, S = W.shape
    Y = np.empty((N, K, H + 2 * pad - R + 1, Wd + 2 * pad - S + 1))
    lib().plain_conv_forward(_p(X), _p(W), _p(Y), N, C, H, Wd, K, R, S, pad)
    return Y


def conv_dgrad(dY, W, pad, H, Wd):
    dY, W = _c(dY), _c(W)
    N, K = dY.shape[:2]
    _, C, R, S = W.shape
    dX = np.empty((N, C, H, Wd))
    lib().plain_conv_dgrad(_p(dY), _p(W), _p(dX), N, C, H, Wd, K, R, S, pad)
    return dX


def conv_wgrad(X, dY, pad, R, S):
    X, dY = _c(X), _c(dY)
    N, C, H, Wd = X.shape
    K = dY.shape[1]
    dW = np.empty((K, C, R, S))
    lib().plain_conv_wgrad(_p(X), _p(dY), _p(dW), N, C, H, Wd, K, R, S, pad)
    return dW
