"""Python face of cost.c (conversion costs, Eq. 2, Eq. 3, brute force, Algorithm 1).

The C file is compiled on first use with gcc into oracle/_build/.  Tilings are
strings over "RCr", cut 0 first.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cost.c")
_LIB = os.path.join(_HERE, "_build", "liboracle_cost.so")
INF = 2 ** 64 - 1
MAXL = 16
LETTER = {"R": 0, "C": 1, "r": 2, "red": 3}
NAMES = "RCr"


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC])
    return _LIB


class _Chain(ctypes.Structure):
    _fields_ = [("L", ctypes.c_int), ("batch", ctypes.c_int64),
                ("width", ctypes.c_int64 * (MAXL + 1)),
                ("xmult", ctypes.c_int64 * (MAXL + 1)),
                ("wmult", ctypes.c_int64 * (MAXL + 1))]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u8p = ctypes.POINTER(ctypes.c_uint8)
        u64p = ctypes.POINTER(ctypes.c_uint64)
        L.oracle_chain_cost.restype = ctypes.c_uint64
        L.oracle_chain_cost.argtypes = [ctypes.POINTER(_Chain), ctypes.c_int, u8p, u8p, u8p, u8p, u64p]
        L.oracle_bruteforce.restype = ctypes.c_uint64
        L.oracle_bruteforce.argtypes = [ctypes.POINTER(_Chain), ctypes.c_int, u8p, u8p, u8p, u8p, ctypes.c_int,
                                        ctypes.POINTER(ctypes.c_int)]
        L.oracle_recursive.restype = ctypes.c_uint64
        L.oracle_recursive.argtypes = [ctypes.POINTER(_Chain), ctypes.c_int, u8p, u8p, u8p, u8p, u8p, u8p, u8p, u64p]
        L.oracle_eq2_term.restype = ctypes.c_uint64
        L.oracle_eq2_term.argtypes = [ctypes.c_int] * 4 + [ctypes.c_uint64] * 3
        L.oracle_conv_cost.restype = ctypes.c_uint64
        L.oracle_conv_cost.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_uint64]
        _lib = L
    return _lib


def make_chain(batch, widths, xmult=None, wmult=None):
    c = _Chain()
    c.L = len(widths) - 1
    assert 1 <= c.L <= MAXL
    c.batch = batch
    for i, w in enumerate(widths):
        c.width[i] = w
        c.xmult[i] = 1 if xmult is None else xmult[i]
        c.wmult[i] = 1 if (wmult is None or i == 0) else wmult[i]
    return c


def _letters(seq_list):
    """list of tiling strings -> flat uint8 ctypes array"""
    flat = [LETTER[ch] for t in seq_list for ch in t]
    return (ctypes.c_uint8 * len(flat))(*flat)


def _pin(t):
    return None if t is None else _letters([t])


def _decode(code, k):
    out = []
    for _ in range(k):
        out.append(NAMES[code % 3])
        code //= 3
    return "".join(reversed(out))


def conv_cost(frm, to, A):
    return lib().oracle_conv_cost(LETTER[frm], LETTER[to], A)


def eq2_term(form, lx, ly, lz, Ax, Ay, Az):
    return lib().oracle_eq2_term(form, LETTER[lx], LETTER[ly], LETTER[lz], Ax, Ay, Az)


def chain_cost(chain, k, x, g, w):
    """Eq. 3 for tilings x[0..L], g[0..L], w[0..L-1] (w[i] tiles W_{i+1}).
    Returns (cost, forms, delta); forms[l][op] is a string over '123' (op order F, B, G)."""
    L = chain.L
    forms = (ctypes.c_uint8 * (3 * L * k))()
    delta = (ctypes.c_uint64 * k)()
    cost = lib().oracle_chain_cost(ctypes.byref(chain), k, _letters(x), _letters(g), _letters(w), forms, delta)
    f = [["".join("123"[forms[((l * 3) + op) * k + j]] for j in range(k)) for op in range(3)] for l in range(L)]
    return cost, f, list(delta)


def bruteforce(chain, k, pin_x0=None, pin_g0=None, pin_xL=None, pin_gL=None, prune=True):
    """Minimum of Eq. 3 over every k-cut graph tiling.  Returns (cost, x, g, w)."""
    L = chain.L
    assign = (ctypes.c_int * (3 * L + 2))()
    cost = lib().oracle_bruteforce(ctypes.byref(chain), k, _pin(pin_x0), _pin(pin_g0), _pin(pin_xL), _pin(pin_gL),
                                   1 if prune else 0, assign)
    if cost == INF:
        return cost, None, None, None
    x = [_decode(assign[0], k)] + [_decode(assign[3 + 3 * l], k) for l in range(L)]
    g = [_decode(assign[1], k)] + [_decode(assign[4 + 3 * l], k) for l in range(L)]
    w = [_decode(assign[2 + 3 * l], k) for l in range(L)]
    return cost, x, g, w


def recursive(chain, k, pin_x0=None, pin_g0=None, pin_xL=None, pin_gL=None):
    """Algorithm 1 with exhaustive one-cut search.  Returns (cost, x, g, w, delta)."""
    L = chain.L
    xo = (ctypes.c_uint8 * ((L + 1) * k))()
    go = (ctypes.c_uint8 * ((L + 1) * k))()
    wo = (ctypes.c_uint8 * (L * k))()
    delta = (ctypes.c_uint64 * k)()
    cost = lib().oracle_recursive(ctypes.byref(chain), k, _pin(pin_x0), _pin(pin_g0), _pin(pin_xL), _pin(pin_gL),
                                  xo, go, wo, delta)
    if cost == INF:
        return cost, None, None, None, None
    s = lambda arr, i: "".join(NAMES[arr[i * k + j]] for j in range(k))
    return (cost, [s(xo, l) for l in range(L + 1)], [s(go, l) for l in range(L + 1)],
            [s(wo, l) for l in range(L)], list(delta))
