"""ctypes binding of libtensor_tiling.so: same names as include/tensor_tiling.h, argument marshalling only.

Shard lists are Python sequences of torch tensors (their data_ptr() is passed) or of integer device addresses.
Tilings are strings over "RCr" (cut 0 first); form sequences are strings over "123".  A non-zero status raises
TilingError.  The HIP stream defaults to torch's current stream.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtensor_tiling.so")

TT_MAX_K = 6
TT_MAX_LAYERS = 16
TT_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024
TT_R, TT_C, TT_REP = 0, 1, 2
TT_F32, TT_BF16 = 0, 1
TT_ACT_NONE, TT_ACT_RELU = 0, 1
TT_FC, TT_CONV2D = 0, 1
TT_PLAN_EXACT, TT_PLAN_RECURSIVE = 0, 1
TT_OP_FWD, TT_OP_DGRAD, TT_OP_WGRAD = 0, 1, 2
TT_TENSOR_X, TT_TENSOR_G, TT_TENSOR_W = 0, 1, 2
STATUS_NAMES = {0: "TT_OK", 1: "TT_EINVAL", 2: "TT_EINFEASIBLE", 3: "TT_EUNSUPPORTED", 4: "TT_ENOMEM",
                5: "TT_EDEVICE", 6: "TT_EWORKSPACE"}

EXPORTS = [
    "tt_strerror", "tt_shard_shape", "tt_plan_chain", "tt_plan_eval", "tt_plan_k", "tt_plan_layers", "tt_plan_cost",
    "tt_plan_delta", "tt_plan_tiling", "tt_plan_forms", "tt_plan_free", "tt_retile", "tt_flatten", "tt_retile_gate", "tt_reduce",
    "tt_shard_gemm", "tt_fc_workspace_bytes", "tt_fc_forward", "tt_fc_forward_static", "tt_fc_backward", "tt_fc_backward_overlapped",
    "tt_conv_workspace_bytes",
    "tt_conv_forward", "tt_conv_backward", "tt_profile_begin", "tt_profile_end", "tt_profile_get",
    "tt_plan_graph", "tt_graph_eval", "tt_graph_plan_cost", "tt_graph_plan_delta", "tt_graph_plan_levels",
    "tt_graph_plan_level_of", "tt_graph_plan_tiling", "tt_graph_plan_forms", "tt_graph_plan_free",
    "tt_conversion_cross_elems", "tt_product_cross_elems", "tt_fc_chain_cross_elems",
]
TT_LETTER_REP, TT_LETTER_FREE = 255, 253
TT_GOP_CONTRACT, TT_GOP_ELEMENTWISE, TT_GOP_BATCH, TT_GOP_SAMPLE_CHANNEL = 0, 1, 2, 3
KERNEL_NAMES = ["convert", "gate", "reduce", "gemm_nn", "gemm_nt", "gemm_tn", "gemm_tt", "gemm_generic", "conv_fwd",
                "conv_dgrad", "conv_wgrad"]


class TilingError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s failed: %s (%s)" % (what, STATUS_NAMES.get(status, status), strerror(status)))


class tt_tiling(ctypes.Structure):
    _fields_ = [("cut", ctypes.c_uint8 * TT_MAX_K)]


class tt_graph_tensor(ctypes.Structure):
    _fields_ = [("ndim", ctypes.c_int32), ("same_as", ctypes.c_int32), ("shape", ctypes.c_int64 * 4)]


class tt_graph_op(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("n_in", ctypes.c_int32), ("in_", ctypes.c_int32 * 4), ("out", ctypes.c_int32),
                ("m", ctypes.c_int32 * 2), ("n", ctypes.c_int32 * 2), ("kk", ctypes.c_int32 * 2)]


class tt_kernel_record(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("count", ctypes.c_int32), ("d0", ctypes.c_int64), ("d1", ctypes.c_int64),
                ("d2", ctypes.c_int64), ("bytes", ctypes.c_uint64), ("flops", ctypes.c_uint64), ("ms", ctypes.c_float)]


class tt_layer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("act", ctypes.c_int32), ("n_in", ctypes.c_int64), ("n_out", ctypes.c_int64),
                ("H", ctypes.c_int64), ("W", ctypes.c_int64), ("R", ctypes.c_int64), ("S", ctypes.c_int64),
                ("pad", ctypes.c_int64)]


_lib = None
_vpp = ctypes.POINTER(ctypes.c_void_p)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_u64p = ctypes.POINTER(ctypes.c_uint64)


def lib():
    """Load the HIP library.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libtensor_tiling.so is not built; run `python -m paper_1805_04170_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.tt_strerror.restype = ctypes.c_char_p
        L.tt_strerror.argtypes = [ctypes.c_int]
        L.tt_shard_shape.argtypes = [ctypes.c_int64, ctypes.c_int64, tt_tiling, ctypes.c_int,
                                     ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
        tp = ctypes.POINTER(tt_tiling)
        lp = ctypes.POINTER(tt_layer)
        L.tt_plan_chain.argtypes = [lp, ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32, tp, tp, tp, tp,
                                    ctypes.POINTER(ctypes.c_void_p)]
        L.tt_plan_eval.argtypes = [lp, ctypes.c_int, ctypes.c_int64, ctypes.c_int, tp, tp, tp, _u64p, _u64p, _u8p]
        L.tt_plan_k.argtypes = [ctypes.c_void_p]
        L.tt_plan_layers.argtypes = [ctypes.c_void_p]
        L.tt_plan_cost.argtypes = [ctypes.c_void_p]
        L.tt_plan_cost.restype = ctypes.c_uint64
        L.tt_plan_delta.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.tt_plan_delta.restype = ctypes.c_uint64
        L.tt_plan_tiling.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, tp]
        L.tt_plan_forms.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, _u8p]
        L.tt_plan_free.argtypes = [ctypes.c_void_p]
        L.tt_plan_free.restype = None
        L.tt_conversion_cross_elems.argtypes = [ctypes.c_int64, ctypes.c_int64, tt_tiling, tt_tiling, ctypes.c_int, _u64p]
        L.tt_product_cross_elems.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, tt_tiling, tt_tiling, tt_tiling,
                                             _u8p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, _u64p]
        L.tt_fc_chain_cross_elems.argtypes = [lp, ctypes.c_int, ctypes.c_int64, ctypes.c_int, tp, tp, tp, _u8p, _u64p]
        gtp, gop = ctypes.POINTER(tt_graph_tensor), ctypes.POINTER(tt_graph_op)
        L.tt_plan_graph.argtypes = [gtp, ctypes.c_int, gop, ctypes.c_int, ctypes.c_int, ctypes.c_uint32, _u8p,
                                    ctypes.POINTER(ctypes.c_void_p)]
        L.tt_graph_eval.argtypes = [gtp, ctypes.c_int, gop, ctypes.c_int, ctypes.c_int, _u8p, _u64p, _u64p, _u8p]
        L.tt_graph_plan_cost.argtypes = [ctypes.c_void_p]
        L.tt_graph_plan_cost.restype = ctypes.c_uint64
        L.tt_graph_plan_delta.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.tt_graph_plan_delta.restype = ctypes.c_uint64
        L.tt_graph_plan_levels.argtypes = [ctypes.c_void_p]
        L.tt_graph_plan_level_of.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.tt_graph_plan_tiling.argtypes = [ctypes.c_void_p, ctypes.c_int, _u8p]
        L.tt_graph_plan_forms.argtypes = [ctypes.c_void_p, ctypes.c_int, _u8p]
        L.tt_graph_plan_free.argtypes = [ctypes.c_void_p]
        L.tt_graph_plan_free.restype = None
        L.tt_retile.argtypes = [_vpp, tt_tiling, _vpp, tt_tiling, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                ctypes.c_int, ctypes.c_void_p]
        L.tt_flatten.argtypes = [_vpp, tt_tiling, _vpp, tt_tiling, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                 ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        L.tt_retile_gate.argtypes = [_vpp, tt_tiling, _vpp, tt_tiling, _vpp, tt_tiling, ctypes.c_int, ctypes.c_int64,
                                     ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]
        L.tt_reduce.argtypes = [_vpp, tt_tiling, ctypes.c_int, _vpp, _u8p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                ctypes.c_int, ctypes.c_void_p]
        L.tt_shard_gemm.argtypes = [ctypes.c_int, _vpp, _vpp, _vpp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                    ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        ws_args = [lp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, tt_tiling, tt_tiling, tt_tiling,
                   tt_tiling, tt_tiling, _u8p, _u8p, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
        fwd_args = [lp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, tt_tiling, tt_tiling, tt_tiling, _u8p, _vpp, _vpp,
                    _vpp, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        bwd_args = [lp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, tt_tiling, tt_tiling, tt_tiling, tt_tiling, tt_tiling,
                    _u8p, _u8p, _vpp, _vpp, _vpp, _vpp, _vpp, _vpp, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.tt_fc_workspace_bytes.argtypes = ws_args
        L.tt_conv_workspace_bytes.argtypes = ws_args
        L.tt_fc_forward.argtypes = fwd_args
        L.tt_conv_forward.argtypes = fwd_args
        L.tt_fc_forward_static.argtypes = fwd_args[:11] + [ctypes.c_void_p]
        L.tt_fc_backward.argtypes = bwd_args
        L.tt_conv_backward.argtypes = bwd_args
        L.tt_fc_backward_overlapped.argtypes = bwd_args + [ctypes.c_void_p]
        L.tt_profile_end.argtypes = [ctypes.POINTER(ctypes.c_int)]
        L.tt_profile_get.argtypes = [ctypes.c_int, ctypes.POINTER(tt_kernel_record)]
        _lib = L
    return _lib


def strerror(status):
    return lib().tt_strerror(int(status)).decode()


def _check(status, what):
    if status != 0:
        raise TilingError(status, what)


_LETTER = {"R": TT_R, "C": TT_C, "r": TT_REP}
_NAMES = "RCr"


def tiling(t):
    """'RCr' string (or tt_tiling) -> tt_tiling"""
    if isinstance(t, tt_tiling):
        return t
    out = tt_tiling()
    if len(t) > TT_MAX_K:
        raise TilingError(1, "tiling(%r)" % (t,))
    for j, ch in enumerate(t):
        out.cut[j] = _LETTER[ch] if ch in _LETTER else 255
    return out


def tiling_str(t, k):
    return "".join(_NAMES[t.cut[j]] for j in range(k))


def forms(f):
    """'123' string -> uint8 array, None -> NULL"""
    if f is None:
        return None
    return (ctypes.c_uint8 * max(len(f), 1))(*[int(ch) - 1 for ch in f])


def layer(kind="fc", act="none", n_in=0, n_out=0, H=0, W=0, R=0, S=0, pad=0):
    return tt_layer(TT_FC if kind == "fc" else TT_CONV2D, TT_ACT_RELU if act == "relu" else TT_ACT_NONE, n_in, n_out,
                    H, W, R, S, pad)


def ptrs(shards):
    """sequence of tensors / addresses -> void*[]; None -> NULL"""
    if shards is None:
        return None
    vals = [(s.data_ptr() if hasattr(s, "data_ptr") else int(s)) for s in shards]
    return (ctypes.c_void_p * max(len(vals), 1))(*vals)


def _stream(stream):
    if stream is not None:
        # a raw stream handle, or a torch.cuda.Stream
        return ctypes.c_void_p(int(getattr(stream, "cuda_stream", stream)))
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype(d):
    if isinstance(d, int):
        return d
    return {"bf16": TT_BF16, "f32": TT_F32}[d]


# ------------------------------------------------------------------ geometry

def tt_shard_shape(rows, cols, t, k=None):
    k = len(t) if k is None else k
    sr, sc = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().tt_shard_shape(rows, cols, tiling(t), k, ctypes.byref(sr), ctypes.byref(sc)), "tt_shard_shape")
    return sr.value, sc.value


# ------------------------------------------------------------------- planner

class Plan:
    """Owner of a tt_plan; accessors mirror the C ones."""

    def __init__(self, handle):
        self._h = handle

    def __del__(self):
        if getattr(self, "_h", None):
            lib().tt_plan_free(self._h)
            self._h = None

    @property
    def k(self):
        return lib().tt_plan_k(self._h)

    @property
    def n_layers(self):
        return lib().tt_plan_layers(self._h)

    @property
    def cost(self):
        return lib().tt_plan_cost(self._h)

    def delta(self, cut):
        return lib().tt_plan_delta(self._h, cut)

    def tiling(self, which, index):
        out = tt_tiling()
        _check(lib().tt_plan_tiling(self._h, which, index, ctypes.byref(out)), "tt_plan_tiling")
        return tiling_str(out, self.k)

    def forms(self, layer_index, op):
        buf = (ctypes.c_uint8 * max(self.k, 1))()
        _check(lib().tt_plan_forms(self._h, layer_index, op, buf), "tt_plan_forms")
        return "".join("123"[buf[j]] for j in range(self.k))

    def x(self):
        return [self.tiling(TT_TENSOR_X, l) for l in range(self.n_layers + 1)]

    def g(self):
        return [self.tiling(TT_TENSOR_G, l) for l in range(self.n_layers + 1)]

    def w(self):
        return [self.tiling(TT_TENSOR_W, l) for l in range(1, self.n_layers + 1)]


def _layers(layers):
    return (tt_layer * len(layers))(*layers)


def _pin(t):
    return None if t is None else ctypes.byref(tiling(t))


def tt_plan_chain(layers, batch, k, mode=TT_PLAN_EXACT, pin_x0=None, pin_g0=None, pin_xL=None, pin_gL=None):
    h = ctypes.c_void_p()
    _check(lib().tt_plan_chain(_layers(layers), len(layers), batch, k, mode, _pin(pin_x0), _pin(pin_g0), _pin(pin_xL),
                               _pin(pin_gL), ctypes.byref(h)), "tt_plan_chain")
    return Plan(h)


def tt_plan_eval(layers, batch, k, x, g, w):
    """Returns (cost, delta[k], forms[layer][op] as '123' strings)."""
    L = len(layers)
    xa = (tt_tiling * (L + 1))(*[tiling(t) for t in x])
    ga = (tt_tiling * (L + 1))(*[tiling(t) for t in g])
    wa = (tt_tiling * L)(*[tiling(t) for t in w])
    cost = ctypes.c_uint64()
    delta = (ctypes.c_uint64 * max(k, 1))()
    fo = (ctypes.c_uint8 * max(3 * L * k, 1))()
    _check(lib().tt_plan_eval(_layers(layers), L, batch, k, xa, ga, wa, ctypes.byref(cost), delta, fo), "tt_plan_eval")
    f = [["".join("123"[fo[(l * 3 + op) * k + j]] for j in range(k)) for op in range(3)] for l in range(L)]
    return cost.value, [delta[j] for j in range(k)], f


# ------------------------------------------------ what an execution really moves

def tt_conversion_cross_elems(rows, cols, frm, to, k=None):
    k = len(frm) if k is None else k
    out = ctypes.c_uint64()
    _check(lib().tt_conversion_cross_elems(rows, cols, tiling(frm), tiling(to), k, ctypes.byref(out)),
           "tt_conversion_cross_elems")
    return out.value


def tt_product_cross_elems(M, K, N, tX, tY, tZ, form_seq, mult=(1, 1, 1), k=None):
    """Returns [X conversion, Y conversion, output conversion / reduction] in elements."""
    k = len(form_seq) if k is None else k
    out = (ctypes.c_uint64 * 3)()
    _check(lib().tt_product_cross_elems(M, K, N, tiling(tX), tiling(tY), tiling(tZ), forms(form_seq), k, mult[0], mult[1],
                                        mult[2], out), "tt_product_cross_elems")
    return [out[0], out[1], out[2]]


def tt_fc_chain_cross_elems(layers, batch, k, x, g, w, layer_forms):
    """layer_forms[l][op]: form strings ('123') of the forward, data-gradient and weight-gradient product of layer l."""
    L = len(layers)
    xa = (tt_tiling * (L + 1))(*[tiling(t) for t in x])
    ga = (tt_tiling * (L + 1))(*[tiling(t) for t in g])
    wa = (tt_tiling * L)(*[tiling(t) for t in w])
    flat = [int(ch) - 1 for lf in layer_forms for f in lf for ch in f]
    fo = (ctypes.c_uint8 * max(len(flat), 1))(*flat)
    out = ctypes.c_uint64()
    _check(lib().tt_fc_chain_cross_elems(_layers(layers), L, batch, k, xa, ga, wa, fo, ctypes.byref(out)),
           "tt_fc_chain_cross_elems")
    return out.value


# ----------------------------------------------------- planner, general graphs

def graph_tensor(shape, same_as=-1):
    t = tt_graph_tensor()
    t.ndim, t.same_as = len(shape), same_as
    for d, n in enumerate(shape):
        t.shape[d] = n
    return t


def graph_op(kind, ins, out, m=(0, 0), n=(0, 0), kk=(0, 0)):
    o = tt_graph_op()
    o.kind, o.n_in, o.out = kind, len(ins), out
    for i, v in enumerate(ins):
        o.in_[i] = v
    o.m[0], o.m[1], o.n[0], o.n[1], o.kk[0], o.kk[1] = m[0], m[1], n[0], n[1], kk[0], kk[1]
    return o


def _graph_letters(tilings, n_tensors, k):
    """tilings: {tensor: sequence of k letters (dimension index or 'r')}; tensors left out are free"""
    buf = (ctypes.c_uint8 * max(n_tensors * k, 1))(*([TT_LETTER_FREE] * max(n_tensors * k, 1)))
    for i, t in (tilings or {}).items():
        assert len(t) == k
        for j, l in enumerate(t):
            buf[i * k + j] = TT_LETTER_REP if l == "r" else int(l)
    return buf


class GraphPlan:
    """Owner of a tt_graph_plan; accessors mirror the C ones (letters come back as dimension indices or 'r')."""

    def __init__(self, handle, k):
        self._h, self.k = handle, k

    def __del__(self):
        if getattr(self, "_h", None):
            lib().tt_graph_plan_free(self._h)
            self._h = None

    @property
    def cost(self):
        return lib().tt_graph_plan_cost(self._h)

    def delta(self, cut):
        return lib().tt_graph_plan_delta(self._h, cut)

    @property
    def n_levels(self):
        return lib().tt_graph_plan_levels(self._h)

    def level_of(self, op):
        return lib().tt_graph_plan_level_of(self._h, op)

    def tiling(self, tensor):
        buf = (ctypes.c_uint8 * max(self.k, 1))()
        _check(lib().tt_graph_plan_tiling(self._h, tensor, buf), "tt_graph_plan_tiling")
        return tuple("r" if buf[j] == TT_LETTER_REP else int(buf[j]) for j in range(self.k))

    def forms(self, op):
        buf = (ctypes.c_uint8 * max(self.k, 1))()
        _check(lib().tt_graph_plan_forms(self._h, op, buf), "tt_graph_plan_forms")
        return [int(buf[j]) for j in range(self.k)]


def tt_plan_graph(tensors, ops, k, mode=TT_PLAN_EXACT, pins=None):
    ta = (tt_graph_tensor * len(tensors))(*tensors)
    oa = (tt_graph_op * len(ops))(*ops)
    h = ctypes.c_void_p()
    _check(lib().tt_plan_graph(ta, len(tensors), oa, len(ops), k, mode,
                               _graph_letters(pins, len(tensors), k) if pins else None, ctypes.byref(h)), "tt_plan_graph")
    return GraphPlan(h, k)


def tt_graph_eval(tensors, ops, k, tilings):
    """Returns (cost, delta[k], forms[op][k])."""
    ta = (tt_graph_tensor * len(tensors))(*tensors)
    oa = (tt_graph_op * len(ops))(*ops)
    cost = ctypes.c_uint64()
    delta = (ctypes.c_uint64 * max(k, 1))()
    fo = (ctypes.c_uint8 * max(len(ops) * k, 1))()
    _check(lib().tt_graph_eval(ta, len(tensors), oa, len(ops), k, _graph_letters(tilings, len(tensors), k),
                               ctypes.byref(cost), delta, fo), "tt_graph_eval")
    return cost.value, [delta[j] for j in range(k)], [[fo[q * k + j] for j in range(k)] for q in range(len(ops))]


# --------------------------------------------------------------- conversions

def tt_retile(dst, B, src, A, rows, cols, elem_bytes, k=None, stream=None):
    k = len(A) if k is None else k
    _check(lib().tt_retile(ptrs(dst), tiling(B), ptrs(src), tiling(A), k, rows, cols, elem_bytes, _stream(stream)),
           "tt_retile")


def tt_flatten(dst, B, src, A, batch, channels, pixels, elem_bytes, to_matrix=True, k=None, stream=None):
    k = len(A) if k is None else k
    _check(lib().tt_flatten(ptrs(dst), tiling(B), ptrs(src), tiling(A), k, batch, channels, pixels, elem_bytes,
                            1 if to_matrix else 0, _stream(stream)), "tt_flatten")


def tt_retile_gate(dst, B, src, A, mask, Am, rows, cols, dtype, k=None, stream=None):
    k = len(A) if k is None else k
    _check(lib().tt_retile_gate(ptrs(dst), tiling(B), ptrs(src), tiling(A), ptrs(mask), tiling(Am if mask is not None else A),
                                k, rows, cols, _dtype(dtype), _stream(stream)), "tt_retile_gate")


def tt_reduce(dst, B, out_dtype, partials, form_seq, rows, cols, act=TT_ACT_NONE, k=None, stream=None):
    k = len(form_seq) if k is None else k
    _check(lib().tt_reduce(ptrs(dst), tiling(B), _dtype(out_dtype), ptrs(partials), forms(form_seq), k, rows, cols, act,
                           _stream(stream)), "tt_reduce")


# ------------------------------------------------------------ shard products

def tt_shard_gemm(A, B, C, M, N, K, trans_a=0, trans_b=0, in_dtype=TT_BF16, out_dtype=TT_BF16, act=TT_ACT_NONE,
                  stream=None):
    _check(lib().tt_shard_gemm(len(C), ptrs(A), ptrs(B), ptrs(C), M, N, K, trans_a, trans_b, _dtype(in_dtype),
                               _dtype(out_dtype), act, _stream(stream)), "tt_shard_gemm")


# ------------------------------------------------------------- layer execute

def _ws(workspace):
    if workspace is None:
        return None, 0
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def _t_or(t, default):
    return tiling(default if t is None else t)


def _workspace_bytes(fn, what, lay, batch, k, dtype, op, tX, tW, tY, tdY, tdX, forms_a, forms_b, with_dx):
    out = ctypes.c_size_t()
    _check(fn(ctypes.byref(lay), batch, k, _dtype(dtype), op, tiling(tX), tiling(tW), tiling(tY), _t_or(tdY, tY),
              _t_or(tdX, tX), forms(forms_a), forms(forms_b), 1 if with_dx else 0, ctypes.byref(out)), what)
    return out.value


def tt_fc_workspace_bytes(lay, batch, k, dtype, op, tX, tW, tY, tdY=None, tdX=None, forms_a=None, forms_b=None,
                          with_dx=True):
    return _workspace_bytes(lib().tt_fc_workspace_bytes, "tt_fc_workspace_bytes", lay, batch, k, dtype, op, tX, tW, tY,
                            tdY, tdX, forms_a, forms_b, with_dx)


def tt_conv_workspace_bytes(lay, batch, k, dtype, op, tX, tW, tY, tdY=None, tdX=None, forms_a=None, forms_b=None,
                            with_dx=True):
    return _workspace_bytes(lib().tt_conv_workspace_bytes, "tt_conv_workspace_bytes", lay, batch, k, dtype, op, tX, tW,
                            tY, tdY, tdX, forms_a, forms_b, with_dx)


def _forward(fn, what, lay, batch, k, dtype, tX, tW, tY, form_seq, X, W, Y, workspace, stream):
    wp, wb = _ws(workspace)
    _check(fn(ctypes.byref(lay), batch, k, _dtype(dtype), tiling(tX), tiling(tW), tiling(tY), forms(form_seq), ptrs(X),
              ptrs(W), ptrs(Y), wp, wb, _stream(stream)), what)


def _backward(fn, what, lay, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_dgrad, forms_wgrad, X, W, Y, dY, dX, dW,
              workspace, stream):
    wp, wb = _ws(workspace)
    _check(fn(ctypes.byref(lay), batch, k, _dtype(dtype), tiling(tX), tiling(tW), tiling(tY), tiling(tdY),
              _t_or(tdX, tX), forms(forms_dgrad), forms(forms_wgrad), ptrs(X), ptrs(W), ptrs(Y), ptrs(dY), ptrs(dX),
              ptrs(dW), wp, wb, _stream(stream)), what)


def tt_fc_forward(lay, batch, k, dtype, tX, tW, tY, form_seq, X, W, Y, workspace=None, stream=None):
    _forward(lib().tt_fc_forward, "tt_fc_forward", lay, batch, k, dtype, tX, tW, tY, form_seq, X, W, Y, workspace, stream)


def tt_fc_forward_static(lay, batch, k, dtype, tX, tW, tY, form_seq, X, W, Y, stream=None):
    _check(lib().tt_fc_forward_static(ctypes.byref(lay), batch, k, _dtype(dtype), tiling(tX), tiling(tW), tiling(tY),
                                      forms(form_seq), ptrs(X), ptrs(W), ptrs(Y), _stream(stream)), "tt_fc_forward_static")


def tt_fc_backward(lay, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_dgrad, forms_wgrad, X, W, Y, dY, dX, dW,
                   workspace=None, stream=None):
    _backward(lib().tt_fc_backward, "tt_fc_backward", lay, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_dgrad,
              forms_wgrad, X, W, Y, dY, dX, dW, workspace, stream)


def tt_fc_backward_overlapped(lay, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_dgrad, forms_wgrad, X, W, Y, dY, dX, dW,
                              workspace=None, stream=None, aux_stream=None):
    wp, wb = _ws(workspace)
    _check(lib().tt_fc_backward_overlapped(
        ctypes.byref(lay), batch, k, _dtype(dtype), tiling(tX), tiling(tW), tiling(tY), tiling(tdY), _t_or(tdX, tX),
        forms(forms_dgrad), forms(forms_wgrad), ptrs(X), ptrs(W), ptrs(Y), ptrs(dY), ptrs(dX), ptrs(dW), wp, wb,
        _stream(stream), _stream(aux_stream) if aux_stream is not None else None), "tt_fc_backward_overlapped")


def tt_conv_forward(lay, batch, k, dtype, tX, tW, tY, form_seq, X, W, Y, workspace=None, stream=None):
    _forward(lib().tt_conv_forward, "tt_conv_forward", lay, batch, k, dtype, tX, tW, tY, form_seq, X, W, Y, workspace,
             stream)


def tt_conv_backward(lay, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_dgrad, forms_wgrad, X, W, Y, dY, dX, dW,
                     workspace=None, stream=None):
    _backward(lib().tt_conv_backward, "tt_conv_backward", lay, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_dgrad,
              forms_wgrad, X, W, Y, dY, dX, dW, workspace, stream)


# ------------------------------------------------------------- kernel timing

def tt_profile_begin():
    _check(lib().tt_profile_begin(), "tt_profile_begin")


def tt_profile_end():
    """Returns the list of per-launch records as dicts."""
    n = ctypes.c_int()
    _check(lib().tt_profile_end(ctypes.byref(n)), "tt_profile_end")
    out = []
    for i in range(n.value):
        r = tt_kernel_record()
        _check(lib().tt_profile_get(i, ctypes.byref(r)), "tt_profile_get")
        out.append(dict(kernel=KERNEL_NAMES[r.kernel], count=r.count, d0=r.d0, d1=r.d1, d2=r.d2, bytes=r.bytes,
                        flops=r.flops, ms=r.ms))
    return out
