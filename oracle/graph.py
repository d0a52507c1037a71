"""Oracle for the tiling search on a general dataflow graph.  TEST INFRASTRUCTURE ONLY.

Written from arXiv 1805.04170 Sec. 4.2 (cost of a graph tiling = sum over operators of the cheapest aligned form,
Eqs. 2-3), Sec. 4.3 (Algorithm 1 and Theorem 1) and Sec. 4.5 (tensors with d dimensions: one basic tiling per
dimension plus replication; operators other than products differ only in their set of aligned tilings).  Everything
here is the definition written out: a graph tiling is priced operator by operator, the optimum is found by trying
every assignment.  No levels, no dynamic programming, no tables - small graphs only.

Vocabulary
  tensor   {"shape": (n0, ..., n_{d-1}), "same_as": index of an earlier tensor whose tiling it must share, or None}
           (the gradient of a weight is stored like the weight: the update is element-wise, Sec. 2.1)
  letter   an int i (the basic tiling that halves dimension i) or "r" (replicate); "red" only as an aligned output
  tiling   a tuple of k letters, cut 0 (the first, outermost cut) first
  operator {"kind": "contract", "ins": [x, y], "out": z, "m": (dx, dz), "n": (dy, dz), "k": (dx, dy)}
               z = contraction of x and y; m: the dimension of x (and of z) that only x has, n: the same for y,
               k: the contracted dimension in x and in y.  Aligned forms (Sec. 4.2.1):
                 1: x cut along m, y replicated, z cut along m      2: x replicated, y cut along n, z cut along n
                 3: x and y cut along k, z holds partial sums ("red")
               A matrix product x.y is m=(0,0), n=(1,1), k=(1,0); x.y^T is n=(0,1), k=(1,1); x^T.y is m=(1,0), k=(0,0);
               a convolution X[N,C,H,W] * W[K,C,R,S] -> Y[N,K,P,Q] is m=(0,0), n=(0,1), k=(1,1) (Sec. 4.5: batch and
               channel dimensions only).
           {"kind": "elementwise", "ins": [...], "out": z}   same shape everywhere; aligned: every operand cut along
               the same dimension (all replicated is redundant computation and not allowed)
           {"kind": "batch", "ins": [...], "out": z}         any other operator: every operand cut along dimension 0
           {"kind": "sample_channel", "ins": [...], "out": z}  works on every (sample, channel) pair by itself - pooling,
               the flattening of channel-major images in front of a fully-connected layer: operands may differ in shape
               beyond dimensions 0 and 1; aligned: all cut along dimension 0, or all along dimension 1 (a cut of the
               flattened columns is a channel cut as long as the channel count, the smallest extent 1, is even)

Readings (the same as for the layer chain): conversion cost of a tile with A elements over two devices, summed over
both: same letter 0; between two different cuts A/2; cut -> replicated A; replicated -> anything 0; partial sums ->
cut A, -> replicated 2A.  Cut j prices the tiles left by cuts 0..j-1 and carries weight 2^j.  Only even cuts: a
letter i needs an even extent, a form needs an even extent of the dimension it halves.  An operator's cost under
k-cut tilings is the minimum over feasible form sequences of sum_j 2^j (cost of form f_j at cut j).

Parity pins (tests/test_oracle_graph.py): one-cut costs of the element-wise, batch-only and per-sample-and-channel
operators by explicit index-set counts; chains and convolutions written as graphs against the chain oracle (cost.c,
other code) on random tilings of one to three cuts and on optima; closed forms.  The paper prints no cost of a general
graph and no k-cut value: beyond those pins the k-cut figures are "parity unpinned by the paper".
"""
import itertools

INF = float("inf")
REP = "r"
RED = "red"


def conv_cost(frm, to, area):
    if frm == REP:
        return 0
    if frm == RED:
        return 2 * area if to == REP else area
    if frm == to:
        return 0
    if to == REP:
        return area
    assert area % 2 == 0
    return area // 2


def root(tensors, i):
    while tensors[i].get("same_as") is not None:
        i = tensors[i]["same_as"]
    return i


def letters_of(tensor):
    return list(range(len(tensor["shape"]))) + [REP]


def tile_areas(shape, tiling):
    """element count of the stored tile that each cut works on; None if some cut is uneven"""
    shape = list(shape)
    areas = []
    for letter in tiling:
        a = 1
        for n in shape:
            a *= n
        areas.append(a)
        if letter != REP:
            if shape[letter] % 2:
                return None
            shape[letter] //= 2
    return areas


def forms_of(op, tensors):
    """list of (aligned letters of the inputs, aligned letter of the output, extent that the form halves)"""
    ins, out = op["ins"], op["out"]
    if op["kind"] == "contract":
        x, y = tensors[ins[0]]["shape"], tensors[ins[1]]["shape"]
        (mx, mz), (ny, nz), (kx, ky) = op["m"], op["n"], op["k"]
        assert x[mx] == tensors[out]["shape"][mz] and y[ny] == tensors[out]["shape"][nz] and x[kx] == y[ky]
        return [((mx, REP), mz, x[mx]), ((REP, ny), nz, y[ny]), ((kx, ky), RED, x[kx])]
    shape = tensors[out]["shape"]
    if op["kind"] == "elementwise":
        assert all(tensors[i]["shape"] == shape for i in ins)
        return [(tuple(d for _ in ins), d, shape[d]) for d in range(len(shape))]
    if op["kind"] == "sample_channel":
        shapes = [tensors[i]["shape"] for i in ins] + [shape]
        chans = min(sh[1] for sh in shapes)
        assert all(sh[0] == shape[0] and sh[1] % chans == 0 for sh in shapes)
        return [(tuple(0 for _ in ins), 0, shape[0]), (tuple(1 for _ in ins), 1, chans)]
    assert op["kind"] == "batch"
    assert all(tensors[i]["shape"][0] == shape[0] for i in ins)
    return [(tuple(0 for _ in ins), 0, shape[0])]


def op_cost(op, tensors, tilings, k, want_forms=False):
    """cheapest feasible form sequence of one operator under k-cut tilings of its operands"""
    ids = [root(tensors, i) for i in op["ins"]] + [root(tensors, op["out"])]
    areas = [tile_areas(tensors[i]["shape"], tilings[i]) for i in ids]
    if any(a is None for a in areas):
        return (INF, None) if want_forms else INF
    forms = forms_of(op, tensors)
    best, arg = INF, None
    for seq in itertools.product(range(len(forms)), repeat=k):
        # the dimension a form halves must still be even when the form is used
        ok = True
        for f in set(seq):
            if forms[f][2] % (2 ** seq.count(f)):
                ok = False
        if not ok:
            continue
        total = 0
        for j, f in enumerate(seq):
            a_in, a_out, _ = forms[f]
            c = sum(conv_cost(tilings[ids[q]][j], a_in[q], areas[q][j]) for q in range(len(a_in)))
            c += conv_cost(a_out, tilings[ids[-1]][j], areas[-1][j])
            total += c << j
        if total < best:
            best, arg = total, seq
    return (best, arg) if want_forms else best


def graph_cost(tensors, ops, k, tilings):
    """Eq. 3 over a general graph; tilings: {tensor index (any member of a same_as group): tuple of k letters}"""
    t = {root(tensors, i): tuple(v) for i, v in tilings.items()}
    total = 0
    for op in ops:
        c = op_cost(op, tensors, t, k)
        if c == INF:
            return INF
        total += c
    return total


def variables(tensors):
    return [i for i in range(len(tensors)) if tensors[i].get("same_as") is None]


def feasible_tilings(tensor, k):
    return [t for t in itertools.product(letters_of(tensor), repeat=k) if tile_areas(tensor["shape"], t) is not None]


def bruteforce(tensors, ops, k, pins=None):
    """minimum of graph_cost over every assignment; returns (cost, {variable: tiling})"""
    pins = {root(tensors, i): tuple(v) for i, v in (pins or {}).items()}
    var = variables(tensors)
    choices = [[pins[v]] if v in pins else feasible_tilings(tensors[v], k) for v in var]
    best, arg = INF, None
    for combo in itertools.product(*choices):
        t = dict(zip(var, combo))
        c = graph_cost(tensors, ops, k, t)
        if c < best:
            best, arg = c, t
    return best, arg


def greedy_is_valid(tensors, ops, k, tilings, forms, deltas):
    """Check a plan that claims to come from Algorithm 1: at every cut j the letters chosen for that cut must reach
    the one-cut optimum of the graph left by cuts 0..j-1 (tiles of the stored tensors; operator extents halved by the
    forms the plan used), the plan's delta_j must be that optimum, and Theorem 1 gives the total.
    tilings: {variable: tuple of k letters}; forms: list over ops of k form indices; deltas: k ints."""
    shapes = {v: list(tensors[v]["shape"]) for v in variables(tensors)}
    extents = [[f[2] for f in forms_of(op, tensors)] for op in ops]

    def one_cut_cost(assign, check_forms=None):
        total = 0
        for q, op in enumerate(ops):
            ids = [root(tensors, i) for i in op["ins"]] + [root(tensors, op["out"])]
            fl = forms_of(op, tensors)
            best, arg = INF, None
            for f, (a_in, a_out, _) in enumerate(fl):
                if extents[q][f] % 2:
                    continue
                c = 0
                for p in range(len(a_in)):
                    c += conv_cost(assign[ids[p]], a_in[p], _area(shapes[ids[p]]))
                c += conv_cost(a_out, assign[ids[-1]], _area(shapes[ids[-1]]))
                if c < best:
                    best, arg = c, f
            if best == INF:
                return INF
            if check_forms is not None:
                f = check_forms[q]
                a_in, a_out, _ = fl[f]
                if extents[q][f] % 2:
                    return INF
                c = sum(conv_cost(assign[ids[p]], a_in[p], _area(shapes[ids[p]])) for p in range(len(a_in)))
                c += conv_cost(a_out, assign[ids[-1]], _area(shapes[ids[-1]]))
                if c != best:
                    return INF  # the plan's form is not a cheapest one
            total += best
        return total

    var = variables(tensors)
    for j in range(k):
        opts = []
        for v in var:
            opts.append([l for l in letters_of(tensors[v]) if l == REP or shapes[v][l] % 2 == 0])
        optimum = min(one_cut_cost(dict(zip(var, combo))) for combo in itertools.product(*opts))
        mine = {v: tilings[v][j] for v in var}
        for v in var:
            if mine[v] != REP and shapes[v][mine[v]] % 2:
                return False
        got = one_cut_cost(mine, [forms[q][j] for q in range(len(ops))])
        if got != optimum or deltas[j] != optimum:
            return False
        for v in var:
            if mine[v] != REP:
                shapes[v][mine[v]] //= 2
        for q in range(len(ops)):
            extents[q][forms[q][j]] //= 2
    return True


def _area(shape):
    a = 1
    for n in shape:
        a *= n
    return a


# ---- builders used by the tests (graph descriptions only; no arithmetic of the method)

def matmul(x, y, z, ta=False, tb=False):
    m = (1, 0) if ta else (0, 0)
    kx = 0 if ta else 1
    n = (0, 1) if tb else (1, 1)
    ky = 1 if tb else 0
    return {"kind": "contract", "ins": [x, y], "out": z, "m": m, "n": n, "k": (kx, ky)}


def mlp_graph(batch, widths):
    """the 3L products of an L-layer chain (forward, backward, gradient; Sec. 4.2.2): tensors x_0..x_L, g_0..g_L,
    W_1..W_L and dW_1..dW_L stored like W_l.  Returns (tensors, ops, index maps)."""
    L = len(widths) - 1
    tensors, ops = [], []
    x = []
    g = []
    w = []
    for l in range(L + 1):
        x.append(len(tensors)); tensors.append({"shape": (batch, widths[l]), "same_as": None})
        g.append(len(tensors)); tensors.append({"shape": (batch, widths[l]), "same_as": None})
    for l in range(1, L + 1):
        w.append(len(tensors)); tensors.append({"shape": (widths[l - 1], widths[l]), "same_as": None})
    dw = []
    for l in range(1, L + 1):
        dw.append(len(tensors)); tensors.append({"shape": (widths[l - 1], widths[l]), "same_as": w[l - 1]})
    for l in range(1, L + 1):
        ops.append(matmul(x[l - 1], w[l - 1], x[l]))
        ops.append(matmul(g[l], w[l - 1], g[l - 1], tb=True))
        ops.append(matmul(x[l - 1], g[l], dw[l - 1], ta=True))
    return tensors, ops, {"x": x, "g": g, "w": w, "dw": dw}
