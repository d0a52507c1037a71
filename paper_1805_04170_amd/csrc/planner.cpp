// Host-side tiling planner (Sec. 4 of arXiv 1805.04170): communication cost of a graph tiling (Eq. 2, Eq. 3,
// Theorem 1) and the search for the cheapest k-cut tiling of a layer chain (one-cut dynamic program Eqs. 4-5,
// k-cut recursion Algorithm 1, and an exact joint dynamic program over k-cut sequences).
//
// Cost model as implemented (the paper prints the principle, not the table):
//   conversion cost c(from -> to) of a tensor tile with A elements, two devices, summed over both:
//        R->R, C->C: 0;  R<->C: A/2;  R->r, C->r: A;  r->anything: 0;  red->R, red->C: A;  red->r: 2A
//   cut j works on the tiles left by cuts 0..j-1 (R halves rows, C halves columns, r keeps the shape);
//   product cost = min over feasible form sequences of sum_j 2^j * Eq.2-term(form_j); a sequence is feasible when
//   M, N, K divide by 2^(#F1), 2^(#F2), 2^(#F3); a tensor tiling is feasible when every cut is even.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <new>
#include <vector>

#include "tt_internal.h"

namespace tt {
namespace {

constexpr uint64_t kInf = std::numeric_limits<uint64_t>::max();

inline uint64_t add_sat(uint64_t a, uint64_t b) { return (a == kInf || b == kInf) ? kInf : a + b; }

// conversion-cost numerator in halves of A: cost = A * half[from][to] / 2
const uint8_t kHalf[4][3] = {
    /* R   */ {0, 1, 2},
    /* C   */ {1, 0, 2},
    /* r   */ {0, 0, 0},
    /* red */ {2, 2, 4},
};
inline uint64_t convert_cost(int from, int to, uint64_t area) { return area * kHalf[from][to] / 2; }

const uint8_t kAlignedX[3] = {TT_R, TT_REP, TT_C};
const uint8_t kAlignedY[3] = {TT_REP, TT_C, TT_R};
const uint8_t kAlignedZ[3] = {TT_R, TT_C, kRed};

inline uint64_t form_cost(int f, int lx, int ly, int lz, uint64_t ax, uint64_t ay, uint64_t az)
{
    return convert_cost(lx, kAlignedX[f], ax) + convert_cost(ly, kAlignedY[f], ay) + convert_cost(kAlignedZ[f], lz, az);
}

// per-cut areas of a tensor under a stored tiling; false if some cut is uneven
bool tile_areas(const CostTensor &t, const uint8_t *cuts, int k, uint64_t *area)
{
    int64_t r = t.rows, c = t.cols;
    for (int j = 0; j < k; ++j) {
        area[j] = (uint64_t)r * (uint64_t)c * (uint64_t)t.mult;
        if (cuts[j] == TT_R) { if (r & 1) return false; r >>= 1; }
        else if (cuts[j] == TT_C) { if (c & 1) return false; c >>= 1; }
    }
    return true;
}

int max_pow2(int64_t v, int cap)
{
    int n = 0;
    while (n < cap && v > 0 && (v & 1) == 0) { v >>= 1; ++n; }
    return v == 0 ? cap : n;
}

struct FormSearch {
    int k;
    int cap[3];
    uint64_t c[TT_MAX_K][3];
    uint64_t best;
    uint8_t cur[TT_MAX_K], arg[TT_MAX_K];
    void go(int j, int n1, int n2, int n3, uint64_t acc)
    {
        if (j == k) { if (acc < best) { best = acc; std::memcpy(arg, cur, sizeof(arg)); } return; }
        const int n[3] = {n1, n2, n3};
        for (int f = 0; f < 3; ++f) {
            if (n[f] + 1 > cap[f]) continue;
            cur[j] = (uint8_t)f;
            go(j + 1, n1 + (f == 0), n2 + (f == 1), n3 + (f == 2), acc + (c[j][f] << j));
        }
    }
};

} // namespace

uint64_t matmul_cost(const CostTensor &X, const CostTensor &Y, const CostTensor &Z, int64_t M, int64_t K, int64_t N,
                     const uint8_t *tx, const uint8_t *ty, const uint8_t *tz, int k, uint8_t *forms_out,
                     uint64_t *level_out)
{
    uint64_t ax[TT_MAX_K], ay[TT_MAX_K], az[TT_MAX_K];
    if (!tile_areas(X, tx, k, ax) || !tile_areas(Y, ty, k, ay) || !tile_areas(Z, tz, k, az)) return kInf;
    FormSearch fs;
    fs.k = k;
    fs.cap[0] = max_pow2(M, k);
    fs.cap[1] = max_pow2(N, k);
    fs.cap[2] = max_pow2(K, k);
    for (int j = 0; j < k; ++j)
        for (int f = 0; f < 3; ++f) fs.c[j][f] = form_cost(f, tx[j], ty[j], tz[j], ax[j], ay[j], az[j]);
    // unconstrained optimum: cheapest form per cut, lowest index on ties
    uint8_t pick[TT_MAX_K];
    int cnt[3] = {0, 0, 0};
    uint64_t total = 0;
    for (int j = 0; j < k; ++j) {
        int f = 0;
        if (fs.c[j][1] < fs.c[j][f]) f = 1;
        if (fs.c[j][2] < fs.c[j][f]) f = 2;
        pick[j] = (uint8_t)f;
        cnt[f]++;
        total += fs.c[j][f] << j;
    }
    if (cnt[0] > fs.cap[0] || cnt[1] > fs.cap[1] || cnt[2] > fs.cap[2]) {
        fs.best = kInf;
        fs.go(0, 0, 0, 0, 0);
        if (fs.best == kInf) return kInf;
        total = fs.best;
        std::memcpy(pick, fs.arg, sizeof(pick));
    }
    if (forms_out) std::memcpy(forms_out, pick, (size_t)k);
    if (level_out)
        for (int j = 0; j < k; ++j) level_out[j] = fs.c[j][pick[j]];
    return total;
}

namespace {

struct Chain {
    int L = 0;
    int64_t batch = 0;
    int64_t width[TT_MAX_LAYERS + 1];
    int64_t xmult[TT_MAX_LAYERS + 1];
    int64_t wmult[TT_MAX_LAYERS + 1];
};

// Whole networks (Sec. 6: AlexNet and VGG are convolution layers followed by fully-connected ones):
//  - convolution after convolution with a SMALLER image than the previous layer produced: a pooling / striding stage in
//    between.  It works per image and per channel, so like the other element-wise functions (Eq. 1, Sec. 4.5) it moves
//    nothing under any tiling; the tensor between the two layers is charged at the size the next layer reads;
//  - fully-connected after convolution: the flattening of (channels x pixels) per image.  The tensor keeps its channel
//    count as the cuttable column dimension (a column cut is a channel cut, as for the convolution that produced it)
//    and its pixels per channel as the area multiplier; the layer is the convolution whose filter covers the whole
//    image (weights: channels x n_out, times pixels).  n_in must be channels x pixels, pixels at most what the
//    convolution (or the pooling after it) left.
tt_status make_chain(const tt_layer *layers, int n_layers, int64_t batch, Chain *c)
{
    if (!layers || n_layers < 1 || n_layers > TT_MAX_LAYERS || batch <= 0) return TT_EINVAL;
    c->L = n_layers;
    c->batch = batch;
    for (int l = 0; l < n_layers; ++l) {
        const tt_layer &y = layers[l];
        if (y.n_in <= 0 || y.n_out <= 0) return TT_EINVAL;
        if (y.kind != TT_FC && y.kind != TT_CONV2D) return TT_EINVAL;
        const bool after_conv = l > 0 && layers[l - 1].kind == TT_CONV2D;
        if (l > 0 && y.kind == TT_CONV2D && !after_conv) return TT_EUNSUPPORTED; // fc -> conv is not modelled
        int64_t in_mult = 1, out_mult = 1, w_mult = 1;
        if (y.kind == TT_CONV2D) {
            if (l > 0 && y.n_in != layers[l - 1].n_out) return TT_EINVAL;
            if (y.H <= 0 || y.W <= 0 || y.R <= 0 || y.S <= 0 || y.pad < 0) return TT_EINVAL;
            int64_t P = y.H + 2 * y.pad - y.R + 1, Q = y.W + 2 * y.pad - y.S + 1;
            if (P <= 0 || Q <= 0) return TT_EINVAL;
            in_mult = y.H * y.W;
            out_mult = P * Q;
            w_mult = y.R * y.S;
            if (l > 0) {
                if (in_mult > c->xmult[l]) return TT_EINVAL; // nothing here enlarges an image
                c->xmult[l] = in_mult;                       // pooled in between: charged at the size this layer reads
            }
        } else if (after_conv) {
            const int64_t ch = layers[l - 1].n_out;
            if (y.n_in % ch) return TT_EINVAL;
            const int64_t pixels = y.n_in / ch;
            if (pixels > c->xmult[l]) return TT_EINVAL;
            c->xmult[l] = pixels;
            w_mult = pixels;
        } else if (l > 0 && y.n_in != layers[l - 1].n_out) {
            return TT_EINVAL;
        }
        if (l == 0) { c->width[0] = y.n_in; c->xmult[0] = in_mult; }
        c->width[l + 1] = y.n_out;
        c->xmult[l + 1] = out_mult;
        c->wmult[l + 1] = w_mult;
    }
    return TT_OK;
}

inline void swap_rc(const uint8_t *t, int k, uint8_t *o)
{
    for (int j = 0; j < k; ++j) o[j] = t[j] == TT_R ? TT_C : (t[j] == TT_C ? TT_R : TT_REP);
}

// cost of product op (0 F, 1 B, 2 G) of layer l (1-based) under the given tilings
uint64_t product_cost(const Chain &c, int l, int op, int k, const uint8_t *xp, const uint8_t *gp, const uint8_t *w,
                      const uint8_t *x, const uint8_t *g, uint8_t *forms, uint64_t *levels)
{
    const int64_t b = c.batch, ni = c.width[l - 1], no = c.width[l];
    const CostTensor Xp{b, ni, c.xmult[l - 1]}, Xn{b, no, c.xmult[l]}, W{ni, no, c.wmult[l]};
    uint8_t tt[TT_MAX_K];
    if (op == TT_OP_FWD) return matmul_cost(Xp, W, Xn, b, ni, no, xp, w, x, k, forms, levels);
    if (op == TT_OP_DGRAD) {
        swap_rc(w, k, tt);
        const CostTensor Wt{no, ni, c.wmult[l]};
        return matmul_cost(Xn, Wt, Xp, b, no, ni, g, tt, gp, k, forms, levels);
    }
    swap_rc(xp, k, tt);
    const CostTensor Xt{ni, b, c.xmult[l - 1]};
    return matmul_cost(Xt, Xn, W, ni, b, no, tt, g, w, k, forms, levels);
}

inline void decode(int code, int k, uint8_t *t)
{
    for (int j = k - 1; j >= 0; --j) { t[j] = (uint8_t)(code % 3); code /= 3; }
}
inline int encode(const uint8_t *t, int k)
{
    int c = 0;
    for (int j = 0; j < k; ++j) c = c * 3 + t[j];
    return c;
}

} // namespace
} // namespace tt

struct tt_plan {
    int k = 0, L = 0;
    uint64_t cost = 0;
    uint64_t delta[TT_MAX_K] = {};
    std::vector<tt_tiling> x, g, w; // x,g: L+1; w: L
    std::vector<uint8_t> forms;     // 3*L*k
};

namespace tt {
namespace {

tt_status eval_into(const Chain &c, int k, const tt_tiling *x, const tt_tiling *g, const tt_tiling *w, uint64_t *cost,
                    uint64_t *delta, uint8_t *forms)
{
    uint64_t total = 0, d[TT_MAX_K] = {};
    for (int l = 1; l <= c.L; ++l)
        for (int op = 0; op < 3; ++op) {
            uint8_t f[TT_MAX_K];
            uint64_t lev[TT_MAX_K];
            uint64_t v = product_cost(c, l, op, k, x[l - 1].cut, g[l - 1].cut, w[l - 1].cut, x[l].cut, g[l].cut, f, lev);
            if (v == kInf) return TT_EINFEASIBLE;
            total += v;
            for (int j = 0; j < k; ++j) d[j] += lev[j];
            if (forms) std::memcpy(forms + ((l - 1) * 3 + op) * k, f, (size_t)k);
        }
    *cost = total;
    if (delta) std::memcpy(delta, d, sizeof(uint64_t) * (size_t)k);
    return TT_OK;
}

// ---- exact joint search: Eqs. 4-5 with whole k-cut sequences as the per-level states
tt_status plan_exact(const Chain &c, int k, const tt_tiling *pins[4], tt_plan *plan)
{
    if (k > 4) return TT_EUNSUPPORTED;
    int n = 1;
    for (int j = 0; j < k; ++j) n *= 3;
    const size_t n2 = (size_t)n * n, n3 = n2 * n;
    std::vector<uint64_t> best(n2, kInf), next(n2), inner(n);
    std::vector<uint64_t> F(n3), B(n3), G(n3);
    // back pointers per layer: for (x,g): chosen x', W; for (W,g,x'): chosen g'
    std::vector<std::vector<int>> bp_xw(c.L + 1), bp_g(c.L + 1);
    std::vector<std::vector<uint8_t>> seqs(n, std::vector<uint8_t>(TT_MAX_K));
    for (int a = 0; a < n; ++a) decode(a, k, seqs[a].data());

    const int pin_x0 = pins[0] ? encode(pins[0]->cut, k) : -1, pin_g0 = pins[1] ? encode(pins[1]->cut, k) : -1;
    const int pin_xL = pins[2] ? encode(pins[2]->cut, k) : -1, pin_gL = pins[3] ? encode(pins[3]->cut, k) : -1;
    for (int x = 0; x < n; ++x)
        for (int g = 0; g < n; ++g)
            if ((pin_x0 < 0 || x == pin_x0) && (pin_g0 < 0 || g == pin_g0)) best[(size_t)x * n + g] = 0;

    for (int l = 1; l <= c.L; ++l) {
        for (int a = 0; a < n; ++a)
            for (int b = 0; b < n; ++b)
                for (int d = 0; d < n; ++d) {
                    const uint8_t *ta = seqs[a].data(), *tb = seqs[b].data(), *td = seqs[d].data();
                    size_t i = ((size_t)a * n + b) * n + d;
                    F[i] = product_cost(c, l, TT_OP_FWD, k, ta, nullptr, tb, td, nullptr, nullptr, nullptr);   // [x'][W][x]
                    B[i] = product_cost(c, l, TT_OP_DGRAD, k, nullptr, td, tb, nullptr, ta, nullptr, nullptr); // [g][W][g']
                    G[i] = product_cost(c, l, TT_OP_WGRAD, k, ta, nullptr, td, nullptr, tb, nullptr, nullptr); // [x'][g][W]
                }
        std::fill(next.begin(), next.end(), kInf);
        bp_xw[l].assign(n2 * 2, -1);
        bp_g[l].assign(n3, -1);
        for (int w = 0; w < n; ++w)
            for (int g = 0; g < n; ++g) {
                const bool last = l == c.L;
                if (last && pin_gL >= 0 && g != pin_gL) continue;
                // inner[x'] = min_{g'} best[x'][g'] + B[g][W][g']
                for (int xp = 0; xp < n; ++xp) {
                    uint64_t m = kInf;
                    int arg = -1;
                    const uint64_t *brow = &B[((size_t)g * n + w) * n];
                    const uint64_t *prow = &best[(size_t)xp * n];
                    for (int gp = 0; gp < n; ++gp) {
                        uint64_t v = add_sat(prow[gp], brow[gp]);
                        if (v < m) { m = v; arg = gp; }
                    }
                    m = add_sat(m, G[((size_t)xp * n + g) * n + w]);
                    inner[xp] = m;
                    bp_g[l][((size_t)w * n + g) * n + xp] = arg;
                }
                for (int x = 0; x < n; ++x) {
                    if (last && pin_xL >= 0 && x != pin_xL) continue;
                    uint64_t &slot = next[(size_t)x * n + g];
                    for (int xp = 0; xp < n; ++xp) {
                        uint64_t v = add_sat(inner[xp], F[((size_t)xp * n + w) * n + x]);
                        if (v < slot) {
                            slot = v;
                            bp_xw[l][((size_t)x * n + g) * 2] = xp;
                            bp_xw[l][((size_t)x * n + g) * 2 + 1] = w;
                        }
                    }
                }
            }
        best.swap(next);
    }
    uint64_t opt = kInf;
    int ax = -1, ag = -1;
    for (int x = 0; x < n; ++x)
        for (int g = 0; g < n; ++g)
            if (best[(size_t)x * n + g] < opt) { opt = best[(size_t)x * n + g]; ax = x; ag = g; }
    if (opt == kInf) return TT_EINFEASIBLE;
    plan->x.resize(c.L + 1);
    plan->g.resize(c.L + 1);
    plan->w.resize(c.L);
    for (int l = c.L; l >= 1; --l) {
        decode(ax, k, plan->x[l].cut);
        decode(ag, k, plan->g[l].cut);
        int xp = bp_xw[l][((size_t)ax * n + ag) * 2], w = bp_xw[l][((size_t)ax * n + ag) * 2 + 1];
        int gp = bp_g[l][((size_t)w * n + ag) * n + xp];
        decode(w, k, plan->w[l - 1].cut);
        ax = xp;
        ag = gp;
    }
    decode(ax, k, plan->x[0].cut);
    decode(ag, k, plan->g[0].cut);
    plan->forms.assign((size_t)3 * c.L * k, 0);
    uint64_t check = 0;
    tt_status st = eval_into(c, k, plan->x.data(), plan->g.data(), plan->w.data(), &check, plan->delta, plan->forms.data());
    if (st != TT_OK) return st;
    if (check != opt) return TT_EINVAL; // internal inconsistency; never expected
    plan->cost = opt;
    return TT_OK;
}

// ---- Algorithm 1: one-cut dynamic program per cut, then recurse on the tile graph
struct Shape { int64_t rows, cols, mult; };
struct Dims { int64_t M, K, N; };

uint64_t onecut_product(const Shape &X, const Shape &Y, const Shape &Z, const Dims &d, int lx, int ly, int lz, int *form)
{
    if ((lx == TT_R && (X.rows & 1)) || (lx == TT_C && (X.cols & 1))) return kInf;
    if ((ly == TT_R && (Y.rows & 1)) || (ly == TT_C && (Y.cols & 1))) return kInf;
    if ((lz == TT_R && (Z.rows & 1)) || (lz == TT_C && (Z.cols & 1))) return kInf;
    const uint64_t ax = (uint64_t)X.rows * X.cols * X.mult, ay = (uint64_t)Y.rows * Y.cols * Y.mult, az = (uint64_t)Z.rows * Z.cols * Z.mult;
    const int64_t dim[3] = {d.M, d.N, d.K};
    uint64_t best = kInf;
    for (int f = 0; f < 3; ++f) {
        if (dim[f] & 1) continue;
        uint64_t v = form_cost(f, lx, ly, lz, ax, ay, az);
        if (v < best) { best = v; if (form) *form = f; }
    }
    return best;
}

inline Shape tr(const Shape &s) { return Shape{s.cols, s.rows, s.mult}; }
inline int trl(int l) { return l == TT_R ? TT_C : (l == TT_C ? TT_R : TT_REP); }
inline void cut_shape(Shape &s, int l) { if (l == TT_R) s.rows >>= 1; else if (l == TT_C) s.cols >>= 1; }
inline void cut_dims(Dims &d, int f) { if (f == 0) d.M >>= 1; else if (f == 1) d.N >>= 1; else d.K >>= 1; }

tt_status plan_recursive(const Chain &c, int k, const tt_tiling *pins[4], tt_plan *plan)
{
    const int L = c.L;
    std::vector<Shape> X(L + 1), Gs(L + 1), W(L + 1);
    std::vector<Dims> dF(L + 1), dB(L + 1), dG(L + 1);
    for (int l = 0; l <= L; ++l) X[l] = Gs[l] = Shape{c.batch, c.width[l], c.xmult[l]};
    for (int l = 1; l <= L; ++l) {
        W[l] = Shape{c.width[l - 1], c.width[l], c.wmult[l]};
        dF[l] = Dims{c.batch, c.width[l - 1], c.width[l]};
        dB[l] = Dims{c.batch, c.width[l], c.width[l - 1]};
        dG[l] = Dims{c.width[l - 1], c.batch, c.width[l]};
    }
    plan->x.assign(L + 1, tt_tiling{});
    plan->g.assign(L + 1, tt_tiling{});
    plan->w.assign(L, tt_tiling{});
    plan->forms.assign((size_t)3 * L * k, 0);
    uint64_t total = 0;
    // layer cost for one cut: lc[l][xp][gp][w][x][g]
    std::vector<uint64_t> lc((size_t)(L + 1) * 243);
    auto LC = [&](int l, int xp, int gp, int w, int x, int g) -> uint64_t & {
        return lc[(size_t)l * 243 + (((xp * 3 + gp) * 3 + w) * 3 + x) * 3 + g];
    };
    for (int j = 0; j < k; ++j) {
        for (int l = 1; l <= L; ++l)
            for (int xp = 0; xp < 3; ++xp) for (int gp = 0; gp < 3; ++gp) for (int w = 0; w < 3; ++w)
                for (int x = 0; x < 3; ++x) for (int g = 0; g < 3; ++g) {
                    uint64_t v = onecut_product(X[l - 1], W[l], X[l], dF[l], xp, w, x, nullptr);
                    v = add_sat(v, onecut_product(Gs[l], tr(W[l]), Gs[l - 1], dB[l], g, trl(w), gp, nullptr));
                    v = add_sat(v, onecut_product(tr(X[l - 1]), Gs[l], W[l], dG[l], trl(xp), g, w, nullptr));
                    LC(l, xp, gp, w, x, g) = v;
                }
        // suffix costs h[l][x][g]: cheapest completion of layers l+1..L (Eqs. 4-5 run from the far end)
        std::vector<uint64_t> h((size_t)(L + 1) * 9, kInf);
        for (int x = 0; x < 3; ++x) for (int g = 0; g < 3; ++g) {
            bool ok = (!pins[2] || pins[2]->cut[j] == x) && (!pins[3] || pins[3]->cut[j] == g);
            h[(size_t)L * 9 + x * 3 + g] = ok ? 0 : kInf;
        }
        for (int l = L; l >= 1; --l)
            for (int xp = 0; xp < 3; ++xp) for (int gp = 0; gp < 3; ++gp) {
                uint64_t m = kInf;
                for (int w = 0; w < 3; ++w) for (int x = 0; x < 3; ++x) for (int g = 0; g < 3; ++g)
                    m = std::min(m, add_sat(LC(l, xp, gp, w, x, g), h[(size_t)l * 9 + x * 3 + g]));
                h[(size_t)(l - 1) * 9 + xp * 3 + gp] = m;
            }
        uint64_t opt = kInf;
        for (int x = 0; x < 3; ++x) for (int g = 0; g < 3; ++g) {
            if ((pins[0] && pins[0]->cut[j] != x) || (pins[1] && pins[1]->cut[j] != g)) continue;
            opt = std::min(opt, h[x * 3 + g]);
        }
        if (opt == kInf) return TT_EINFEASIBLE;
        // first optimal assignment in the order x_0, g_0, W_1, x_1, g_1, ... with R < C < r
        int cx = -1, cg = -1;
        for (int x = 0; x < 3 && cx < 0; ++x) for (int g = 0; g < 3; ++g) {
            if ((pins[0] && pins[0]->cut[j] != x) || (pins[1] && pins[1]->cut[j] != g)) continue;
            if (h[x * 3 + g] == opt) { cx = x; cg = g; break; }
        }
        plan->x[0].cut[j] = (uint8_t)cx;
        plan->g[0].cut[j] = (uint8_t)cg;
        uint64_t remaining = opt;
        std::vector<int> lw(L + 1), lx(L + 1), lg(L + 1);
        lx[0] = cx; lg[0] = cg;
        for (int l = 1; l <= L; ++l) {
            bool found = false;
            for (int w = 0; w < 3 && !found; ++w) for (int x = 0; x < 3 && !found; ++x) for (int g = 0; g < 3; ++g) {
                uint64_t v = add_sat(LC(l, lx[l - 1], lg[l - 1], w, x, g), h[(size_t)l * 9 + x * 3 + g]);
                if (v == remaining) { lw[l] = w; lx[l] = x; lg[l] = g; found = true; break; }
            }
            if (!found) return TT_EINVAL; // cannot happen: remaining is attained by construction
            remaining -= LC(l, lx[l - 1], lg[l - 1], lw[l], lx[l], lg[l]);
            plan->w[l - 1].cut[j] = (uint8_t)lw[l];
            plan->x[l].cut[j] = (uint8_t)lx[l];
            plan->g[l].cut[j] = (uint8_t)lg[l];
        }
        plan->delta[j] = opt;
        total += opt << j;
        // fix forms, build the tile graph for the next cut
        for (int l = 1; l <= L; ++l) {
            int f = 0;
            onecut_product(X[l - 1], W[l], X[l], dF[l], lx[l - 1], lw[l], lx[l], &f);
            plan->forms[((l - 1) * 3 + 0) * k + j] = (uint8_t)f; cut_dims(dF[l], f);
            onecut_product(Gs[l], tr(W[l]), Gs[l - 1], dB[l], lg[l], trl(lw[l]), lg[l - 1], &f);
            plan->forms[((l - 1) * 3 + 1) * k + j] = (uint8_t)f; cut_dims(dB[l], f);
            onecut_product(tr(X[l - 1]), Gs[l], W[l], dG[l], trl(lx[l - 1]), lg[l], lw[l], &f);
            plan->forms[((l - 1) * 3 + 2) * k + j] = (uint8_t)f; cut_dims(dG[l], f);
        }
        for (int l = 0; l <= L; ++l) { cut_shape(X[l], lx[l]); cut_shape(Gs[l], lg[l]); }
        for (int l = 1; l <= L; ++l) cut_shape(W[l], lw[l]);
    }
    plan->cost = total;
    return TT_OK;
}

} // namespace
} // namespace tt

extern "C" tt_status tt_plan_chain(const tt_layer *layers, int n_layers, int64_t batch, int k, uint32_t mode,
                                   const tt_tiling *pin_x0, const tt_tiling *pin_g0, const tt_tiling *pin_xL,
                                   const tt_tiling *pin_gL, tt_plan **out)
{
    if (!out) return TT_EINVAL;
    *out = nullptr;
    if (!tt::valid_k(k)) return TT_EINVAL;
    if (mode != TT_PLAN_EXACT && mode != TT_PLAN_RECURSIVE) return TT_EINVAL;
    const tt_tiling *pins[4] = {pin_x0, pin_g0, pin_xL, pin_gL};
    for (auto p : pins)
        if (p && !tt::valid_tiling(*p, k)) return TT_EINVAL;
    tt::Chain c;
    tt_status st = tt::make_chain(layers, n_layers, batch, &c);
    if (st != TT_OK) return st;
    tt_plan *plan = new (std::nothrow) tt_plan;
    if (!plan) return TT_ENOMEM;
    plan->k = k;
    plan->L = c.L;
    try {
        st = mode == TT_PLAN_EXACT ? tt::plan_exact(c, k, pins, plan) : tt::plan_recursive(c, k, pins, plan);
    } catch (const std::bad_alloc &) {
        st = TT_ENOMEM;
    }
    if (st != TT_OK) { delete plan; return st; }
    *out = plan;
    return TT_OK;
}

extern "C" tt_status tt_plan_eval(const tt_layer *layers, int n_layers, int64_t batch, int k, const tt_tiling *x,
                                  const tt_tiling *g, const tt_tiling *w, uint64_t *cost_elems, uint64_t *delta_out,
                                  uint8_t *forms_out)
{
    if (!x || !g || !w || !cost_elems || !tt::valid_k(k)) return TT_EINVAL;
    tt::Chain c;
    tt_status st = tt::make_chain(layers, n_layers, batch, &c);
    if (st != TT_OK) return st;
    for (int l = 0; l <= c.L; ++l)
        if (!tt::valid_tiling(x[l], k) || !tt::valid_tiling(g[l], k)) return TT_EINVAL;
    for (int l = 0; l < c.L; ++l)
        if (!tt::valid_tiling(w[l], k)) return TT_EINVAL;
    return tt::eval_into(c, k, x, g, w, cost_elems, delta_out, forms_out);
}

extern "C" int tt_plan_k(const tt_plan *p) { return p ? p->k : -1; }
extern "C" int tt_plan_layers(const tt_plan *p) { return p ? p->L : -1; }
extern "C" uint64_t tt_plan_cost(const tt_plan *p) { return p ? p->cost : 0; }
extern "C" uint64_t tt_plan_delta(const tt_plan *p, int cut) { return (p && cut >= 0 && cut < p->k) ? p->delta[cut] : 0; }

extern "C" tt_status tt_plan_tiling(const tt_plan *p, int which, int index, tt_tiling *out)
{
    if (!p || !out) return TT_EINVAL;
    if (which == TT_TENSOR_X || which == TT_TENSOR_G) {
        if (index < 0 || index > p->L) return TT_EINVAL;
        *out = which == TT_TENSOR_X ? p->x[index] : p->g[index];
        return TT_OK;
    }
    if (which == TT_TENSOR_W) {
        if (index < 1 || index > p->L) return TT_EINVAL;
        *out = p->w[index - 1];
        return TT_OK;
    }
    return TT_EINVAL;
}

extern "C" tt_status tt_plan_forms(const tt_plan *p, int layer, int op, uint8_t *forms_out)
{
    if (!p || !forms_out || layer < 1 || layer > p->L || op < 0 || op > 2) return TT_EINVAL;
    std::memcpy(forms_out, p->forms.data() + ((layer - 1) * 3 + op) * p->k, (size_t)p->k);
    return TT_OK;
}

extern "C" void tt_plan_free(tt_plan *p) { delete p; }
