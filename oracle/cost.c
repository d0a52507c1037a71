/* Oracle for the communication-cost model and the tiling search.
 * TEST INFRASTRUCTURE ONLY - never linked into or called by the product library.
 *
 * Written from arXiv 1805.04170: Sec. 4.2.1 (conversion cost = ghost area minus
 * area already held; Eq. 2 = min over the three aligned forms), Sec. 4.2.2
 * (Eq. 3, the sum over all matrix multiplications), Sec. 4.3 (Algorithm 1 and
 * Theorem 1: c_k = delta_first + 2 c_{k-1}).  Integer arithmetic throughout.
 *
 * Readings where the paper is silent (each repeated in the design notes):
 *  - cut 0 is the first (outermost) cut; its per-cut cost has weight 2^0, cut j
 *    has weight 2^j (Theorem 1 with the paper's index reversed).
 *  - the sub-problem after a cut is the same chain with every tensor replaced
 *    by its tile (R halves rows, C halves columns, r keeps the shape); the area
 *    in a conversion cost at cut j is the element count of the stored tile
 *    produced by cuts 0..j-1.
 *  - a matmul of an N-layer chain: F_l: x_l = x_{l-1} W_l, B_l: g_{l-1} = g_l W_l^T,
 *    G_l: dW_l = x_{l-1}^T g_l with t(dW_l) = t(W_l); a transposed operand has R
 *    and C swapped in its tiling.  All 3L products are counted.
 *  - only even cuts: a tensor tiling is feasible iff each R (C) cut finds an
 *    even row (column) count; a form sequence is feasible iff M, N, K are
 *    divisible by 2^(number of F1, F2, F3 cuts).
 *  - cost of a matmul under k-cut tilings = min over feasible form sequences of
 *    sum_j 2^j * (Eq. 2 term of form f_j at cut j).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define INF UINT64_MAX
#define MAXK 6
#define MAXL 16

enum { L_R = 0, L_C = 1, L_r = 2, L_RED = 3 };

/* c(from -> to) for a tensor of A elements split over two devices (groups), summed
 * over both.  R->C: each side holds one half and needs another half, a quarter
 * overlaps.  red->R: each side needs the other's partial for its half.  red->r:
 * each side needs the other's whole partial. */
static uint64_t conv_cost(int from, int to, uint64_t A)
{
    if (from == L_r) return 0;
    if (from == L_RED) return to == L_r ? 2 * A : A;
    if (from == to) return 0;
    if (to == L_r) return A;
    return A / 2; /* R<->C; A is even because the stored cut itself was even */
}

static const int AX[3] = { L_R, L_r, L_C };   /* aligned X letter of form F1,F2,F3 */
static const int AY[3] = { L_r, L_C, L_R };
static const int AZ[3] = { L_R, L_C, L_RED };

static uint64_t eq2_term(int form, int lx, int ly, int lz, uint64_t Ax, uint64_t Ay, uint64_t Az)
{
    return conv_cost(lx, AX[form], Ax) + conv_cost(ly, AY[form], Ay) + conv_cost(AZ[form], lz, Az);
}

typedef struct { int64_t rows, cols, mult; } tensor_t;

static int tiling_feasible(tensor_t T, const uint8_t *t, int k)
{
    int64_t r = T.rows, c = T.cols;
    for (int j = 0; j < k; ++j) {
        if (t[j] == L_R) { if (r & 1) return 0; r >>= 1; }
        else if (t[j] == L_C) { if (c & 1) return 0; c >>= 1; }
    }
    return 1;
}

/* element count of the stored tile before cut j */
static uint64_t area_at(tensor_t T, const uint8_t *t, int j)
{
    uint64_t A = (uint64_t)T.rows * (uint64_t)T.cols * (uint64_t)T.mult;
    for (int i = 0; i < j; ++i) if (t[i] != L_r) A >>= 1;
    return A;
}

static void transpose_letters(const uint8_t *t, int k, uint8_t *out)
{
    for (int j = 0; j < k; ++j) out[j] = t[j] == L_R ? L_C : (t[j] == L_C ? L_R : L_r);
}

/* Cost of one matmul Z = X Y (M x K times K x N) whose operand tilings tx, ty, tz
 * are already expressed on X, Y, Z as multiplied (transposes applied by the caller).
 * forms_out (k entries) and level_out (k entries) receive the first minimising form
 * sequence (cut 0 varies slowest) and its per-cut Eq. 2 terms. */
static uint64_t matmul_cost(tensor_t X, tensor_t Y, tensor_t Z, int64_t M, int64_t K, int64_t N,
                            const uint8_t *tx, const uint8_t *ty, const uint8_t *tz, int k,
                            uint8_t *forms_out, uint64_t *level_out)
{
    if (!tiling_feasible(X, tx, k) || !tiling_feasible(Y, ty, k) || !tiling_feasible(Z, tz, k)) return INF;
    uint64_t best = INF;
    int nseq = 1;
    for (int j = 0; j < k; ++j) nseq *= 3;
    for (int code = 0; code < nseq; ++code) {
        uint8_t f[MAXK];
        int c = code;
        for (int j = k - 1; j >= 0; --j) { f[j] = (uint8_t)(c % 3); c /= 3; }
        int n1 = 0, n2 = 0, n3 = 0;
        for (int j = 0; j < k; ++j) { n1 += f[j] == 0; n2 += f[j] == 1; n3 += f[j] == 2; }
        if (M % ((int64_t)1 << n1) || N % ((int64_t)1 << n2) || K % ((int64_t)1 << n3)) continue;
        uint64_t tot = 0, lev[MAXK];
        for (int j = 0; j < k; ++j) {
            lev[j] = eq2_term(f[j], tx[j], ty[j], tz[j], area_at(X, tx, j), area_at(Y, ty, j), area_at(Z, tz, j));
            tot += lev[j] << j;
        }
        if (tot < best) {
            best = tot;
            if (forms_out) memcpy(forms_out, f, (size_t)k);
            if (level_out) memcpy(level_out, lev, sizeof(uint64_t) * (size_t)k);
        }
    }
    return best;
}

/* A chain: activations x_0..x_L (batch x width[l], times xmult[l] elements per entry,
 * e.g. H*W of a feature map), weights W_1..W_L (width[l-1] x width[l], times wmult[l],
 * e.g. the R*S filter taps); gradients g_l have the shape of x_l. */
typedef struct {
    int L;
    int64_t batch;
    int64_t width[MAXL + 1];
    int64_t xmult[MAXL + 1];
    int64_t wmult[MAXL + 1];
} chain_t;

static tensor_t act_tensor(const chain_t *c, int l) { tensor_t t = { c->batch, c->width[l], c->xmult[l] }; return t; }
static tensor_t act_tensor_T(const chain_t *c, int l) { tensor_t t = { c->width[l], c->batch, c->xmult[l] }; return t; }
static tensor_t w_tensor(const chain_t *c, int l) { tensor_t t = { c->width[l - 1], c->width[l], c->wmult[l] }; return t; }
static tensor_t w_tensor_T(const chain_t *c, int l) { tensor_t t = { c->width[l], c->width[l - 1], c->wmult[l] }; return t; }

/* The three products of layer l.  op: 0 = F_l, 1 = B_l, 2 = G_l.
 * txp/tgp: tilings of x_{l-1}, g_{l-1}; tw: of W_l; tx/tg: of x_l, g_l. */
static uint64_t layer_op_cost(const chain_t *c, int l, int op, int k, const uint8_t *txp, const uint8_t *tgp,
                              const uint8_t *tw, const uint8_t *tx, const uint8_t *tg, uint8_t *forms_out,
                              uint64_t *level_out)
{
    uint8_t tt[MAXK];
    int64_t b = c->batch, nin = c->width[l - 1], nout = c->width[l];
    if (op == 0) /* x_l = x_{l-1} W_l */
        return matmul_cost(act_tensor(c, l - 1), w_tensor(c, l), act_tensor(c, l), b, nin, nout, txp, tw, tx, k,
                           forms_out, level_out);
    if (op == 1) { /* g_{l-1} = g_l W_l^T */
        transpose_letters(tw, k, tt);
        return matmul_cost(act_tensor(c, l), w_tensor_T(c, l), act_tensor(c, l - 1), b, nout, nin, tg, tt, tgp, k,
                           forms_out, level_out);
    }
    /* dW_l = x_{l-1}^T g_l, stored with the tiling of W_l */
    transpose_letters(txp, k, tt);
    return matmul_cost(act_tensor_T(c, l - 1), act_tensor(c, l), w_tensor(c, l), nin, b, nout, tt, tg, tw, k, forms_out,
                       level_out);
}

static uint64_t sat_add(uint64_t a, uint64_t b) { return (a == INF || b == INF) ? INF : a + b; }

/* Eq. 3 for a k-cut graph tiling.  x, g: (L+1)*k letters; w: L*k letters (w[(l-1)*k + j]).
 * forms_out: 3*L*k (layer-major, then op F,B,G, then cut); delta_out: k per-cut costs. */
uint64_t oracle_chain_cost(const chain_t *c, int k, const uint8_t *x, const uint8_t *g, const uint8_t *w,
                           uint8_t *forms_out, uint64_t *delta_out)
{
    uint64_t total = 0, delta[MAXK] = { 0 };
    for (int l = 1; l <= c->L; ++l)
        for (int op = 0; op < 3; ++op) {
            uint8_t f[MAXK];
            uint64_t lev[MAXK];
            uint64_t v = layer_op_cost(c, l, op, k, x + (l - 1) * k, g + (l - 1) * k, w + (l - 1) * k, x + l * k,
                                       g + l * k, f, lev);
            if (v == INF) return INF;
            total += v;
            for (int j = 0; j < k; ++j) delta[j] += lev[j];
            if (forms_out) memcpy(forms_out + ((l - 1) * 3 + op) * k, f, (size_t)k);
        }
    if (delta_out) memcpy(delta_out, delta, sizeof(uint64_t) * (size_t)k);
    return total;
}

/* ------------------------------------------------------------------------
 * Brute force over every graph tiling (the planner's optimum by definition).
 * Tensor order x_0, g_0, W_1, x_1, g_1, W_2, ...; each takes all 3^k sequences.
 * Per-layer op costs are tabulated first (same matmul_cost), so that the
 * innermost loop adds one layer's three products.
 * pin_*: NULL = free, else the k letters the tensor is fixed to.
 * ------------------------------------------------------------------------ */
static void decode(int code, int k, uint8_t *t)
{
    for (int j = k - 1; j >= 0; --j) { t[j] = (uint8_t)(code % 3); code /= 3; }
}
static int encode(const uint8_t *t, int k)
{
    int code = 0;
    for (int j = 0; j < k; ++j) code = code * 3 + t[j];
    return code;
}

typedef struct {
    const chain_t *c;
    int k, n; /* n = 3^k */
    uint64_t *F[MAXL + 1], *B[MAXL + 1], *G[MAXL + 1]; /* F[l][(xp*n + w)*n + x], B[l][(g*n + w)*n + gp], G[l][(xp*n + g)*n + w] */
    int pin_xL, pin_gL;
    int prune;
} bf_t;

typedef struct { uint64_t best; int assign[3 * MAXL + 2]; int cur[3 * MAXL + 2]; } bf_state_t;

static void bf_rec(const bf_t *bf, bf_state_t *st, int l, int xp, int gp, uint64_t acc)
{
    const int n = bf->n, L = bf->c->L;
    if (l > L) {
        if (acc < st->best) { st->best = acc; memcpy(st->assign, st->cur, sizeof(st->cur)); }
        return;
    }
    for (int w = 0; w < n; ++w)
        for (int x = 0; x < n; ++x) {
            if (l == L && bf->pin_xL >= 0 && x != bf->pin_xL) continue;
            uint64_t cf = bf->F[l][((size_t)xp * n + w) * n + x];
            if (cf == INF) continue;
            for (int g = 0; g < n; ++g) {
                if (l == L && bf->pin_gL >= 0 && g != bf->pin_gL) continue;
                uint64_t cb = bf->B[l][((size_t)g * n + w) * n + gp];
                uint64_t cg = bf->G[l][((size_t)xp * n + g) * n + w];
                if (cb == INF || cg == INF) continue;
                uint64_t tot = acc + cf + cb + cg;
                if (bf->prune && tot >= st->best) continue; /* costs are non-negative */
                st->cur[2 + 3 * (l - 1)] = w;
                st->cur[3 + 3 * (l - 1)] = x;
                st->cur[4 + 3 * (l - 1)] = g;
                bf_rec(bf, st, l + 1, x, g, tot);
            }
        }
}

/* Returns the minimum cost (INF if nothing is feasible); assign_out gets the first
 * minimiser found as sequence codes in tensor order x_0,g_0,W_1,x_1,g_1,... */
uint64_t oracle_bruteforce(const chain_t *c, int k, const uint8_t *pin_x0, const uint8_t *pin_g0,
                           const uint8_t *pin_xL, const uint8_t *pin_gL, int prune, int *assign_out)
{
    bf_t bf;
    bf.c = c; bf.k = k; bf.prune = prune;
    int n = 1;
    for (int j = 0; j < k; ++j) n *= 3;
    bf.n = n;
    bf.pin_xL = pin_xL ? encode(pin_xL, k) : -1;
    bf.pin_gL = pin_gL ? encode(pin_gL, k) : -1;
    size_t n3 = (size_t)n * n * n;
    for (int l = 1; l <= c->L; ++l) {
        bf.F[l] = malloc(n3 * sizeof(uint64_t));
        bf.B[l] = malloc(n3 * sizeof(uint64_t));
        bf.G[l] = malloc(n3 * sizeof(uint64_t));
#pragma omp parallel for schedule(dynamic)
        for (int a = 0; a < n; ++a)
            for (int b = 0; b < n; ++b)
                for (int d = 0; d < n; ++d) {
                    uint8_t ta[MAXK], tb[MAXK], td[MAXK];
                    decode(a, k, ta); decode(b, k, tb); decode(d, k, td);
                    size_t idx = ((size_t)a * n + b) * n + d;
                    /* F: a = x_{l-1}, b = W, d = x_l */
                    bf.F[l][idx] = layer_op_cost(c, l, 0, k, ta, NULL, tb, td, NULL, NULL, NULL);
                    /* B: a = g_l, b = W, d = g_{l-1} */
                    bf.B[l][idx] = layer_op_cost(c, l, 1, k, NULL, td, tb, NULL, ta, NULL, NULL);
                    /* G: a = x_{l-1}, b = g_l, d = W */
                    bf.G[l][idx] = layer_op_cost(c, l, 2, k, ta, NULL, td, NULL, tb, NULL, NULL);
                }
    }
    int x0lo = 0, x0hi = n, g0lo = 0, g0hi = n;
    if (pin_x0) { x0lo = encode(pin_x0, k); x0hi = x0lo + 1; }
    if (pin_g0) { g0lo = encode(pin_g0, k); g0hi = g0lo + 1; }
    uint64_t best = INF;
    int best_assign[3 * MAXL + 2];
    memset(best_assign, 0, sizeof(best_assign));
    int npairs = (x0hi - x0lo) * (g0hi - g0lo);
#pragma omp parallel for schedule(dynamic)
    for (int p = 0; p < npairs; ++p) {
        int x0 = x0lo + p / (g0hi - g0lo), g0 = g0lo + p % (g0hi - g0lo);
        bf_state_t st;
        st.best = INF;
        memset(st.cur, 0, sizeof(st.cur));
        st.cur[0] = x0; st.cur[1] = g0;
        bf_rec(&bf, &st, 1, x0, g0, 0);
#pragma omp critical
        {
            /* keep the minimiser that comes first in enumeration order among equal costs */
            int earlier = 0;
            if (st.best == best && st.best != INF)
                for (int i = 0; i < 3 * c->L + 2; ++i)
                    if (st.assign[i] != best_assign[i]) { earlier = st.assign[i] < best_assign[i]; break; }
            if (st.best < best || earlier) {
                best = st.best;
                memcpy(best_assign, st.assign, sizeof(best_assign));
            }
        }
    }
    for (int l = 1; l <= c->L; ++l) { free(bf.F[l]); free(bf.B[l]); free(bf.G[l]); }
    if (assign_out) memcpy(assign_out, best_assign, sizeof(int) * (size_t)(3 * c->L + 2));
    return best;
}

/* ------------------------------------------------------------------------
 * Algorithm 1 taken literally: at each cut, from the outermost in, try every
 * assignment of one letter per tensor (3^(3L+2) of them), cost it with Eq. 2 on
 * the current sub-problem, keep the first minimum in lexicographic order
 * (tensor order x_0,g_0,W_1,x_1,g_1,...; R < C < r), fix each product's form to
 * its lowest-index minimising feasible form, halve shapes, go on.
 * Total = sum_j 2^j delta_j (Theorem 1).
 * ------------------------------------------------------------------------ */
typedef struct { int64_t M, K, N; } dims_t;

static uint64_t onecut_matmul(tensor_t X, tensor_t Y, tensor_t Z, dims_t d, int lx, int ly, int lz, int *form_out)
{
    /* letter feasibility on the current tiles */
    if ((lx == L_R && (X.rows & 1)) || (lx == L_C && (X.cols & 1))) return INF;
    if ((ly == L_R && (Y.rows & 1)) || (ly == L_C && (Y.cols & 1))) return INF;
    if ((lz == L_R && (Z.rows & 1)) || (lz == L_C && (Z.cols & 1))) return INF;
    uint64_t Ax = (uint64_t)X.rows * X.cols * X.mult, Ay = (uint64_t)Y.rows * Y.cols * Y.mult,
             Az = (uint64_t)Z.rows * Z.cols * Z.mult;
    uint64_t best = INF;
    for (int f = 0; f < 3; ++f) {
        int64_t dim = f == 0 ? d.M : (f == 1 ? d.N : d.K);
        if (dim & 1) continue;
        uint64_t v = eq2_term(f, lx, ly, lz, Ax, Ay, Az);
        if (v < best) { best = v; if (form_out) *form_out = f; }
    }
    return best;
}

static tensor_t cut_tensor(tensor_t T, int letter)
{
    if (letter == L_R) T.rows >>= 1;
    else if (letter == L_C) T.cols >>= 1;
    return T;
}
static tensor_t transposed(tensor_t T) { tensor_t o = { T.cols, T.rows, T.mult }; return o; }
static int tr_letter(int l) { return l == L_R ? L_C : (l == L_C ? L_R : L_r); }

/* x_out, g_out: (L+1)*k letters, w_out: L*k letters, delta_out: k.
 * pins as in oracle_bruteforce (k letters each, cut j uses letter j). */
uint64_t oracle_recursive(const chain_t *c, int k, const uint8_t *pin_x0, const uint8_t *pin_g0,
                          const uint8_t *pin_xL, const uint8_t *pin_gL, uint8_t *x_out, uint8_t *g_out,
                          uint8_t *w_out, uint64_t *delta_out)
{
    const int L = c->L, nt = 3 * L + 2;
    tensor_t X[MAXL + 1], Gt[MAXL + 1], W[MAXL + 1];
    dims_t dF[MAXL + 1], dB[MAXL + 1], dG[MAXL + 1];
    for (int l = 0; l <= L; ++l) { X[l] = act_tensor(c, l); Gt[l] = act_tensor(c, l); }
    for (int l = 1; l <= L; ++l) {
        W[l] = w_tensor(c, l);
        dims_t f = { c->batch, c->width[l - 1], c->width[l] }; dF[l] = f;
        dims_t b = { c->batch, c->width[l], c->width[l - 1] }; dB[l] = b;
        dims_t g = { c->width[l - 1], c->batch, c->width[l] }; dG[l] = g;
    }
    uint64_t total = 0;
    for (int j = 0; j < k; ++j) {
        uint64_t best = INF;
        int best_let[3 * MAXL + 2], let[3 * MAXL + 2];
        long ncomb = 1;
        for (int i = 0; i < nt; ++i) ncomb *= 3;
        for (long code = 0; code < ncomb; ++code) {
            long cc = code;
            for (int i = nt - 1; i >= 0; --i) { let[i] = (int)(cc % 3); cc /= 3; }
            if (pin_x0 && let[0] != pin_x0[j]) continue;
            if (pin_g0 && let[1] != pin_g0[j]) continue;
            if (pin_xL && let[3 + 3 * (L - 1)] != pin_xL[j]) continue;
            if (pin_gL && let[4 + 3 * (L - 1)] != pin_gL[j]) continue;
            uint64_t tot = 0;
            for (int l = 1; l <= L && tot != INF; ++l) {
                int lxp = l == 1 ? let[0] : let[3 + 3 * (l - 2)], lgp = l == 1 ? let[1] : let[4 + 3 * (l - 2)];
                int lw = let[2 + 3 * (l - 1)], lx = let[3 + 3 * (l - 1)], lg = let[4 + 3 * (l - 1)];
                tot = sat_add(tot, onecut_matmul(X[l - 1], W[l], X[l], dF[l], lxp, lw, lx, NULL));
                tot = sat_add(tot, onecut_matmul(Gt[l], transposed(W[l]), Gt[l - 1], dB[l], lg, tr_letter(lw), lgp, NULL));
                tot = sat_add(tot, onecut_matmul(transposed(X[l - 1]), Gt[l], W[l], dG[l], tr_letter(lxp), lg, lw, NULL));
            }
            if (tot < best) { best = tot; memcpy(best_let, let, sizeof(let)); }
        }
        if (best == INF) return INF;
        delta_out[j] = best;
        total += best << j;
        /* record letters, fix forms, build the sub-problem */
        for (int l = 1; l <= L; ++l) {
            int lxp = l == 1 ? best_let[0] : best_let[3 + 3 * (l - 2)], lgp = l == 1 ? best_let[1] : best_let[4 + 3 * (l - 2)];
            int lw = best_let[2 + 3 * (l - 1)], lx = best_let[3 + 3 * (l - 1)], lg = best_let[4 + 3 * (l - 1)];
            int f = 0;
            onecut_matmul(X[l - 1], W[l], X[l], dF[l], lxp, lw, lx, &f);
            if (f == 0) dF[l].M >>= 1; else if (f == 1) dF[l].N >>= 1; else dF[l].K >>= 1;
            onecut_matmul(Gt[l], transposed(W[l]), Gt[l - 1], dB[l], lg, tr_letter(lw), lgp, &f);
            if (f == 0) dB[l].M >>= 1; else if (f == 1) dB[l].N >>= 1; else dB[l].K >>= 1;
            onecut_matmul(transposed(X[l - 1]), Gt[l], W[l], dG[l], tr_letter(lxp), lg, lw, &f);
            if (f == 0) dG[l].M >>= 1; else if (f == 1) dG[l].N >>= 1; else dG[l].K >>= 1;
        }
        x_out[j] = (uint8_t)best_let[0];
        g_out[j] = (uint8_t)best_let[1];
        for (int l = 1; l <= L; ++l) {
            w_out[(l - 1) * k + j] = (uint8_t)best_let[2 + 3 * (l - 1)];
            x_out[l * k + j] = (uint8_t)best_let[3 + 3 * (l - 1)];
            g_out[l * k + j] = (uint8_t)best_let[4 + 3 * (l - 1)];
        }
        X[0] = cut_tensor(X[0], best_let[0]);
        Gt[0] = cut_tensor(Gt[0], best_let[1]);
        for (int l = 1; l <= L; ++l) {
            W[l] = cut_tensor(W[l], best_let[2 + 3 * (l - 1)]);
            X[l] = cut_tensor(X[l], best_let[3 + 3 * (l - 1)]);
            Gt[l] = cut_tensor(Gt[l], best_let[4 + 3 * (l - 1)]);
        }
    }
    return total;
}

/* single Eq. 2 evaluation for one cut, exposed for the k = 1 pins */
uint64_t oracle_eq2_term(int form, int lx, int ly, int lz, uint64_t Ax, uint64_t Ay, uint64_t Az)
{
    return eq2_term(form, lx, ly, lz, Ax, Ay, Az);
}
uint64_t oracle_conv_cost(int from, int to, uint64_t A) { return conv_cost(from, to, A); }
