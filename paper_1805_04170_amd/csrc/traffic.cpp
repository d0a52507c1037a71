// Elements that cross from one shard to another during the conversions of a tiled product: what the execution really
// moves between devices, counted block by block (arXiv 1805.04170 Sec. 4.2.1: a device fetches the part of its
// aligned tile that it does not already hold - ghost area minus held area; for the third aligned form every device
// fetches the other devices' partial sums of the elements it is to store).  Host arithmetic only.
//
// For one cut this count IS the planner's cost (Eq. 2); for several cuts the planner's cost is the paper's recursive
// model (cut j prices the tiles left by the earlier cuts, weight 2^j), which is not the same number: the two are
// reported side by side, and equality is only claimed at k = 1.
#include <cstring>

#include "tt_internal.h"

namespace tt {
namespace {

// overlap of two dyadic intervals of [0, n): interval ia of 2^pa equal parts, interval ib of 2^pb equal parts
inline uint64_t overlap(int64_t n, int pa, uint32_t ia, int pb, uint32_t ib)
{
    if (pa <= pb) return (ib >> (pb - pa)) == ia ? (uint64_t)(n >> pb) : 0;
    return (ia >> (pa - pb)) == ib ? (uint64_t)(n >> pa) : 0;
}

// elements of shard s's block under `to` that lie inside the same shard's block under `from`
inline uint64_t held(const Grid &from, const Grid &to, uint32_t s)
{
    const int k = to.k;
    return overlap(to.rows, from.kR, extract(s, from.maskR, k), to.kR, extract(s, to.maskR, k)) *
           overlap(to.cols, from.kC, extract(s, from.maskC, k), to.kC, extract(s, to.maskC, k));
}

} // namespace

// letters: R, C, replicate (for `from`: kRed allowed = the shards hold different partial sums of their block)
tt_status cross_elems(int64_t rows, int64_t cols, const uint8_t *from, const uint8_t *to, int k, uint64_t mult, uint64_t *out)
{
    Grid A, B;
    if (!make_grid(from, k, rows, cols, &A) || !make_grid(to, k, rows, cols, &B)) return TT_EINFEASIBLE;
    int k3 = 0;
    for (int j = 0; j < k; ++j) k3 += from[j] == kRed;
    const uint64_t block = (uint64_t)B.srows * (uint64_t)B.scols;
    uint64_t total = 0;
    for (uint32_t s = 0; s < (1u << k); ++s) {
        // every element of the destination block is needed once per partial sum; what the shard made itself stays
        total += (block << k3) - held(A, B, s);
    }
    *out = total * mult;
    return TT_OK;
}

} // namespace tt

extern "C" tt_status tt_conversion_cross_elems(int64_t rows, int64_t cols, tt_tiling from, tt_tiling to, int k, uint64_t *elems)
{
    if (!elems || !tt::valid_k(k) || rows <= 0 || cols <= 0) return TT_EINVAL;
    if (!tt::valid_tiling(from, k) || !tt::valid_tiling(to, k)) return TT_EINVAL;
    return tt::cross_elems(rows, cols, from.cut, to.cut, k, 1, elems);
}

extern "C" tt_status tt_product_cross_elems(int64_t M, int64_t K, int64_t N, tt_tiling tX, tt_tiling tY, tt_tiling tZ,
                                            const uint8_t *forms, int k, uint64_t mult_x, uint64_t mult_y, uint64_t mult_z,
                                            uint64_t *elems)
{
    if (!elems || !forms || !tt::valid_k(k) || M <= 0 || K <= 0 || N <= 0) return TT_EINVAL;
    if (!tt::valid_tiling(tX, k) || !tt::valid_tiling(tY, k) || !tt::valid_tiling(tZ, k)) return TT_EINVAL;
    int n[3] = {0, 0, 0};
    for (int j = 0; j < k; ++j) {
        if (forms[j] > TT_F3) return TT_EINVAL;
        n[forms[j]]++;
    }
    if (M % (int64_t(1) << n[0]) || N % (int64_t(1) << n[1]) || K % (int64_t(1) << n[2])) return TT_EINFEASIBLE;
    tt_tiling aX, aY;
    uint8_t aZ[TT_MAX_K];
    tt::aligned_tilings(forms, k, &aX, &aY, aZ);
    tt_status st = tt::cross_elems(M, K, tX.cut, aX.cut, k, mult_x, &elems[0]);
    if (st != TT_OK) return st;
    st = tt::cross_elems(K, N, tY.cut, aY.cut, k, mult_y, &elems[1]);
    if (st != TT_OK) return st;
    return tt::cross_elems(M, N, aZ, tZ.cut, k, mult_z, &elems[2]);
}

extern "C" tt_status tt_fc_chain_cross_elems(const tt_layer *layers, int n_layers, int64_t batch, int k, const tt_tiling *x,
                                             const tt_tiling *g, const tt_tiling *w, const uint8_t *forms, uint64_t *elems)
{
    if (!layers || !x || !g || !w || !forms || !elems || n_layers < 1 || n_layers > TT_MAX_LAYERS || batch <= 0) return TT_EINVAL;
    if (!tt::valid_k(k)) return TT_EINVAL;
    uint64_t total = 0;
    for (int l = 1; l <= n_layers; ++l) {
        const tt_layer &y = layers[l - 1];
        if (y.kind != TT_FC) return TT_EUNSUPPORTED;
        if (y.n_in <= 0 || y.n_out <= 0 || (l > 1 && y.n_in != layers[l - 2].n_out)) return TT_EINVAL;
        const uint8_t *f = forms + (size_t)(l - 1) * 3 * k;
        uint64_t e[3];
        // the three products in the planner's orientation (Sec. 4.2.2): x_l = x_{l-1} W_l; g_{l-1} = g_l W_l^T;
        // dW_l = x_{l-1}^T g_l, stored like W_l
        tt_status st = tt_product_cross_elems(batch, y.n_in, y.n_out, x[l - 1], w[l - 1], x[l], f, k, 1, 1, 1, e);
        if (st != TT_OK) return st;
        total += e[0] + e[1] + e[2];
        st = tt_product_cross_elems(batch, y.n_out, y.n_in, g[l], tt::transpose_tiling(w[l - 1], k), g[l - 1], f + k, k, 1, 1, 1, e);
        if (st != TT_OK) return st;
        total += e[0] + e[1] + e[2];
        st = tt_product_cross_elems(y.n_in, batch, y.n_out, tt::transpose_tiling(x[l - 1], k), g[l], w[l - 1], f + 2 * k, k, 1, 1, 1, e);
        if (st != TT_OK) return st;
        total += e[0] + e[1] + e[2];
    }
    *elems = total;
    return TT_OK;
}
