// Tiling search on a general dataflow graph (arXiv 1805.04170 Sec. 4.2.2: operators organised into breadth-first
// levels and the dynamic program of Eqs. 4-5 over the tensors shared by adjacent levels; Sec. 4.3: Algorithm 1 and
// Theorem 1; Sec. 4.5: tensors with d dimensions - one basic tiling per dimension plus replication - and operators
// other than products, which differ only in their sets of aligned tilings).
//
// Cost model: the one of planner.cpp with dimension indices in place of the letters R and C.  Conversion of a tile with
// A elements: same letter 0; cut -> other cut A/2; cut -> replicated A; replicated -> anything 0; partial sums -> cut A,
// -> replicated 2A.  Cut j prices the tiles left by cuts 0..j-1 with weight 2^j.  A letter needs an even extent, a form
// needs an even extent of the dimension it halves.  An operator costs the minimum over its feasible form sequences.
//
// Aligned forms:
//   contraction z = x (.) y with (m: dim of x, dim of z), (n: dim of y, dim of z), (k: dim of x, dim of y):
//       form 0: x cut along m, y replicated, z cut along m;  form 1: x replicated, y cut along n, z cut along n;
//       form 2: x and y cut along k, z = partial sums
//   element-wise (same shape everywhere): one form per dimension, every operand cut along it
//   batch-only (any other operator): every operand cut along dimension 0
//   per sample and channel (pooling; flattening channel-major images): every operand cut along dimension 0, or every
//       operand along dimension 1 - a column cut of the flattened matrix is a channel cut while the channel count is even
#include <algorithm>
#include <cstring>
#include <limits>
#include <new>
#include <vector>

#include "tt_internal.h"

struct tt_graph_plan {
    int k = 0, n_tensors = 0, n_ops = 0, n_levels = 0;
    uint64_t cost = 0;
    uint64_t delta[TT_MAX_K] = {};
    std::vector<uint8_t> letters; // n_tensors * k
    std::vector<uint8_t> forms;   // n_ops * k
    std::vector<int> level;       // n_ops
};

namespace tt {
namespace {

constexpr uint64_t kInf = std::numeric_limits<uint64_t>::max();
constexpr uint8_t kRep = TT_LETTER_REP, kRedL = 254;
constexpr int kMaxOperands = TT_GRAPH_MAX_INPUTS + 1;
constexpr int kMaxForms = TT_GRAPH_MAX_DIMS;

inline uint64_t add_sat(uint64_t a, uint64_t b) { return (a == kInf || b == kInf) ? kInf : a + b; }

inline uint64_t convert_cost(uint8_t from, uint8_t to, uint64_t area)
{
    if (from == kRep) return 0;
    if (from == kRedL) return to == kRep ? 2 * area : area;
    if (from == to) return 0;
    if (to == kRep) return area;
    return area / 2;
}

struct Var { // one tiling variable: a tensor and everything declared to be stored like it
    int ndim = 0;
    int64_t shape[TT_GRAPH_MAX_DIMS] = {};
};

struct Form {
    uint8_t in[TT_GRAPH_MAX_INPUTS];
    uint8_t out;
};

struct Op {
    int n_in = 0;
    int var[kMaxOperands];  // inputs, then the output
    int n_forms = 0;
    Form form[kMaxForms];
    int64_t extent[kMaxForms]; // the extent form f halves
};

struct Graph {
    std::vector<Var> vars;
    std::vector<int> var_of; // tensor -> variable
    std::vector<Op> ops;
};

uint64_t area_of(const Var &v)
{
    uint64_t a = 1;
    for (int d = 0; d < v.ndim; ++d) a *= (uint64_t)v.shape[d];
    return a;
}

tt_status build_graph(const tt_graph_tensor *tensors, int n_tensors, const tt_graph_op *ops, int n_ops, Graph *g)
{
    if (!tensors || !ops || n_tensors < 1 || n_ops < 1 || n_tensors > TT_GRAPH_MAX_TENSORS || n_ops > TT_GRAPH_MAX_OPS)
        return TT_EINVAL;
    g->var_of.assign(n_tensors, -1);
    for (int i = 0; i < n_tensors; ++i) {
        const tt_graph_tensor &t = tensors[i];
        if (t.ndim < 1 || t.ndim > TT_GRAPH_MAX_DIMS) return TT_EINVAL;
        uint64_t a = 1;
        for (int d = 0; d < t.ndim; ++d) {
            if (t.shape[d] <= 0) return TT_EINVAL;
            if (a > (uint64_t(1) << 44) / (uint64_t)t.shape[d]) return TT_EUNSUPPORTED; // summed, weighted costs stay below 2^64
            a *= (uint64_t)t.shape[d];
        }
        if (t.same_as >= 0) {
            if (t.same_as >= i) return TT_EINVAL;
            const tt_graph_tensor &o = tensors[t.same_as];
            if (o.ndim != t.ndim || std::memcmp(o.shape, t.shape, sizeof(int64_t) * (size_t)t.ndim)) return TT_EINVAL;
            g->var_of[i] = g->var_of[t.same_as];
        } else {
            Var v;
            v.ndim = t.ndim;
            std::memcpy(v.shape, t.shape, sizeof(int64_t) * (size_t)t.ndim);
            g->var_of[i] = (int)g->vars.size();
            g->vars.push_back(v);
        }
    }
    g->ops.resize(n_ops);
    for (int q = 0; q < n_ops; ++q) {
        const tt_graph_op &s = ops[q];
        Op &o = g->ops[q];
        if (s.n_in < 1 || s.n_in > TT_GRAPH_MAX_INPUTS || s.out < 0 || s.out >= n_tensors) return TT_EINVAL;
        for (int i = 0; i < s.n_in; ++i)
            if (s.in[i] < 0 || s.in[i] >= n_tensors) return TT_EINVAL;
        o.n_in = s.n_in;
        for (int i = 0; i < s.n_in; ++i) o.var[i] = g->var_of[s.in[i]];
        o.var[s.n_in] = g->var_of[s.out];
        const tt_graph_tensor &z = tensors[s.out];
        if (s.kind == TT_GOP_CONTRACT) {
            if (s.n_in != 2) return TT_EINVAL;
            const tt_graph_tensor &x = tensors[s.in[0]], &y = tensors[s.in[1]];
            const int mx = s.m[0], mz = s.m[1], ny = s.n[0], nz = s.n[1], kx = s.kk[0], ky = s.kk[1];
            if (mx < 0 || mx >= x.ndim || kx < 0 || kx >= x.ndim || mx == kx) return TT_EINVAL;
            if (ny < 0 || ny >= y.ndim || ky < 0 || ky >= y.ndim || ny == ky) return TT_EINVAL;
            if (mz < 0 || mz >= z.ndim || nz < 0 || nz >= z.ndim || mz == nz) return TT_EINVAL;
            if (x.shape[mx] != z.shape[mz] || y.shape[ny] != z.shape[nz] || x.shape[kx] != y.shape[ky]) return TT_EINVAL;
            o.n_forms = 3;
            o.form[0].in[0] = (uint8_t)mx; o.form[0].in[1] = kRep;        o.form[0].out = (uint8_t)mz; o.extent[0] = x.shape[mx];
            o.form[1].in[0] = kRep;        o.form[1].in[1] = (uint8_t)ny; o.form[1].out = (uint8_t)nz; o.extent[1] = y.shape[ny];
            o.form[2].in[0] = (uint8_t)kx; o.form[2].in[1] = (uint8_t)ky; o.form[2].out = kRedL;       o.extent[2] = x.shape[kx];
        } else if (s.kind == TT_GOP_ELEMENTWISE) {
            for (int i = 0; i < s.n_in; ++i) {
                const tt_graph_tensor &x = tensors[s.in[i]];
                if (x.ndim != z.ndim || std::memcmp(x.shape, z.shape, sizeof(int64_t) * (size_t)z.ndim)) return TT_EINVAL;
            }
            o.n_forms = z.ndim;
            for (int d = 0; d < z.ndim; ++d) {
                for (int i = 0; i < s.n_in; ++i) o.form[d].in[i] = (uint8_t)d;
                o.form[d].out = (uint8_t)d;
                o.extent[d] = z.shape[d];
            }
        } else if (s.kind == TT_GOP_SAMPLE_CHANNEL) {
            int64_t chans = z.ndim >= 2 ? z.shape[1] : 0;
            for (int i = 0; i < s.n_in; ++i) {
                const tt_graph_tensor &x = tensors[s.in[i]];
                if (x.ndim < 2 || z.ndim < 2 || x.shape[0] != z.shape[0]) return TT_EINVAL;
                chans = std::min(chans, x.shape[1]);
            }
            if (chans <= 0 || z.shape[1] % chans) return TT_EINVAL;
            for (int i = 0; i < s.n_in; ++i)
                if (tensors[s.in[i]].shape[1] % chans) return TT_EINVAL;
            o.n_forms = 2;
            for (int d = 0; d < 2; ++d) {
                for (int i = 0; i < s.n_in; ++i) o.form[d].in[i] = (uint8_t)d;
                o.form[d].out = (uint8_t)d;
            }
            o.extent[0] = z.shape[0];
            o.extent[1] = chans;
        } else if (s.kind == TT_GOP_BATCH) {
            for (int i = 0; i < s.n_in; ++i)
                if (tensors[s.in[i]].shape[0] != z.shape[0]) return TT_EINVAL;
            o.n_forms = 1;
            for (int i = 0; i < s.n_in; ++i) o.form[0].in[i] = 0;
            o.form[0].out = 0;
            o.extent[0] = z.shape[0];
        } else {
            return TT_EINVAL;
        }
    }
    return TT_OK;
}

bool valid_letter(uint8_t l, int ndim) { return l == kRep || l < ndim; }

// element counts of the stored tile each cut works on; false if a cut is uneven
bool tile_areas(const Var &v, const uint8_t *t, int k, uint64_t *area)
{
    int64_t s[TT_GRAPH_MAX_DIMS];
    std::memcpy(s, v.shape, sizeof(s));
    for (int j = 0; j < k; ++j) {
        uint64_t a = 1;
        for (int d = 0; d < v.ndim; ++d) a *= (uint64_t)s[d];
        area[j] = a;
        if (t[j] != kRep) {
            if (s[t[j]] & 1) return false;
            s[t[j]] >>= 1;
        }
    }
    return true;
}

int max_pow2(int64_t v, int cap)
{
    int n = 0;
    while (n < cap && (v & 1) == 0) { v >>= 1; ++n; }
    return n;
}

// cheapest feasible form sequence of one operator; t[q]: k letters of operand q, area[q]: its per-cut tile areas
uint64_t op_cost(const Op &o, int k, const uint8_t *const *t, const uint64_t (*area)[TT_MAX_K], uint8_t *forms_out,
                 uint64_t *level_out)
{
    const int nq = o.n_in + 1;
    uint64_t c[TT_MAX_K][kMaxForms];
    for (int j = 0; j < k; ++j)
        for (int f = 0; f < o.n_forms; ++f) {
            uint64_t v = convert_cost(o.form[f].out, t[nq - 1][j], area[nq - 1][j]);
            for (int q = 0; q < o.n_in; ++q) v += convert_cost(t[q][j], o.form[f].in[q], area[q][j]);
            c[j][f] = v;
        }
    int cap[kMaxForms];
    for (int f = 0; f < o.n_forms; ++f) cap[f] = max_pow2(o.extent[f], k);
    // cheapest form per cut (lowest index on ties) if that respects the divisibility caps, else full search
    uint8_t pick[TT_MAX_K];
    int cnt[kMaxForms] = {};
    uint64_t total = 0;
    bool ok = true;
    for (int j = 0; j < k; ++j) {
        int f = 0;
        for (int e = 1; e < o.n_forms; ++e)
            if (c[j][e] < c[j][f]) f = e;
        pick[j] = (uint8_t)f;
        total += c[j][f] << j;
        if (++cnt[f] > cap[f]) ok = false;
    }
    if (!ok) {
        uint64_t best = kInf;
        uint8_t cur[TT_MAX_K], arg[TT_MAX_K] = {};
        int used[kMaxForms] = {};
        // depth-first over form sequences, lexicographic order, first minimum kept
        struct Rec {
            const Op &o; int k; const uint64_t (*c)[kMaxForms]; const int *cap; int *used; uint8_t *cur, *arg; uint64_t *best;
            void go(int j, uint64_t acc)
            {
                if (j == k) { if (acc < *best) { *best = acc; std::memcpy(arg, cur, (size_t)k); } return; }
                for (int f = 0; f < o.n_forms; ++f) {
                    if (used[f] + 1 > cap[f]) continue;
                    ++used[f];
                    cur[j] = (uint8_t)f;
                    go(j + 1, acc + (c[j][f] << j));
                    --used[f];
                }
            }
        } rec{o, k, c, cap, used, cur, arg, &best};
        rec.go(0, 0);
        if (best == kInf) return kInf;
        total = best;
        std::memcpy(pick, arg, (size_t)k);
    }
    if (forms_out) std::memcpy(forms_out, pick, (size_t)k);
    if (level_out)
        for (int j = 0; j < k; ++j) level_out[j] = c[j][pick[j]];
    return total;
}

// ---- levels (Sec. 4.2.2): breadth-first search over the operators, two operators being adjacent when they share a
// tiling variable.  Operators that share a variable end up in the same or in adjacent levels.
void bfs_levels(const Graph &g, std::vector<int> *level, int *n_levels)
{
    const int n = (int)g.ops.size(), nv = (int)g.vars.size();
    std::vector<std::vector<int>> users(nv);
    for (int q = 0; q < n; ++q)
        for (int i = 0; i <= g.ops[q].n_in; ++i) users[g.ops[q].var[i]].push_back(q);
    level->assign(n, -1);
    int next_level = 0;
    for (int root = 0; root < n; ++root) {
        if ((*level)[root] >= 0) continue;
        std::vector<int> frontier{root};
        (*level)[root] = next_level;
        while (!frontier.empty()) {
            std::vector<int> nxt;
            for (int q : frontier)
                for (int i = 0; i <= g.ops[q].n_in; ++i)
                    for (int u : users[g.ops[q].var[i]])
                        if ((*level)[u] < 0) { (*level)[u] = (*level)[q] + 1; nxt.push_back(u); }
            ++next_level;
            frontier.swap(nxt);
        }
    }
    *n_levels = next_level;
}

// ---- Eqs. 4-5 over the levels, used for every single cut of Algorithm 1.  Every variable has a domain of candidate
// letters; cost(q, idx) prices operator q when its operands take the candidates idx[0..n_in].  Returns the optimum
// and one optimal candidate per variable (the first found in a fixed enumeration order).
struct LevelSearch {
    const Graph &g;
    const std::vector<int> &level;
    int n_levels;
    std::vector<int> dom; // candidates per variable

    template <class CostFn> tt_status run(CostFn &&cost, uint64_t *opt, std::vector<int> *choice) const
    {
        const int nv = (int)g.vars.size(), nops = (int)g.ops.size();
        std::vector<int> first(nv, n_levels), last(nv, -1);
        for (int q = 0; q < nops; ++q)
            for (int i = 0; i <= g.ops[q].n_in; ++i) {
                const int v = g.ops[q].var[i];
                first[v] = std::min(first[v], level[q]);
                last[v] = std::max(last[v], level[q]);
            }
        choice->assign(nv, 0);
        for (int v = 0; v < nv; ++v)
            if (dom[v] < 1) return TT_EINFEASIBLE;

        // per level: the variables it touches (those shared with the previous level first), the shared ones after it
        std::vector<std::vector<int>> touched(n_levels), carry(n_levels);
        for (int l = 0; l < n_levels; ++l) {
            for (int v = 0; v < nv; ++v)
                if (first[v] < l && last[v] >= l) touched[l].push_back(v);
            for (int v = 0; v < nv; ++v)
                if (first[v] == l) touched[l].push_back(v);
            for (int v = 0; v < nv; ++v)
                if (first[v] <= l && last[v] > l) carry[l].push_back(v);
        }
        auto space = [&](const std::vector<int> &vs, uint64_t *n) {
            uint64_t s = 1;
            for (int v : vs) {
                if (s > (uint64_t(1) << 28) / (uint64_t)dom[v]) return false; // more states than a search should walk through
                s *= (uint64_t)dom[v];
            }
            *n = s;
            return true;
        };
        std::vector<uint64_t> prev(1, 0); // table over carry[l-1]
        std::vector<std::vector<uint32_t>> back(n_levels); // per carry state of level l: best state of touched[l]
        std::vector<int> pos(nv, -1), val(nv, 0);
        for (int l = 0; l < n_levels; ++l) {
            uint64_t n_touch = 0, n_carry = 0;
            if (!space(touched[l], &n_touch) || !space(carry[l], &n_carry)) return TT_EUNSUPPORTED;
            std::vector<uint64_t> cur(n_carry, kInf);
            back[l].assign(n_carry, 0);
            std::vector<int> ops_here;
            for (int q = 0; q < nops; ++q)
                if (level[q] == l) ops_here.push_back(q);
            const std::vector<int> &tv = touched[l];
            const std::vector<int> &pv = l > 0 ? carry[l - 1] : carry[l]; // (unused for l = 0)
            std::fill(val.begin(), val.end(), 0);
            for (uint64_t s = 0; s < n_touch; ++s) {
                // decode the mixed-radix state (last variable fastest)
                uint64_t r = s;
                for (int i = (int)tv.size() - 1; i >= 0; --i) { val[tv[i]] = (int)(r % (uint64_t)dom[tv[i]]); r /= (uint64_t)dom[tv[i]]; }
                uint64_t c = 0;
                if (l > 0) {
                    uint64_t pi = 0;
                    for (int v : pv) pi = pi * (uint64_t)dom[v] + (uint64_t)val[v];
                    c = prev[pi];
                    if (c == kInf) continue;
                }
                for (int q : ops_here) {
                    int idx[kMaxOperands];
                    for (int i = 0; i <= g.ops[q].n_in; ++i) idx[i] = val[g.ops[q].var[i]];
                    c = add_sat(c, cost(q, idx));
                    if (c == kInf) break;
                }
                if (c == kInf) continue;
                uint64_t ci = 0;
                for (int v : carry[l]) ci = ci * (uint64_t)dom[v] + (uint64_t)val[v];
                if (c < cur[ci]) { cur[ci] = c; back[l][ci] = (uint32_t)s; }
            }
            prev.swap(cur);
        }
        // after the last level nothing is carried: one state
        if (prev.empty() || prev[0] == kInf) return TT_EINFEASIBLE;
        *opt = prev[0];
        // walk back: the state of touched[l] fixes its variables; the carried ones index the previous table
        uint64_t ci = 0;
        for (int l = n_levels - 1; l >= 0; --l) {
            uint64_t r = back[l][ci];
            const std::vector<int> &tv = touched[l];
            for (int i = (int)tv.size() - 1; i >= 0; --i) { (*choice)[tv[i]] = (int)(r % (uint64_t)dom[tv[i]]); r /= (uint64_t)dom[tv[i]]; }
            if (l > 0) {
                ci = 0;
                for (int v : carry[l - 1]) ci = ci * (uint64_t)dom[v] + (uint64_t)(*choice)[v];
            }
        }
        return TT_OK;
    }
};

// candidates of a variable for the exact search: every feasible k-cut sequence that agrees with the pin
struct Candidates {
    std::vector<std::vector<uint8_t>> seq;   // [variable][candidate * k + j]
    std::vector<std::vector<uint64_t>> area; // [variable][candidate * k + j]
};

void enumerate_sequences(const Graph &g, int k, const std::vector<const uint8_t *> &pin, Candidates *c)
{
    const int nv = (int)g.vars.size();
    c->seq.assign(nv, {});
    c->area.assign(nv, {});
    for (int v = 0; v < nv; ++v) {
        const Var &var = g.vars[v];
        const int nl = var.ndim + 1;
        uint64_t total = 1;
        for (int j = 0; j < k; ++j) total *= (uint64_t)nl;
        for (uint64_t code = 0; code < total; ++code) {
            uint8_t t[TT_MAX_K];
            uint64_t r = code;
            for (int j = k - 1; j >= 0; --j) { const int l = (int)(r % (uint64_t)nl); r /= (uint64_t)nl; t[j] = l == var.ndim ? kRep : (uint8_t)l; }
            if (pin[v] && std::memcmp(pin[v], t, (size_t)k)) continue;
            uint64_t a[TT_MAX_K];
            if (!tile_areas(var, t, k, a)) continue;
            c->seq[v].insert(c->seq[v].end(), t, t + k);
            c->area[v].insert(c->area[v].end(), a, a + k);
        }
    }
}

tt_status eval_graph(const Graph &g, int k, const std::vector<const uint8_t *> &t, uint64_t *cost, uint64_t *delta, uint8_t *forms)
{
    const int nv = (int)g.vars.size();
    std::vector<uint64_t> area((size_t)nv * TT_MAX_K);
    for (int v = 0; v < nv; ++v)
        if (!tile_areas(g.vars[v], t[v], k, &area[(size_t)v * TT_MAX_K])) return TT_EINFEASIBLE;
    uint64_t total = 0, d[TT_MAX_K] = {};
    for (size_t q = 0; q < g.ops.size(); ++q) {
        const Op &o = g.ops[q];
        const uint8_t *tt[kMaxOperands];
        uint64_t aa[kMaxOperands][TT_MAX_K];
        for (int i = 0; i <= o.n_in; ++i) {
            tt[i] = t[o.var[i]];
            std::memcpy(aa[i], &area[(size_t)o.var[i] * TT_MAX_K], sizeof(uint64_t) * TT_MAX_K);
        }
        uint64_t lev[TT_MAX_K];
        uint8_t f[TT_MAX_K];
        const uint64_t c = op_cost(o, k, tt, aa, f, lev);
        if (c == kInf) return TT_EINFEASIBLE;
        total += c;
        for (int j = 0; j < k; ++j) d[j] += lev[j];
        if (forms) std::memcpy(forms + q * (size_t)k, f, (size_t)k);
    }
    *cost = total;
    if (delta) std::memcpy(delta, d, sizeof(uint64_t) * (size_t)k);
    return TT_OK;
}

// ---- exact joint search over whole k-cut sequences.  Walking the joint states of a breadth-first level is hopeless
// here (a level of the layer chain touches eight tensors: 27^8 states at k = 3), so the same minimisation is done one
// tensor at a time: a variable is minimised out of the sum of the cost tables that mention it, which leaves a table over
// the variables it shared them with (the dynamic program of Eqs. 4-5 is this with whole levels minimised out at once).
// The variable whose removal leaves the smallest table goes first.
struct Factor {
    std::vector<int> vars;     // distinct, ascending
    std::vector<uint64_t> tab; // row-major over vars, last variable fastest
};

tt_status plan_exact(const Graph &g, int k, const std::vector<const uint8_t *> &pin, std::vector<std::vector<uint8_t>> *out)
{
    Candidates cand;
    enumerate_sequences(g, k, pin, &cand);
    const int nv = (int)g.vars.size();
    std::vector<int> dom(nv);
    for (int v = 0; v < nv; ++v) {
        dom[v] = k ? (int)(cand.seq[v].size() / (size_t)k) : 1;
        if (dom[v] < 1) return TT_EINFEASIBLE;
    }
    constexpr uint64_t kMaxTable = uint64_t(1) << 24, kMaxWork = uint64_t(1) << 31;
    auto table_size = [&](const std::vector<int> &vs, uint64_t limit, uint64_t *n) {
        uint64_t s = 1;
        for (int v : vs) {
            if (s > limit / (uint64_t)dom[v]) return false;
            s *= (uint64_t)dom[v];
        }
        *n = s;
        return true;
    };
    // one cost table per operator over its distinct variables
    std::vector<Factor> factors;
    for (const Op &o : g.ops) {
        Factor f;
        for (int i = 0; i <= o.n_in; ++i) f.vars.push_back(o.var[i]);
        std::sort(f.vars.begin(), f.vars.end());
        f.vars.erase(std::unique(f.vars.begin(), f.vars.end()), f.vars.end());
        uint64_t n = 0;
        if (!table_size(f.vars, kMaxTable, &n)) return TT_EUNSUPPORTED;
        f.tab.resize(n);
        std::vector<int> val(nv, 0);
        for (uint64_t s = 0; s < n; ++s) {
            uint64_t r = s;
            for (int i = (int)f.vars.size() - 1; i >= 0; --i) { val[f.vars[i]] = (int)(r % (uint64_t)dom[f.vars[i]]); r /= (uint64_t)dom[f.vars[i]]; }
            const uint8_t *tt[kMaxOperands];
            uint64_t aa[kMaxOperands][TT_MAX_K];
            for (int i = 0; i <= o.n_in; ++i) {
                tt[i] = cand.seq[o.var[i]].data() + (size_t)val[o.var[i]] * k;
                if (k > 0) std::memcpy(aa[i], cand.area[o.var[i]].data() + (size_t)val[o.var[i]] * k, sizeof(uint64_t) * (size_t)k);
            }
            f.tab[s] = op_cost(o, k, tt, aa, nullptr, nullptr);
        }
        factors.push_back(std::move(f));
    }
    struct Step { int var; std::vector<int> rest; std::vector<uint32_t> arg; };
    std::vector<Step> steps;
    std::vector<bool> gone(nv, false);
    uint64_t constant = 0;
    for (int round = 0; round < nv; ++round) {
        // the variable that leaves the smallest table
        int pickv = -1;
        uint64_t pick_size = 0;
        std::vector<int> pick_rest;
        for (int v = 0; v < nv; ++v) {
            if (gone[v]) continue;
            std::vector<int> rest;
            for (const Factor &f : factors)
                if (std::find(f.vars.begin(), f.vars.end(), v) != f.vars.end())
                    for (int u : f.vars)
                        if (u != v) rest.push_back(u);
            std::sort(rest.begin(), rest.end());
            rest.erase(std::unique(rest.begin(), rest.end()), rest.end());
            uint64_t n = 0;
            if (!table_size(rest, kMaxTable, &n)) continue;
            if (pickv < 0 || n < pick_size) { pickv = v; pick_size = n; pick_rest = rest; }
        }
        if (pickv < 0) return TT_EUNSUPPORTED; // every remaining variable would leave a table that is too large
        if (pick_size > kMaxWork / (uint64_t)dom[pickv]) return TT_EUNSUPPORTED;
        std::vector<Factor> bucket, keep;
        for (Factor &f : factors) {
            if (std::find(f.vars.begin(), f.vars.end(), pickv) != f.vars.end()) bucket.push_back(std::move(f));
            else keep.push_back(std::move(f));
        }
        Step st;
        st.var = pickv;
        st.rest = pick_rest;
        st.arg.assign(pick_size, 0);
        Factor nf;
        nf.vars = pick_rest;
        nf.tab.assign(pick_size, kInf);
        // strides of every bucket table with respect to the variables of the new table and to the one going away
        const size_t nr = pick_rest.size(), nb = bucket.size();
        std::vector<uint64_t> stride(nb * (nr + 1), 0);
        for (size_t b = 0; b < nb; ++b) {
            uint64_t s = 1;
            for (int i = (int)bucket[b].vars.size() - 1; i >= 0; --i) {
                const int u = bucket[b].vars[i];
                if (u == pickv) stride[b * (nr + 1) + nr] = s;
                else stride[b * (nr + 1) + (size_t)(std::find(pick_rest.begin(), pick_rest.end(), u) - pick_rest.begin())] = s;
                s *= (uint64_t)dom[u];
            }
        }
        std::vector<int> digit(nr, 0);
        std::vector<uint64_t> base(nb, 0);
        for (uint64_t s = 0; s < pick_size; ++s) {
            uint64_t best = kInf;
            uint32_t arg = 0;
            for (int x = 0; x < dom[pickv]; ++x) {
                uint64_t c = 0;
                for (size_t b = 0; b < nb && c != kInf; ++b) c = add_sat(c, bucket[b].tab[base[b] + (uint64_t)x * stride[b * (nr + 1) + nr]]);
                if (c < best) { best = c; arg = (uint32_t)x; }
            }
            nf.tab[s] = best;
            st.arg[s] = arg;
            // next assignment of the remaining variables (last fastest), bases updated incrementally
            for (int i = (int)nr - 1; i >= 0; --i) {
                const int u = pick_rest[i];
                if (++digit[i] < dom[u]) {
                    for (size_t b = 0; b < nb; ++b) base[b] += stride[b * (nr + 1) + (size_t)i];
                    break;
                }
                for (size_t b = 0; b < nb; ++b) base[b] -= (uint64_t)(dom[u] - 1) * stride[b * (nr + 1) + (size_t)i];
                digit[i] = 0;
            }
        }
        gone[pickv] = true;
        steps.push_back(std::move(st));
        factors.swap(keep);
        if (nf.vars.empty()) {
            if (nf.tab[0] == kInf) return TT_EINFEASIBLE;
            constant += nf.tab[0];
        } else {
            factors.push_back(std::move(nf));
        }
    }
    (void)constant;
    // back substitution in reverse order of removal
    std::vector<int> choice(nv, 0);
    for (int i = (int)steps.size() - 1; i >= 0; --i) {
        uint64_t idx = 0;
        for (int u : steps[i].rest) idx = idx * (uint64_t)dom[u] + (uint64_t)choice[u];
        choice[steps[i].var] = (int)steps[i].arg[idx];
    }
    out->assign(nv, std::vector<uint8_t>(TT_MAX_K, kRep));
    for (int v = 0; v < nv; ++v)
        for (int j = 0; j < k; ++j) (*out)[v][j] = cand.seq[v][(size_t)choice[v] * k + j];
    return TT_OK;
}

// Algorithm 1: the one-cut search on the current graph, then the same on the graph of tiles it leaves
// (delta[j]: the one-cut optimum of cut j; forms: the cheapest form of every operator at every cut, lowest index on
// ties; the plan's cost is Theorem 1's weighted sum of the deltas).
tt_status plan_recursive(Graph g, const std::vector<int> &level, int n_levels, int k,
                         const std::vector<const uint8_t *> &pin, std::vector<std::vector<uint8_t>> *out,
                         uint64_t *delta, uint8_t *forms)
{
    const int nv = (int)g.vars.size();
    out->assign(nv, std::vector<uint8_t>(TT_MAX_K, kRep));
    for (int j = 0; j < k; ++j) {
        // candidates: the letters that find an even extent (and agree with the pin)
        std::vector<std::vector<uint8_t>> letters(nv);
        for (int v = 0; v < nv; ++v)
            for (int l = 0; l <= g.vars[v].ndim; ++l) {
                const uint8_t letter = l == g.vars[v].ndim ? kRep : (uint8_t)l;
                if (pin[v] && pin[v][j] != letter) continue;
                if (letter != kRep && (g.vars[v].shape[letter] & 1)) continue;
                letters[v].push_back(letter);
            }
        LevelSearch ls{g, level, n_levels, {}};
        ls.dom.resize(nv);
        for (int v = 0; v < nv; ++v) ls.dom[v] = (int)letters[v].size();
        auto one_cut = [&](int q, const int *idx, int *form) -> uint64_t {
            const Op &o = g.ops[q];
            uint8_t t[kMaxOperands];
            uint64_t a[kMaxOperands];
            for (int i = 0; i <= o.n_in; ++i) {
                for (int e = 0; e < i; ++e)
                    if (o.var[e] == o.var[i] && idx[e] != idx[i]) return kInf;
                t[i] = letters[o.var[i]][idx[i]];
                a[i] = area_of(g.vars[o.var[i]]);
            }
            uint64_t best = kInf;
            for (int f = 0; f < o.n_forms; ++f) {
                if (o.extent[f] & 1) continue;
                uint64_t c = convert_cost(o.form[f].out, t[o.n_in], a[o.n_in]);
                for (int i = 0; i < o.n_in; ++i) c += convert_cost(t[i], o.form[f].in[i], a[i]);
                if (c < best) { best = c; if (form) *form = f; }
            }
            return best;
        };
        uint64_t opt = 0;
        std::vector<int> choice;
        tt_status st = ls.run([&](int q, const int *idx) { return one_cut(q, idx, nullptr); }, &opt, &choice);
        if (st != TT_OK) return st;
        // the graph of tiles: a cut tensor loses half of the cut dimension, an operator half of the extent its form split
        for (size_t q = 0; q < g.ops.size(); ++q) {
            int idx[kMaxOperands], f = 0;
            for (int i = 0; i <= g.ops[q].n_in; ++i) idx[i] = choice[g.ops[q].var[i]];
            one_cut((int)q, idx, &f);
            g.ops[q].extent[f] >>= 1;
            forms[q * (size_t)k + j] = (uint8_t)f;
        }
        delta[j] = opt;
        for (int v = 0; v < nv; ++v) {
            const uint8_t letter = letters[v][choice[v]];
            (*out)[v][j] = letter;
            if (letter != kRep) g.vars[v].shape[letter] >>= 1;
        }
    }
    return TT_OK;
}

tt_status read_letters(const Graph &g, const tt_graph_tensor *tensors, int n_tensors, int k, const uint8_t *letters, bool allow_free,
                       std::vector<const uint8_t *> *per_var)
{
    per_var->assign(g.vars.size(), nullptr);
    if (!letters) return allow_free ? TT_OK : TT_EINVAL;
    for (int i = 0; i < n_tensors; ++i) {
        const uint8_t *t = letters + (size_t)i * k;
        if (k > 0 && t[0] == TT_LETTER_FREE) {
            if (!allow_free) return TT_EINVAL;
            continue;
        }
        for (int j = 0; j < k; ++j)
            if (!valid_letter(t[j], tensors[i].ndim)) return TT_EINVAL;
        const uint8_t *&slot = (*per_var)[g.var_of[i]];
        if (slot && std::memcmp(slot, t, (size_t)k)) return TT_EINVAL; // two tensors stored alike, two different tilings
        slot = t;
    }
    if (!allow_free)
        for (const uint8_t *p : *per_var)
            if (!p && k > 0) return TT_EINVAL;
    return TT_OK;
}

} // namespace
} // namespace tt

extern "C" tt_status tt_plan_graph(const tt_graph_tensor *tensors, int n_tensors, const tt_graph_op *ops, int n_ops, int k,
                                   uint32_t mode, const uint8_t *pins, tt_graph_plan **out)
{
    if (!out) return TT_EINVAL;
    *out = nullptr;
    if (!tt::valid_k(k)) return TT_EINVAL;
    if (mode != TT_PLAN_EXACT && mode != TT_PLAN_RECURSIVE) return TT_EINVAL;
    try {
        tt::Graph g;
        tt_status st = tt::build_graph(tensors, n_tensors, ops, n_ops, &g);
        if (st != TT_OK) return st;
        std::vector<const uint8_t *> pin;
        st = tt::read_letters(g, tensors, n_tensors, k, pins, true, &pin);
        if (st != TT_OK) return st;
        std::vector<int> level;
        int n_levels = 0;
        tt::bfs_levels(g, &level, &n_levels);
        std::vector<std::vector<uint8_t>> t;
        uint64_t greedy_delta[TT_MAX_K] = {};
        std::vector<uint8_t> greedy_forms((size_t)n_ops * k);
        st = mode == TT_PLAN_EXACT ? tt::plan_exact(g, k, pin, &t)
                                   : tt::plan_recursive(g, level, n_levels, k, pin, &t, greedy_delta, greedy_forms.data());
        if (st != TT_OK) return st;
        tt_graph_plan *plan = new tt_graph_plan;
        plan->k = k;
        plan->n_tensors = n_tensors;
        plan->n_ops = n_ops;
        plan->n_levels = n_levels;
        plan->level = level;
        plan->letters.resize((size_t)n_tensors * k);
        for (int i = 0; i < n_tensors; ++i)
            for (int j = 0; j < k; ++j) plan->letters[(size_t)i * k + j] = t[g.var_of[i]][j];
        plan->forms.assign((size_t)n_ops * k, 0);
        std::vector<const uint8_t *> per_var(g.vars.size());
        for (size_t v = 0; v < g.vars.size(); ++v) per_var[v] = t[v].data();
        if (mode == TT_PLAN_EXACT) {
            st = tt::eval_graph(g, k, per_var, &plan->cost, plan->delta, plan->forms.data());
            if (st != TT_OK) { delete plan; return st; }
        } else {
            plan->forms = greedy_forms;
            for (int j = 0; j < k; ++j) { plan->delta[j] = greedy_delta[j]; plan->cost += greedy_delta[j] << j; }
        }
        *out = plan;
        return TT_OK;
    } catch (const std::bad_alloc &) {
        return TT_ENOMEM;
    }
}

extern "C" tt_status tt_graph_eval(const tt_graph_tensor *tensors, int n_tensors, const tt_graph_op *ops, int n_ops, int k,
                                   const uint8_t *letters, uint64_t *cost_elems, uint64_t *delta_out, uint8_t *forms_out)
{
    if (!cost_elems || !tt::valid_k(k)) return TT_EINVAL;
    try {
        tt::Graph g;
        tt_status st = tt::build_graph(tensors, n_tensors, ops, n_ops, &g);
        if (st != TT_OK) return st;
        std::vector<const uint8_t *> t;
        st = tt::read_letters(g, tensors, n_tensors, k, letters, false, &t);
        if (st != TT_OK) return st;
        static const uint8_t none[TT_MAX_K] = {};
        if (k == 0)
            for (auto &p : t) p = none;
        return tt::eval_graph(g, k, t, cost_elems, delta_out, forms_out);
    } catch (const std::bad_alloc &) {
        return TT_ENOMEM;
    }
}

extern "C" uint64_t tt_graph_plan_cost(const tt_graph_plan *p) { return p ? p->cost : 0; }
extern "C" uint64_t tt_graph_plan_delta(const tt_graph_plan *p, int cut) { return (p && cut >= 0 && cut < p->k) ? p->delta[cut] : 0; }
extern "C" int tt_graph_plan_levels(const tt_graph_plan *p) { return p ? p->n_levels : -1; }
extern "C" int tt_graph_plan_level_of(const tt_graph_plan *p, int op) { return (p && op >= 0 && op < p->n_ops) ? p->level[op] : -1; }

extern "C" tt_status tt_graph_plan_tiling(const tt_graph_plan *p, int tensor, uint8_t *letters_out)
{
    if (!p || !letters_out || tensor < 0 || tensor >= p->n_tensors) return TT_EINVAL;
    if (p->k > 0) std::memcpy(letters_out, p->letters.data() + (size_t)tensor * p->k, (size_t)p->k);
    return TT_OK;
}

extern "C" tt_status tt_graph_plan_forms(const tt_graph_plan *p, int op, uint8_t *forms_out)
{
    if (!p || !forms_out || op < 0 || op >= p->n_ops) return TT_EINVAL;
    if (p->k > 0) std::memcpy(forms_out, p->forms.data() + (size_t)op * p->k, (size_t)p->k);
    return TT_OK;
}

extern "C" void tt_graph_plan_free(tt_graph_plan *p) { delete p; }
