// One training step of a layer chain through the library's execute calls, on the host, for checking memory accesses
// without a GPU: the whole library is built for the host (address mode: every thread of every launch run in turn, the
// stand-in MFMA multiplies nothing) and linked with this driver under the address sanitizer.  Shards and the workspace
// have exactly the sizes the library asks for (the workspace exactly tt_*_workspace_bytes, 256-byte aligned), operands
// are zero, outputs start as 0x5a bytes.  Checked: every call succeeds, no access outside any buffer, every output byte
// of every layer (activations, activation gradients, weight gradients) written.
//
//   emu_step fc   batch k dtype L  w_0..w_L  relu_1..relu_L  tx_0..tx_L  tg_0..tg_L  tw_1..tw_L  (f_fwd f_dgrad f_wgrad)_1..L
//   emu_step conv N k C K H W R S pad relu  tX tW tY tdY tdX  f_fwd f_dgrad f_wgrad
// tilings: letters R, C, r, one per cut ("-" for no cut); forms: digits 1..3, one per cut ("-": the library's default)
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>
#include "tensor_tiling.h"

// the buffers live until the process ends
extern "C" const char *__asan_default_options() { return "detect_leaks=0"; }

namespace {

struct Shards {
    std::vector<void *> p;
    size_t bytes = 0;
    const void *const *in() const { return p.data(); }
    void *const *out() const { return p.data(); }
};

tt_tiling tiling_of(const std::string &s, int k)
{
    tt_tiling t;
    std::memset(&t, 0, sizeof(t));
    if ((int)(s == "-" ? 0 : s.size()) != k) { std::fprintf(stderr, "tiling %s does not have %d cuts\n", s.c_str(), k); std::exit(64); }
    for (int j = 0; j < k; ++j) t.cut[j] = s[j] == 'R' ? TT_R : s[j] == 'C' ? TT_C : TT_REP;
    return t;
}

std::vector<uint8_t> forms_of(const std::string &s, int k)
{
    std::vector<uint8_t> f;
    if (s == "-") return f;
    if ((int)s.size() != k) { std::fprintf(stderr, "forms %s do not have %d cuts\n", s.c_str(), k); std::exit(64); }
    for (char c : s) f.push_back((uint8_t)(c - '1'));   // TT_F1 = 0
    return f;
}
const uint8_t *ptr(const std::vector<uint8_t> &f) { return f.empty() ? nullptr : f.data(); }

Shards make(int64_t rows, int64_t cols, tt_tiling t, int k, size_t elem, int fill)
{
    int64_t sr = 0, sc = 0;
    if (tt_shard_shape(rows, cols, t, k, &sr, &sc) != TT_OK) { std::fprintf(stderr, "infeasible tiling\n"); std::exit(65); }
    Shards s;
    s.bytes = (size_t)sr * (size_t)sc * elem;
    for (int i = 0; i < (1 << k); ++i) {
        void *m = std::malloc(s.bytes ? s.bytes : 1);
        std::memset(m, fill, s.bytes);
        s.p.push_back(m);
    }
    return s;
}

bool all_written(const Shards &s, const char *what, int layer)
{
    for (size_t i = 0; i < s.p.size(); ++i) {
        const unsigned char *b = static_cast<const unsigned char *>(s.p[i]);
        for (size_t j = 0; j < s.bytes; ++j)
            if (b[j] != 0) { std::printf("%s of layer %d: shard %zu byte %zu never written\n", what, layer, i, j); return false; }
    }
    return true;
}

// EMU_WS_LIE=n: the workspace is n bytes shorter than the calls are told (self-check of the checker: the sanitizer
// must report the launches that use its end)
void *workspace(size_t bytes)
{
    const char *lie = std::getenv("EMU_WS_LIE");
    const size_t shorter = lie ? (size_t)std::atol(lie) : 0;
    void *w = nullptr;
    if (posix_memalign(&w, 256, bytes > shorter ? bytes - shorter : 1) != 0) std::exit(66);
    return w;
}

#define OK(call) do { const tt_status st_ = (call); if (st_ != TT_OK) { std::printf("%s: %s\n", #call, tt_strerror(st_)); return 2; } } while (0)

int run_fc(int argc, char **argv)
{
    int a = 2;
    const int64_t batch = std::atol(argv[a++]);
    const int k = std::atoi(argv[a++]);
    const int dtype = std::strcmp(argv[a++], "bf16") == 0 ? TT_BF16 : TT_F32;
    const size_t e = dtype == TT_BF16 ? 2 : 4;
    const int L = std::atoi(argv[a++]);
    if (argc != 6 + (L + 1) + L + 2 * (L + 1) + L + 3 * L) { std::fprintf(stderr, "fc: wrong number of arguments\n"); return 64; }
    std::vector<int64_t> w(L + 1);
    for (auto &v : w) v = std::atol(argv[a++]);
    std::vector<int> relu(L);
    for (auto &v : relu) v = std::atoi(argv[a++]);
    std::vector<tt_tiling> tx(L + 1), tg(L + 1), tw(L);
    for (auto &t : tx) t = tiling_of(argv[a++], k);
    for (auto &t : tg) t = tiling_of(argv[a++], k);
    for (auto &t : tw) t = tiling_of(argv[a++], k);
    std::vector<std::vector<uint8_t>> f(3 * L);
    for (auto &v : f) v = forms_of(argv[a++], k);

    std::vector<tt_layer> lay(L);
    std::vector<Shards> x(L + 1), g(L + 1), W(L), dW(L);
    for (int l = 0; l <= L; ++l) {
        x[l] = make(batch, w[l], tx[l], k, e, l == 0 ? 0 : 0x5a);
        g[l] = make(batch, w[l], tg[l], k, e, l == L ? 0 : 0x5a);
    }
    size_t need = 0;
    for (int l = 0; l < L; ++l) {
        std::memset(&lay[l], 0, sizeof(tt_layer));
        lay[l].kind = TT_FC;
        lay[l].act = relu[l] ? TT_ACT_RELU : TT_ACT_NONE;
        lay[l].n_in = w[l];
        lay[l].n_out = w[l + 1];
        W[l] = make(w[l], w[l + 1], tw[l], k, e, 0);
        dW[l] = make(w[l], w[l + 1], tw[l], k, e, 0x5a);
        size_t b = 0;
        OK(tt_fc_workspace_bytes(&lay[l], batch, k, dtype, TT_OP_FWD, tx[l], tw[l], tx[l + 1], tg[l + 1], tg[l], ptr(f[3 * l]), nullptr, 1, &b));
        if (b > need) need = b;
        OK(tt_fc_workspace_bytes(&lay[l], batch, k, dtype, TT_OP_DGRAD, tx[l], tw[l], tx[l + 1], tg[l + 1], tg[l], ptr(f[3 * l + 1]), ptr(f[3 * l + 2]), 1, &b));
        if (b > need) need = b;
    }
    void *ws = workspace(need);
    void *stream = nullptr, *aux = reinterpret_cast<void *>(0x10);   // two distinct streams: the overlapped backward's own path
    for (int l = 0; l < L; ++l)
        OK(tt_fc_forward(&lay[l], batch, k, dtype, tx[l], tw[l], tx[l + 1], ptr(f[3 * l]), x[l].in(), W[l].in(), x[l + 1].out(), ws, need, stream));
    for (int l = L - 1; l >= 0; --l)
        OK(tt_fc_backward_overlapped(&lay[l], batch, k, dtype, tx[l], tw[l], tx[l + 1], tg[l + 1], tg[l], ptr(f[3 * l + 1]), ptr(f[3 * l + 2]),
                                     x[l].in(), W[l].in(), x[l + 1].in(), g[l + 1].in(), g[l].out(), dW[l].out(), ws, need, stream, aux));
    for (int l = 0; l < L; ++l)
        if (!all_written(x[l + 1], "activations", l + 1) || !all_written(g[l], "activation gradients", l) || !all_written(dW[l], "weight gradients", l + 1))
            return 1;
    std::printf("ok fc step: %d layers, workspace %zu bytes\n", L, need);
    return 0;
}

int run_conv(int argc, char **argv)
{
    if (argc != 20) { std::fprintf(stderr, "conv: wrong number of arguments\n"); return 64; }
    int a = 2;
    const int64_t N = std::atol(argv[a++]);
    const int k = std::atoi(argv[a++]);
    tt_layer lay;
    std::memset(&lay, 0, sizeof(lay));
    lay.kind = TT_CONV2D;
    lay.n_in = std::atol(argv[a++]);
    lay.n_out = std::atol(argv[a++]);
    lay.H = std::atol(argv[a++]);
    lay.W = std::atol(argv[a++]);
    lay.R = std::atol(argv[a++]);
    lay.S = std::atol(argv[a++]);
    lay.pad = std::atol(argv[a++]);
    lay.act = std::atoi(argv[a++]) ? TT_ACT_RELU : TT_ACT_NONE;
    const std::string sW = argv[a + 1];
    const tt_tiling tX = tiling_of(argv[a], k), tW = tiling_of(sW, k), tY = tiling_of(argv[a + 2], k), tdY = tiling_of(argv[a + 3], k),
                    tdX = tiling_of(argv[a + 4], k);
    a += 5;
    std::string sWs = sW;                       // letters on the (K*R*S) x C storage matrix of the filters
    for (char &c : sWs) c = c == 'R' ? 'C' : c == 'C' ? 'R' : c;
    const tt_tiling tWs = tiling_of(sWs, k);
    const std::vector<uint8_t> f0 = forms_of(argv[a], k), f1 = forms_of(argv[a + 1], k), f2 = forms_of(argv[a + 2], k);
    const int64_t P = lay.H + 2 * lay.pad - lay.R + 1, Q = lay.W + 2 * lay.pad - lay.S + 1;
    Shards X = make(N * lay.H * lay.W, lay.n_in, tX, k, 2, 0), Wt = make(lay.n_out * lay.R * lay.S, lay.n_in, tWs, k, 2, 0),
           dY = make(N * P * Q, lay.n_out, tdY, k, 2, 0), Y = make(N * P * Q, lay.n_out, tY, k, 2, 0x5a),
           dX = make(N * lay.H * lay.W, lay.n_in, tdX, k, 2, 0x5a), dW = make(lay.n_out * lay.R * lay.S, lay.n_in, tWs, k, 2, 0x5a);
    size_t need = 0, b = 0;
    OK(tt_conv_workspace_bytes(&lay, N, k, TT_BF16, TT_OP_FWD, tX, tW, tY, tdY, tdX, ptr(f0), nullptr, 1, &need));
    OK(tt_conv_workspace_bytes(&lay, N, k, TT_BF16, TT_OP_DGRAD, tX, tW, tY, tdY, tdX, ptr(f1), ptr(f2), 1, &b));
    if (b > need) need = b;
    void *ws = workspace(need);
    OK(tt_conv_forward(&lay, N, k, TT_BF16, tX, tW, tY, ptr(f0), X.in(), Wt.in(), Y.out(), ws, need, nullptr));
    OK(tt_conv_backward(&lay, N, k, TT_BF16, tX, tW, tY, tdY, tdX, ptr(f1), ptr(f2), X.in(), Wt.in(), Y.in(), dY.in(), dX.out(), dW.out(), ws, need,
                        nullptr));
    if (!all_written(Y, "activations", 1) || !all_written(dX, "activation gradients", 0) || !all_written(dW, "weight gradients", 1)) return 1;
    std::printf("ok conv step: workspace %zu bytes\n", need);
    return 0;
}

} // namespace

int main(int argc, char **argv)
{
    if (argc >= 6 && std::strcmp(argv[1], "fc") == 0) return run_fc(argc, argv);
    if (argc >= 3 && std::strcmp(argv[1], "conv") == 0) return run_conv(argc, argv);
    std::fprintf(stderr, "usage: emu_step fc|conv ...\n");
    return 64;
}
