// Host build of the convolution kernels WITH their launch code (csrc/conv.hip compiled as it is; tt::launch_conv
// chooses tiles and grids exactly as in the library) for checking their memory accesses without a GPU.  Operands and
// outputs have exactly the shard sizes; the stand-in MFMA multiplies nothing, so the check is: no access outside any
// buffer or outside the LDS of the launch (address sanitizer), every output byte written.
#include <cstdio>
#include <cstdlib>
#include <vector>

#define TT_HOST_EMULATION 1
#include <cstdint>
namespace tt {
namespace {
alignas(16) thread_local uint16_t smem[96 * 1024]; // what the kernels' `extern __shared__ uint16_t smem[]` refers to here
}
} // namespace tt
#include "conv.hip"

namespace tt {
ProfileScope::ProfileScope(void *, int, int, int64_t, int64_t, int64_t, uint64_t, uint64_t) : slot(-1), stream(nullptr) {}
ProfileScope::~ProfileScope() {}
} // namespace tt

int main(int argc, char **argv)
{
    emu_register_lds(tt::smem, sizeof(tt::smem));
    // emu_conv op count Ns Cs Ks H W R S pad out_bf16 relu flip
    if (argc != 14) { std::fprintf(stderr, "usage: emu_conv op count Ns Cs Ks H W R S pad out_bf16 relu flip\n"); return 64; }
    const int op = std::atoi(argv[1]), count = std::atoi(argv[2]);
    const long Ns = std::atol(argv[3]), Cs = std::atol(argv[4]), Ks = std::atol(argv[5]), H = std::atol(argv[6]), W = std::atol(argv[7]);
    const long R = std::atol(argv[8]), S = std::atol(argv[9]), pad = std::atol(argv[10]);
    const bool obf = std::atoi(argv[11]) != 0;
    const int relu = std::atoi(argv[12]);
    const bool flip = std::atoi(argv[13]) != 0;
    const long P = H + 2 * pad - R + 1, Q = W + 2 * pad - S + 1;
    if (op == 3) {
        // the filter gradient with every block's reduction range cut into `parts` runs: the arguments after pad are
        // parts, shards per block, engine; the F3 cuts are taken to be the innermost ones (low id bits)
        const int parts = std::atoi(argv[11]), nred = std::atoi(argv[12]), nblk = count / nred, engine = std::atoi(argv[13]);
        int k = 0;
        while ((1 << k) < count) ++k;
        std::vector<uint8_t> blk_ids(nblk), red_ids(nred);
        for (int b = 0; b < nblk; ++b) blk_ids[b] = (uint8_t)(b * nred);
        for (int q = 0; q < nred; ++q) red_ids[q] = (uint8_t)q;
        const size_t xb = (size_t)Ns * H * W * Cs * 2, yb = (size_t)Ns * P * Q * Ks * 2, cb = (size_t)Ks * R * S * Cs * 4;
        std::vector<std::vector<char>> A(count), B(count), C(nblk * parts);
        std::vector<const void *> Ap, Bp;
        std::vector<void *> Cp;
        for (int s = 0; s < count; ++s) {
            A[s].assign(yb, 0); B[s].assign(xb, 0);
            Ap.push_back(A[s].data()); Bp.push_back(B[s].data());
        }
        for (auto &c : C) { c.assign(cb, (char)0x5a); Cp.push_back(c.data()); }
        const tt_status st = tt::launch_conv_wgrad_split(k, nblk, nred, blk_ids.data(), red_ids.data(), parts, Ap.data(), Bp.data(),
                                                         Cp.data(), Ns, Cs, Ks, H, W, R, S, pad, engine, nullptr);
        if (st != TT_OK) { std::printf("status %d\n", (int)st); return 2; }
        for (size_t b = 0; b < C.size(); ++b)
            for (size_t i = 0; i < C[b].size(); ++i)
                if (C[b][i] != 0) { std::printf("partial sum %zu byte %zu never written\n", b, i); return 1; }
        std::printf("ok conv op 3: %llu threads run\n", g_emu_threads_run);
        return 0;
    }
    const size_t x_b = (size_t)Ns * H * W * Cs * 2, y_b = (size_t)Ns * P * Q * Ks * 2, w_b = (size_t)Ks * R * S * Cs * 2;
    const size_t ob = obf ? 2 : 4;
    size_t a_b, b_b, c_b;
    if (op == TT_OP_FWD) { a_b = x_b; b_b = w_b; c_b = (size_t)Ns * P * Q * Ks * ob; }
    else if (op == TT_OP_DGRAD) { a_b = y_b; b_b = w_b; c_b = (size_t)Ns * H * W * Cs * ob; }
    else { a_b = y_b; b_b = x_b; c_b = (size_t)Ks * R * S * Cs * ob; }
    std::vector<std::vector<char>> A(count), B(count), C(count), F(count);
    std::vector<const void *> Ap, Bp;
    std::vector<void *> Cp, Fp;
    for (int s = 0; s < count; ++s) {
        A[s].assign(a_b, 0); B[s].assign(b_b, 0); C[s].assign(c_b, (char)0x5a); F[s].assign(w_b, 0);
        Ap.push_back(A[s].data()); Bp.push_back(B[s].data()); Cp.push_back(C[s].data()); Fp.push_back(F[s].data());
    }
    const tt_status st = tt::launch_conv(op, count, Ap.data(), Bp.data(), Cp.data(), Ns, Cs, Ks, H, W, R, S, pad, obf ? TT_BF16 : TT_F32,
                                         relu ? TT_ACT_RELU : TT_ACT_NONE, nullptr, flip ? Fp.data() : nullptr);
    if (st != TT_OK) { std::printf("status %d\n", (int)st); return 2; }
    for (int s = 0; s < count; ++s)
        for (size_t i = 0; i < C[s].size(); ++i)
            if (C[s][i] != 0) { std::printf("output %d byte %zu never written\n", s, i); return 1; }
    std::printf("ok conv op %d: %llu threads run\n", op, g_emu_threads_run);
    return 0;
}
