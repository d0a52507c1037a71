// Host build of the register-staged tile engine (csrc/gemm_core.h) for checking its memory accesses without a GPU; one
// kernel configuration per build (chosen with -D, as the template parameters of gemm_bf16_kernel in csrc/gemm.hip).
// Same method as emu_gemm3.cpp: every thread of every workgroup in turn, all-zero operands, every output byte must be
// written, every access is a real host access checked by the address sanitizer.
#include <cstdio>
#include <cstdlib>
#include <type_traits>
#include <vector>

#define TT_HOST_EMULATION 1
#include "gemm_core.h"
#include "tt_internal.h"

namespace tt {
} // namespace tt

using namespace tt;

#ifndef E1_BM
#error "define E1_BM E1_BN E1_WM E1_WN E1_DEPTH E1_KMASK E1_AKC E1_BKC E1_BF16 E1_VEC"
#endif

int main(int argc, char **argv)
{
    if (argc != 7) { std::fprintf(stderr, "usage: emu_gemm1 count M N K relu ksplit\n"); return 64; }
    const int count = std::atoi(argv[1]);
    const long M = std::atol(argv[2]), N = std::atol(argv[3]), K = std::atol(argv[4]);
    const int relu = std::atoi(argv[5]), ksplit = std::atoi(argv[6]);
    constexpr int BM = E1_BM, BN = E1_BN, WM = E1_WM, WN = E1_WN, DEPTH = E1_DEPTH;
    constexpr bool KMASK = E1_KMASK, A_KC = E1_AKC, B_KC = E1_BKC, OUT_BF16 = E1_BF16, VEC = E1_VEC;
    if ((K % 64 != 0) != KMASK) { std::fprintf(stderr, "K and KMASK do not match\n"); return 64; }
    const size_t out_b = OUT_BF16 ? 2 : 4;
    std::vector<std::vector<char>> A(count), B(count), C(count * ksplit);
    for (int s = 0; s < count; ++s) { A[s].assign((size_t)M * K * 2, 0); B[s].assign((size_t)K * N * 2, 0); }
    for (auto &v : C) v.assign((size_t)M * N * out_b, (char)0x5a);
    const long kchunk = ksplit == 1 ? K : ((K + ksplit - 1) / ksplit + 63) / 64 * 64;
    const int lda = A_KC ? K : M, ldb = B_KC ? K : N, ldc = N;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int total = tiles_m * tiles_n * count * ksplit;
    const int per_xcd = (total + core::kXcds - 1) / core::kXcds;
    constexpr int NT = WM * WN * 64;
    std::vector<uint16_t> lds(core::smem_bytes<BM, BN, DEPTH>() / 2);
    dev::g_lds = reinterpret_cast<char *>(lds.data());
    dev::g_lds_bytes = lds.size() * 2;
    for (unsigned b = 0; b < (unsigned)per_xcd * core::kXcds; ++b)
        for (unsigned t = 0; t < (unsigned)NT; ++t) {
            blockIdx = {b, 0, 0};
            threadIdx = {t, 0, 0};
            // the body of gemm_bf16_kernel (csrc/gemm.hip)
            const int logical = core::logical_block(per_xcd, total);
            if (logical < 0) continue;
            const int tiles = tiles_m * tiles_n;
            const int vshard = logical / tiles;
            const int tt_ = logical - vshard * tiles;
            int tm, tn;
            core::grouped_tile(tt_, tiles_m, tiles_n, &tm, &tn);
            const int shard = vshard / ksplit;
            const int kbeg = (vshard - shard * ksplit) * (int)kchunk;
            const int klen = K - kbeg < kchunk ? (int)(K - kbeg) : (int)kchunk;
            using LA = std::conditional_t<A_KC, core::DenseKC<core::Slots<BM, true, NT>::value>, core::DenseRC<core::Slots<BM, false, NT>::value>>;
            using LB = std::conditional_t<B_KC, core::DenseKC<core::Slots<BN, true, NT>::value>, core::DenseRC<core::Slots<BN, false, NT>::value>>;
            LA la;
            la.base = A[shard].data() + (size_t)kbeg * (A_KC ? 2 : 2 * (size_t)lda);
            la.ld = lda; la.rows = (int)M; la.K = klen;
            LB lb;
            lb.base = B[shard].data() + (size_t)kbeg * (B_KC ? 2 : 2 * (size_t)ldb);
            lb.ld = ldb; lb.rows = (int)N; lb.K = klen;
            core::tile_product<BM, BN, WM, WN, DEPTH, KMASK, OUT_BF16, VEC>(la, lb, C[vshard].data(), ldc, (int)M, (int)N, klen, tm * BM,
                                                                             tn * BN, relu != 0, lds.data());
        }
    for (size_t s = 0; s < C.size(); ++s)
        for (size_t i = 0; i < C[s].size(); ++i)
            if (C[s][i] != 0) { std::printf("output %zu byte %zu never written\n", s, i); return 1; }
    std::printf("ok engine 1 tile %dx%d count %d %ldx%ldx%ld ksplit %d\n", BM, BN, count, M, N, K, ksplit);
    return 0;
}
