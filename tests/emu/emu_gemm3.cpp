// Host build of the direct-to-LDS tile engine (csrc/gemm_core2.h), the persistent one (csrc/gemm_core3.h) and the
// 256 x 128 one (csrc/gemm_core4.h) for checking their memory accesses without a GPU: for a list of products the launch parameters are derived exactly as the
// launchers derive them (csrc/gemm3_params.h), every workgroup and every thread of the grid is run in turn, and every
// access they make has to stay inside the operands, the outputs and the LDS of the launch; afterwards every element of
// every output must have been written.  Build: see tests/test_kernel_emulation.py (host clang, address sanitizer).
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <type_traits>
#include <vector>

#define TT_HOST_EMULATION 1
#include "gemm3_params.h"

namespace tt {
} // namespace tt

using namespace tt;

struct Case { int engine, count; long M, N, K; bool a_kc, b_kc, out_bf16; int relu, ksplit; };

template <bool A_KC, bool B_KC, bool OUT_BF16, bool STAGED, bool ILV> void run3(const core3::Params3 &p, unsigned grid)
{
    const size_t smem = core3::smem_bytes3<64, 2, STAGED>();
    std::vector<char> lds(smem);
    dev::g_lds = lds.data();
    dev::g_lds_bytes = smem;
    for (unsigned b = 0; b < grid; ++b)
        for (unsigned t = 0; t < (unsigned)core3::kThreads3; ++t) {
            blockIdx = {b, 0, 0};
            threadIdx = {t, 0, 0};
            core3::run_tiles<64, 2, A_KC, B_KC, OUT_BF16, STAGED, ILV>(p, lds.data());
        }
}

template <bool A_KC, bool B_KC, bool OUT_BF16, bool STAGED> void run4(const core3::Params3 &p, unsigned grid)
{
    std::vector<char> lds(core4::kSmem4);
    dev::g_lds = lds.data();
    dev::g_lds_bytes = core4::kSmem4;
    for (unsigned b = 0; b < grid; ++b)
        for (unsigned t = 0; t < (unsigned)core4::kThreads4; ++t) {
            blockIdx = {b, 0, 0};
            threadIdx = {t, 0, 0};
            // the body of gemm_bf16_v4_kernel (csrc/gemm3.hip)
            const int logical = core::logical_block(p.per_xcd, p.total);
            if (logical < 0) continue;
            const int tiles = p.tiles_m * p.tiles_n;
            const int vshard = logical / tiles;
            const int tt_ = logical - vshard * tiles;
            int tm, tn;
            core::grouped_tile(tt_, p.tiles_m, p.tiles_n, &tm, &tn);
            const int shard = vshard / p.ksplit;
            const int kbeg = (vshard - shard * p.ksplit) * p.kchunk;
            const int klen = p.K - kbeg < p.kchunk ? p.K - kbeg : p.kchunk;
            const char *abase = reinterpret_cast<const char *>(p.A[shard]) + (size_t)kbeg * (A_KC ? 2 : 2 * (size_t)p.lda);
            const char *bbase = reinterpret_cast<const char *>(p.B[shard]) + (size_t)kbeg * (B_KC ? 2 : 2 * (size_t)p.ldb);
            core4::tile_product4<A_KC, B_KC, OUT_BF16, STAGED>(abase, p.lda, bbase, p.ldb, p.C[vshard], p.ldc, p.M, p.N, klen,
                                                               tm * core4::BM4, tn * core4::BN4, p.relu != 0, lds.data());
        }
}

template <bool A_KC, bool B_KC, bool OUT_BF16, bool VEC> void run2(const core3::Params3 &p, unsigned grid)
{
    std::vector<char> lds(core2::kSmemBytes);
    dev::g_lds = lds.data();
    dev::g_lds_bytes = core2::kSmemBytes;
    for (unsigned b = 0; b < grid; ++b)
        for (unsigned t = 0; t < (unsigned)core2::kThreads2; ++t) {
            blockIdx = {b, 0, 0};
            threadIdx = {t, 0, 0};
            // the body of gemm_bf16_v2_kernel (csrc/gemm.hip)
            const int logical = core::logical_block(p.per_xcd, p.total);
            if (logical < 0) continue;
            const int tiles = p.tiles_m * p.tiles_n;
            const int vshard = logical / tiles;
            const int tt_ = logical - vshard * tiles;
            int tm, tn;
            core::grouped_tile(tt_, p.tiles_m, p.tiles_n, &tm, &tn);
            const int shard = vshard / p.ksplit;
            const int kbeg = (vshard - shard * p.ksplit) * p.kchunk;
            const int klen = p.K - kbeg < p.kchunk ? p.K - kbeg : p.kchunk;
            using LA = std::conditional_t<A_KC, core2::DenseKC2, core2::DenseRC2>;
            using LB = std::conditional_t<B_KC, core2::DenseKC2, core2::DenseRC2>;
            LA la;
            la.base = reinterpret_cast<const char *>(p.A[shard]) + (size_t)kbeg * (A_KC ? 2 : 2 * (size_t)p.lda);
            la.ld = p.lda; la.rows = p.M; la.K = klen;
            LB lb;
            lb.base = reinterpret_cast<const char *>(p.B[shard]) + (size_t)kbeg * (B_KC ? 2 : 2 * (size_t)p.ldb);
            lb.ld = p.ldb; lb.rows = p.N; lb.K = klen;
            core2::tile_product2<OUT_BF16, VEC>(la, lb, p.C[vshard], p.ldc, p.M, p.N, klen, tm * 256, tn * 256, p.relu != 0, lds.data());
        }
}

template <bool A_KC, bool B_KC> void dispatch(const Case &c, const core3::Params3 &p, bool vec)
{
    if (c.engine == 2) {
        const unsigned grid = (unsigned)p.per_xcd * core::kXcds;
        if (c.out_bf16) { if (vec) run2<A_KC, B_KC, true, true>(p, grid); else run2<A_KC, B_KC, true, false>(p, grid); }
        else { if (vec) run2<A_KC, B_KC, false, true>(p, grid); else run2<A_KC, B_KC, false, false>(p, grid); }
    } else if (c.engine == 3) {
        const unsigned grid = (unsigned)p.wg_per_xcd * core::kXcds;
        // the choice of launch_layout (csrc/gemm3.hip)
        if (c.out_bf16 && vec) { run3<A_KC, B_KC, true, true, true>(p, grid); return; }
        if (A_KC && !B_KC && !c.out_bf16) { run3<A_KC, B_KC, false, false, true>(p, grid); return; }
        if (c.out_bf16) run3<A_KC, B_KC, true, false, false>(p, grid);
        else run3<A_KC, B_KC, false, false, false>(p, grid);
    } else {
        const unsigned grid = (unsigned)p.per_xcd * core::kXcds;
        if (c.out_bf16 && vec) { run4<A_KC, B_KC, true, true>(p, grid); return; }
        if (c.out_bf16) run4<A_KC, B_KC, true, false>(p, grid);
        else run4<A_KC, B_KC, false, false>(p, grid);
    }
}

int run_case(const Case &c)
{
    const size_t out_b = c.out_bf16 ? 2 : 4;
    std::vector<std::vector<char>> A(c.count), B(c.count), C(c.count * c.ksplit);
    std::vector<const void *> Ap, Bp;
    std::vector<void *> Cp;
    dev::g_n_readable = 0;
    for (int s = 0; s < c.count; ++s) {
        // all-zero operands: whatever a lane reads back from an LDS staging area that other lanes (run later here)
        // fill is zero as well, so "every output byte turned 0" holds for any order of the threads
        A[s].assign((size_t)c.M * c.K * 2, 0);
        B[s].assign((size_t)c.K * c.N * 2, 0);
        Ap.push_back(A[s].data());
        Bp.push_back(B[s].data());
        // EMU_SHRINK: self-check of the checker - the last 16 bytes of every operand are declared out of bounds
        const size_t cut = std::getenv("EMU_SHRINK") ? 16 : 0;
        dev::g_readable[dev::g_n_readable++] = {A[s].data(), A[s].data() + A[s].size() - cut};
        dev::g_readable[dev::g_n_readable++] = {B[s].data(), B[s].data() + B[s].size() - cut};
    }
    for (auto &v : C) {
        v.assign((size_t)c.M * c.N * out_b, (char)0x5a);
        Cp.push_back(v.data());
    }
    const long kchunk = c.ksplit == 1 ? c.K : ((c.K + c.ksplit - 1) / c.ksplit + 63) / 64 * 64; // as tt_shard_gemm splits K
    core3::Params3 p;
    const long lda = c.a_kc ? c.K : c.M, ldb = c.b_kc ? c.K : c.N;
    // (the second engine takes any K: its loaders read a zero chunk past the end; same tile grid as the third's, one
    // workgroup per tile)
    dev::g_readable[dev::g_n_readable++] = {reinterpret_cast<const char *>(core2::g_zero_chunk),
                                            reinterpret_cast<const char *>(core2::g_zero_chunk) + 16};
    const tt_status st = c.engine == 2
        ? fill_params3(&p, 256, 256, 1, 0, c.count, Ap.data(), Bp.data(), Cp.data(), c.M, c.N, c.K, lda, ldb, c.N, c.a_kc, c.b_kc,
                       c.relu, c.ksplit, kchunk)
        : c.engine == 3
        ? fill_params3(&p, core3::BM3, core3::BN3, 64, 256, c.count, Ap.data(), Bp.data(), Cp.data(), c.M, c.N, c.K, lda, ldb, c.N,
                       c.a_kc, c.b_kc, c.relu, c.ksplit, kchunk)
        : fill_params3(&p, core4::BM4, core4::BN4, core4::BK4, 0, c.count, Ap.data(), Bp.data(), Cp.data(), c.M, c.N, c.K, lda, ldb,
                       c.N, c.a_kc, c.b_kc, c.relu, c.ksplit, kchunk);
    if (st != TT_OK) { std::printf("case refused by the launcher (status %d)\n", (int)st); return 2; }
    const bool vec = c.N % (c.out_bf16 ? 8 : 4) == 0;
    dev::g_dma_bytes = 0;
    if (c.a_kc && c.b_kc) dispatch<true, true>(c, p, vec);
    else if (c.a_kc) dispatch<true, false>(c, p, vec);
    else if (c.b_kc) dispatch<false, true>(c, p, vec);
    else dispatch<false, false>(c, p, vec);
    // the stand-in MFMA leaves the accumulators at zero: every output byte must have turned from 0x5a to 0
    for (size_t s = 0; s < C.size(); ++s)
        for (size_t i = 0; i < C[s].size(); ++i)
            if (C[s][i] != 0) { std::printf("output %zu byte %zu never written\n", s, i); return 1; }
    std::printf("ok engine %d count %d %ldx%ldx%ld a_kc %d b_kc %d bf16 %d ksplit %d: %llu bytes global -> LDS\n", c.engine,
                c.count, c.M, c.N, c.K, (int)c.a_kc, (int)c.b_kc, (int)c.out_bf16, c.ksplit, dev::g_dma_bytes);
    return 0;
}

int main(int argc, char **argv)
{
    // engine count M N K a_kc b_kc out_bf16 relu ksplit
    if (argc != 11) { std::fprintf(stderr, "usage: emu_gemm3 engine count M N K a_kc b_kc out_bf16 relu ksplit\n"); return 64; }
    Case c;
    c.engine = std::atoi(argv[1]); c.count = std::atoi(argv[2]);
    c.M = std::atol(argv[3]); c.N = std::atol(argv[4]); c.K = std::atol(argv[5]);
    c.a_kc = std::atoi(argv[6]) != 0; c.b_kc = std::atoi(argv[7]) != 0; c.out_bf16 = std::atoi(argv[8]) != 0;
    c.relu = std::atoi(argv[9]); c.ksplit = std::atoi(argv[10]);
    return run_case(c);
}
