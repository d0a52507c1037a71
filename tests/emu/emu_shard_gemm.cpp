// Host build of the shard-product entry point WITH its launch code (csrc/gemm.hip and csrc/gemm3.hip compiled as they
// are: tt_shard_gemm picks the engine, the tile and the in-launch K split exactly as in the library, on a device with
// 256 compute units) for checking memory accesses without a GPU.  Operands are zero, outputs start as 0x5a bytes and
// have exactly the product's size; the stand-in MFMA multiplies nothing.  Checked: no access outside a buffer or
// outside the launch's LDS (address sanitizer and explicit ranges), every output byte written.
#include <cstdio>
#include <cstdlib>
#include <vector>

#define TT_HOST_EMULATION 1
#include <cstdint>
namespace tt {
namespace {
// what the kernels' `extern __shared__` arrays refer to here (one name per kernel family)
alignas(16) thread_local uint16_t smem[80 * 1024];
alignas(16) thread_local char smem2[160 * 1024], smem3[160 * 1024], smem4[160 * 1024];
}
} // namespace tt
#include "gemm.hip"
#include "gemm3.hip"

namespace tt {
ProfileScope::ProfileScope(void *, int, int, int64_t, int64_t, int64_t, uint64_t, uint64_t) : slot(-1), stream(nullptr) {}
ProfileScope::~ProfileScope() {}
} // namespace tt

static bool read_file(const char *dir, const char *name, int s, std::vector<char> &into)
{
    char path[512];
    std::snprintf(path, sizeof(path), "%s/%s%d.bin", dir, name, s);
    FILE *f = std::fopen(path, "rb");
    if (!f) return false;
    const size_t got = std::fread(into.data(), 1, into.size(), f);
    const bool at_end = std::fgetc(f) == EOF;
    std::fclose(f);
    return got == into.size() && at_end;
}

int main(int argc, char **argv)
{
    // emu_shard_gemm count M N K trans_a trans_b in_bf16 out_bf16 relu ksplit
    // (ksplit 1: the exported entry point; above 1: the in-launch K split the layer-chain code asks launch_gemm for,
    // which writes count * ksplit partial products)
    // With a directory as one more argument (lock-step build): operands are read from a<s>.bin / b<s>.bin there and the
    // results written to c<s>.bin, for the caller to compare with the oracle's.
    if (argc != 11 && argc != 12) { std::fprintf(stderr, "usage: emu_shard_gemm count M N K trans_a trans_b in_bf16 out_bf16 relu ksplit [dir]\n"); return 64; }
    const char *dir = argc == 12 ? argv[11] : nullptr;
    emu_register_lds(tt::smem, sizeof(tt::smem));
    emu_register_lds(tt::smem2, sizeof(tt::smem2));
    emu_register_lds(tt::smem3, sizeof(tt::smem3));
    emu_register_lds(tt::smem4, sizeof(tt::smem4));
    const int count = std::atoi(argv[1]);
    const long M = std::atol(argv[2]), N = std::atol(argv[3]), K = std::atol(argv[4]);
    const int ta = std::atoi(argv[5]), tb = std::atoi(argv[6]), in_bf = std::atoi(argv[7]), out_bf = std::atoi(argv[8]), relu = std::atoi(argv[9]);
    const int ksplit = std::atoi(argv[10]);
    const size_t ib = in_bf ? 2 : 4, ob = out_bf ? 2 : 4;
    std::vector<std::vector<char>> A(count), B(count), C((size_t)count * ksplit);
    std::vector<const void *> Ap, Bp;
    std::vector<void *> Cp;
    tt::dev::g_n_readable = 0;
    tt::dev::g_readable[tt::dev::g_n_readable++] = {reinterpret_cast<const char *>(tt::core2::g_zero_chunk),
                                                    reinterpret_cast<const char *>(tt::core2::g_zero_chunk) + 16};
    for (int s = 0; s < count; ++s) {
        A[s].assign((size_t)M * K * ib, 0);
        B[s].assign((size_t)K * N * ib, 0);
        if (dir && (!read_file(dir, "a", s, A[s]) || !read_file(dir, "b", s, B[s]))) { std::fprintf(stderr, "cannot read operand %d\n", s); return 65; }
        Ap.push_back(A[s].data()); Bp.push_back(B[s].data());
        tt::dev::g_readable[tt::dev::g_n_readable++] = {A[s].data(), A[s].data() + A[s].size()};
        tt::dev::g_readable[tt::dev::g_n_readable++] = {B[s].data(), B[s].data() + B[s].size()};
    }
    for (auto &c : C) { c.assign((size_t)M * N * ob, (char)0x5a); Cp.push_back(c.data()); }
    const int in_dt = in_bf ? TT_BF16 : TT_F32, out_dt = out_bf ? TT_BF16 : TT_F32, act = relu ? TT_ACT_RELU : TT_ACT_NONE;
    const tt_status st = ksplit == 1 ? tt_shard_gemm(count, Ap.data(), Bp.data(), Cp.data(), M, N, K, ta, tb, in_dt, out_dt, act, nullptr)
                                     : tt::launch_gemm(count, Ap.data(), Bp.data(), Cp.data(), M, N, K, ta, tb, in_dt, out_dt, act, ksplit, nullptr);
    if (st != TT_OK) { std::printf("status %d\n", (int)st); return 2; }
    if (dir) {
        for (size_t s = 0; s < C.size(); ++s) {
            char path[512];
            std::snprintf(path, sizeof(path), "%s/c%zu.bin", dir, s);
            FILE *f = std::fopen(path, "wb");
            if (!f || std::fwrite(C[s].data(), 1, C[s].size(), f) != C[s].size()) { std::fprintf(stderr, "cannot write %s\n", path); return 66; }
            std::fclose(f);
        }
        std::printf("ok shard_gemm values: %llu threads run\n", g_emu_threads_run);
        return 0;
    }
    for (size_t s = 0; s < C.size(); ++s)
        for (size_t i = 0; i < C[s].size(); ++i)
            if (C[s][i] != 0) { std::printf("output %zu byte %zu never written\n", s, i); return 1; }
    std::printf("ok shard_gemm: %llu threads run, %llu bytes global -> LDS\n", g_emu_threads_run, tt::dev::g_dma_bytes);
    return 0;
}
