// Host build of the conversion kernels WITH their launch code (csrc/convert.hip compiled as it is: tt_retile,
// tt_retile_gate and tt_reduce run on host buffers, a launch = every thread of every workgroup in turn).  The test
// (tests/test_kernel_emulation.py) writes the shards and what the oracle expects into a directory; this program runs
// the call and compares bit for bit (fp32 sums: the same additions in the same order as on the GPU).  Buffers have
// exactly the shard sizes, so the address sanitizer sees any access past an end.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <string>
#include <vector>

#define TT_HOST_EMULATION 1
#include "convert.hip"

namespace tt {
// measurement hooks: nothing to record here
ProfileScope::ProfileScope(void *, int, int, int64_t, int64_t, int64_t, uint64_t, uint64_t) : slot(-1), stream(nullptr) {}
ProfileScope::~ProfileScope() {}
} // namespace tt

static std::vector<char> slurp(const std::string &path)
{
    std::ifstream f(path, std::ios::binary);
    if (!f) { std::fprintf(stderr, "cannot read %s\n", path.c_str()); std::exit(64); }
    return std::vector<char>((std::istreambuf_iterator<char>(f)), std::istreambuf_iterator<char>());
}

static tt_tiling tiling_of(const char *letters)
{
    tt_tiling t{};
    for (int j = 0; letters[j] && j < TT_MAX_K; ++j) t.cut[j] = letters[j] == 'R' ? TT_R : (letters[j] == 'C' ? TT_C : TT_REP);
    return t;
}

int main(int argc, char **argv)
{
    // emu_convert DIR retile k rows cols elem_bytes A B
    // emu_convert DIR gate   k rows cols dtype A Am B
    // emu_convert DIR reduce k rows cols out_dtype act forms B          (forms: digits 1..3; "-" for k = 0)
    if (argc < 8) { std::fprintf(stderr, "bad arguments\n"); return 64; }
    const std::string dir = argv[1], what = argv[2];
    const int k = std::atoi(argv[3]);
    const long rows = std::atol(argv[4]), cols = std::atol(argv[5]);
    const int n = 1 << k;
    auto load_all = [&](const char *stem, int count) {
        std::vector<std::vector<char>> v;
        for (int s = 0; s < count; ++s) v.push_back(slurp(dir + "/" + stem + std::to_string(s) + ".bin"));
        return v;
    };
    auto strip = [](const char *t) { return std::string(t) == "-" ? std::string() : std::string(t); };
    std::vector<std::vector<char>> expect = load_all("exp", n), out;
    for (auto &e : expect) out.emplace_back(e.size(), (char)0x5a);
    std::vector<void *> dst;
    for (auto &o : out) dst.push_back(o.data());
    tt_status st;
    if (what == "retile") {
        auto src = load_all("src", n);
        std::vector<const void *> sp;
        for (auto &s : src) sp.push_back(s.data());
        st = tt_retile(dst.data(), tiling_of(strip(argv[8]).c_str()), sp.data(), tiling_of(strip(argv[7]).c_str()), k, rows, cols,
                       std::atoi(argv[6]), nullptr);
    } else if (what == "gate") {
        auto src = load_all("src", n), msk = load_all("msk", n);
        std::vector<const void *> sp, mp;
        for (auto &s : src) sp.push_back(s.data());
        for (auto &m : msk) mp.push_back(m.data());
        st = tt_retile_gate(dst.data(), tiling_of(strip(argv[9]).c_str()), sp.data(), tiling_of(strip(argv[7]).c_str()), mp.data(),
                            tiling_of(strip(argv[8]).c_str()), k, rows, cols, std::atoi(argv[6]), nullptr);
    } else if (what == "reduce") {
        auto part = load_all("src", n);
        std::vector<const float *> pp;
        for (auto &s : part) pp.push_back(reinterpret_cast<const float *>(s.data()));
        const std::string f = strip(argv[8]);
        uint8_t forms[TT_MAX_K] = {};
        for (int j = 0; j < k; ++j) forms[j] = (uint8_t)(f[j] - '1');
        st = tt_reduce(dst.data(), tiling_of(strip(argv[9]).c_str()), std::atoi(argv[6]), pp.data(), forms, k, rows, cols,
                       std::atoi(argv[7]), nullptr);
    } else {
        return 64;
    }
    if (st != TT_OK) { std::printf("status %d\n", (int)st); return 2; }
    for (int s = 0; s < n; ++s)
        if (out[s] != expect[s]) {
            size_t i = 0;
            while (out[s][i] == expect[s][i]) ++i;
            std::printf("shard %d differs at byte %zu\n", s, i);
            return 1;
        }
    std::printf("ok %s: %llu threads run\n", what.c_str(), g_emu_threads_run);
    return 0;
}
