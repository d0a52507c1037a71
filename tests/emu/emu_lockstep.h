// Lock-step mode of the host stand-ins (-DTT_EMU_LOCKSTEP): the threads of a workgroup run as cooperative fibers, so
// that what one thread writes to LDS is there when another reads it after a barrier, and the wave-wide instructions
// compute what the hardware computes:
//   - __syncthreads(): nobody passes before every thread of the workgroup that has not ended arrived;
//   - wave barriers and wait counts: the same among the 64 lanes of a wave (on the device a wave's lanes execute an
//     instruction together, so code may read what another lane of the same wave wrote before such a point);
//   - v_mfma_f32_32x32x16_bf16: D = C + A B over the wave's registers in the instruction's lane layout
//     (A: row lane % 32, k = 8 (lane / 32) + 0..7; B: column lane % 32, the same k; C, D: column lane % 32, row
//     8 (r / 4) + 4 (lane / 32) + r % 4 for register r), products and sums in double, rounded once to fp32;
//   - ds_read_b64_tr_b16: in every group of 16 lanes, element e of lane i comes from lane 4 e + i / 4, element i % 4
//     (the 4 x 16 block of 16-bit values the group addressed, transposed).
// Global -> LDS loads land late: a lane's loads stay pending, in order, until a wait count of that lane lets them
// through (s_waitcnt vmcnt(n) lands all but the newest n), which is the latest the hardware may deliver them; its
// register loads, which the hardware counts as well, are not seen here, so the model never lands more than the hardware
// has; stores are counted where a kernel issues them through dev::store16 (kernels that keep stores in flight over a
// wait and subtract them in its count), and not seen otherwise.  A kernel that reads a stage before waiting for it therefore reads stale data here, and one that
// ends with loads still in flight towards LDS is reported.  With this the kernels produce values, which the tests
// compare with the oracle's.
#pragma once
#include <ucontext.h>
#include <deque>
#include <functional>
#include <vector>

namespace emu {

constexpr int kWave = 64;
constexpr size_t kStackBytes = 256 * 1024;

struct WaveState {
    int live = 0, arrived = 0, kind = 0;
    unsigned gen = 0;
    uint16_t a[kWave][8], b[kWave][8];
    float c[kWave][16];
    uint16_t tr[kWave][4];
};

struct PendingLoad { char *dst; const char *src; };

struct Block {
    std::vector<std::deque<PendingLoad>> pending; // per thread: global -> LDS loads issued and not yet landed
    ucontext_t sched;
    std::vector<ucontext_t> ctx;
    std::vector<char> done;
    std::vector<char *> stacks;
    std::vector<WaveState> waves;
    int n = 0, cur = 0, live = 0, bar_arrived = 0;
    unsigned bar_gen = 0;
    unsigned long long progress = 0;
    std::function<void()> body;
};
inline Block g_block;

[[noreturn]] inline void die(const char *what)
{
    std::fprintf(stderr, "EMU FAULT: %s (block %u thread %u)\n", what, blockIdx.x, threadIdx.x);
    std::abort();
}

inline void yield() { swapcontext(&g_block.ctx[g_block.cur], &g_block.sched); }
inline int lane() { return g_block.cur % kWave; }
inline WaveState &my_wave() { return g_block.waves[g_block.cur / kWave]; }

// every lane of the wave that has not ended calls this with the same kind; the last to arrive runs complete()
template <class F> inline void wave_collective(int kind, F &&complete)
{
    WaveState &w = my_wave();
    const unsigned my = w.gen;
    if (w.arrived == 0) w.kind = kind;
    else if (w.kind != kind) die("the lanes of a wave reached different wave-wide operations");
    if (++w.arrived == w.live) {
        complete(w);
        w.arrived = 0;
        ++w.gen;
    } else {
        while (w.gen == my) yield();
    }
    ++g_block.progress;
}
inline void wave_sync() { wave_collective(1, [](WaveState &) {}); }

inline void issue_lds_load(char *dst, const char *src) { g_block.pending[g_block.cur].push_back({dst, src}); }
// a global store that the kernel leaves in flight over a wait: it takes a place in the lane's queue of vector-memory
// operations (its data is written at once: nothing here reads it back)
inline void issue_counted_store() { g_block.pending[g_block.cur].push_back({nullptr, nullptr}); }

// s_waitcnt with the gfx9 encoding of its operand: vmcnt in bits 3:0 and 15:14
inline void wait_counts(unsigned imm)
{
    // EMU_VMCNT_SLACK=n: every wait lets n more loads stay in flight than the kernel asked for (self-check of this model:
    // the kernels' results must then be wrong)
    static const unsigned slack = [] { const char *e = std::getenv("EMU_VMCNT_SLACK"); return e ? (unsigned)std::atoi(e) : 0u; }();
    const unsigned vmcnt = ((imm & 15u) | (((imm >> 14) & 3u) << 4)) + slack;
    std::deque<PendingLoad> &q = g_block.pending[g_block.cur];
    while (q.size() > vmcnt) {
        if (q.front().dst) std::memcpy(q.front().dst, q.front().src, 16);
        q.pop_front();
    }
    wave_sync();
}

inline void block_barrier()
{
    Block &b = g_block;
    const unsigned my = b.bar_gen;
    if (++b.bar_arrived == b.live) {
        b.bar_arrived = 0;
        ++b.bar_gen;
    } else {
        while (b.bar_gen == my) yield();
    }
    ++b.progress;
}

inline float bf16_bits_to_float(uint16_t h)
{
    const uint32_t u = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

template <class AB, class C> inline C mfma_32x32x16_bf16(AB a, AB b, C c)
{
    static_assert(sizeof(AB) == 16 && sizeof(C) == 64, "operand registers of v_mfma_f32_32x32x16_bf16");
    WaveState &w = my_wave();
    const int l = lane();
    std::memcpy(w.a[l], &a, 16);
    std::memcpy(w.b[l], &b, 16);
    std::memcpy(w.c[l], &c, 64);
    wave_collective(2, [](WaveState &v) {
        if (v.live != kWave) die("MFMA in a wave with ended lanes");
        static float d[kWave][16];
        for (int ln = 0; ln < kWave; ++ln)
            for (int r = 0; r < 16; ++r) {
                const int i = 8 * (r / 4) + 4 * (ln / 32) + r % 4, j = ln % 32;
                double s = v.c[ln][r];
                for (int k = 0; k < 16; ++k)
                    s += (double)bf16_bits_to_float(v.a[i + 32 * (k / 8)][k % 8]) * (double)bf16_bits_to_float(v.b[j + 32 * (k / 8)][k % 8]);
                d[ln][r] = (float)s;
            }
        std::memcpy(v.c, d, sizeof(d));
    });
    std::memcpy(&c, w.c[l], 64);
    return c;
}

// the caller has put its own 8 bytes into tr[lane]
inline void transpose_groups_of_16()
{
    wave_collective(3, [](WaveState &v) {
        if (v.live != kWave) die("transpose read in a wave with ended lanes");
        uint16_t r[kWave][4];
        for (int g = 0; g < kWave; g += 16)
            for (int i = 0; i < 16; ++i)
                for (int e = 0; e < 4; ++e) r[g + i][e] = v.tr[g + 4 * e + i / 4][i % 4];
        std::memcpy(v.tr, r, sizeof(r));
    });
}

inline void trampoline()
{
    Block &b = g_block;
    b.body();
    const int t = b.cur;
    for (const PendingLoad &l : b.pending[t])
        if (l.dst) die("the kernel ended with global -> LDS loads still in flight");
    b.done[t] = 1;
    --b.live;
    WaveState &w = b.waves[t / kWave];
    --w.live;
    if (w.arrived > 0 && w.arrived == w.live) die("a lane ended while the rest of its wave waits in a wave-wide operation");
    if (b.bar_arrived > 0 && b.bar_arrived == b.live) { // ended threads do not take part in barriers
        b.bar_arrived = 0;
        ++b.bar_gen;
    }
    ++b.progress;
    swapcontext(&b.ctx[t], &b.sched);
    die("an ended fiber was resumed");
}

template <class F> inline void run_block(F &&body, unsigned threads)
{
    Block &b = g_block;
    b.body = body;
    b.n = (int)threads;
    b.live = b.n;
    b.bar_arrived = 0;
    b.ctx.resize(threads);
    b.done.assign(threads, 0);
    b.pending.assign(threads, std::deque<PendingLoad>());
    b.waves.assign((threads + kWave - 1) / kWave, WaveState());
    while (b.stacks.size() < threads) b.stacks.push_back(static_cast<char *>(std::malloc(kStackBytes)));
    for (unsigned t = 0; t < threads; ++t) {
        getcontext(&b.ctx[t]);
        b.ctx[t].uc_stack.ss_sp = b.stacks[t];
        b.ctx[t].uc_stack.ss_size = kStackBytes;
        b.ctx[t].uc_link = nullptr;
        makecontext(&b.ctx[t], trampoline, 0);
        ++b.waves[t / kWave].live;
    }
    // EMU_ORDER=reverse: the last wave runs ahead of the first instead of behind it (results must not depend on which
    // wave reaches a barrier first)
    static const bool reversed = [] { const char *e = std::getenv("EMU_ORDER"); return e && std::strcmp(e, "reverse") == 0; }();
    while (b.live > 0) {
        const unsigned long long before = b.progress;
        for (unsigned i = 0; i < threads; ++i) {
            const unsigned t = reversed ? threads - 1 - i : i;
            if (!b.done[t]) {
                b.cur = (int)t;
                threadIdx = {t, 0, 0};
                swapcontext(&b.sched, &b.ctx[t]);
            }
        }
        if (b.progress == before) die("deadlock: every thread waits (a barrier or wave-wide operation not reached by all)");
    }
}

} // namespace emu

inline void __syncthreads() { emu::block_barrier(); }
#define __builtin_amdgcn_s_waitcnt(x) emu::wait_counts(x)
#define __builtin_amdgcn_wave_barrier() emu::wave_sync()
#define __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, x, y, z) emu::mfma_32x32x16_bf16(a, b, c)
