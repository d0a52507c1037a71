// bf16 MFMA tile engine shared by the FC shard products and the implicit-GEMM convolutions.
//
// One workgroup (256 threads = four 64-lane waves) computes a BM x BN tile of C = A B with
// v_mfma_f32_32x32x16_bf16 and fp32 accumulators in registers.  Operand tiles (BM x 64 and BN x 64 bf16) are staged
// global -> registers -> LDS, always as K-contiguous LDS rows of 64 + 8 elements (144-byte rows keep the 16-byte
// fragment reads conflict free).  Two tiles are in flight in registers while a third is being multiplied, LDS is double
// buffered.  Where an operand's contiguous dimension is not K it is transposed in registers (4 x 8 blocks) on its way
// to LDS.  How operand elements are addressed is a policy ("loader"): dense matrices for FC, gathered image windows for
// convolution.  The accumulators leave through a wave-private LDS staging area so that global stores are 16-byte
// vectors along C's rows.
#pragma once
#include <cstdint>
#include "tt_device.h"
#include "tt_bf16.h"

namespace tt {
namespace core {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int BK = 64;
constexpr int LDK = BK + 8;
constexpr int kXcds = 8;

using tt::f32_to_bf16_bits;
using tt::pack_bf16x2;

__device__ __forceinline__ u32x4 zero4()
{
    u32x4 z = {0, 0, 0, 0};
    return z;
}

// ---- loaders for dense row-major operands -------------------------------------------------------------------------
// Loader concept:
//   static constexpr bool KC  : true  = the operand's LDS row index ("row": m for A, n for B) has K contiguous in memory
//                               false = rows are contiguous in memory, K strides
//   init(slot, row)           : KC: bind the slot to one row;  !KC: bind the slot to 8 consecutive rows starting at row
//   load(slot, k)             : KC: 8 consecutive k starting at k (multiple of 8);  !KC: the slot's 8 rows at this k
//   begin_tile(k0)            : called once per K tile before its loads (wave-uniform k0)
//   load4<KMASK>(slot, k, out): !KC only: the slot's 8 rows at k, k+1, k+2, k+3
// Out-of-range rows / k return zeros.
// Rows are remembered as 32-bit byte offsets from a wave-uniform base (scalar base + vector offset addressing).
// Loads are UNCONDITIONAL and never sit under a branch or feed a select: a load whose only use is one arm of a select is
// turned back into a branch by the compiler, and a wait for all outstanding loads follows at the join, which serialises
// the prefetch.  Instead addresses are clamped into the operand and, where needed, data is zeroed by AND with a mask.
//   load(slot, k)        : k and the slot's rows are known to be in range (whole tiles)
//   load_masked(slot, k) : k may lie beyond K: address clamped, data zeroed
// Rows beyond the operand are clamped at init() and need no zeroing: they only feed C rows / columns that are never
// stored.  Requires rows >= 1 (>= 8 for DenseRC) and K >= 8, which the 16-byte alignment rules guarantee.
__device__ __forceinline__ u32x4 and_mask(u32x4 v, bool keep)
{
    const uint32_t m = keep ? 0xffffffffu : 0u;
    u32x4 o = {v[0] & m, v[1] & m, v[2] & m, v[3] & m};
    return o;
}
template <int SLOTS> struct DenseKC {
    static constexpr bool KC = true;
    static constexpr bool kFence = true;
    const char *base;
    int ld, rows, K;
    uint32_t off[SLOTS];
    __device__ __forceinline__ void init(int slot, int row)
    {
        off[slot] = (uint32_t)(row < rows ? row : rows - 1) * (uint32_t)ld * 2u;
    }
    __device__ __forceinline__ u32x4 load(int slot, int k) const
    {
        return *reinterpret_cast<const u32x4 *>(base + (size_t)(off[slot] + (uint32_t)k * 2u));
    }
    __device__ __forceinline__ u32x4 load_masked(int slot, int k) const
    {
        return and_mask(load(slot, k < K ? k : K - 8), k < K);
    }
    __device__ __forceinline__ void begin_tile(int) {}
};
template <int SLOTS> struct DenseRC {
    static constexpr bool KC = false;
    static constexpr bool kFence = true;
    const char *base;
    int ld, rows, K;
    uint32_t off[SLOTS];
    __device__ __forceinline__ void init(int slot, int row) { off[slot] = (uint32_t)(row < rows ? row : rows - 8) * 2u; }
    __device__ __forceinline__ u32x4 load(int slot, int k) const
    {
        return *reinterpret_cast<const u32x4 *>(base + (size_t)(off[slot] + (uint32_t)k * (uint32_t)ld * 2u));
    }
    __device__ __forceinline__ u32x4 load_masked(int slot, int k) const
    {
        return and_mask(load(slot, k < K ? k : K - 1), k < K);
    }
    __device__ __forceinline__ void begin_tile(int) {}
    // four consecutive k for one slot
    template <bool KMASK> __device__ __forceinline__ void load4(int slot, int k, u32x4 *out) const
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) out[q] = KMASK ? load_masked(slot, k + q) : load(slot, k + q);
    }
};

// number of loader slots a tile side of ROWS rows needs
template <int ROWS, bool KC, int NT = kThreads> struct Slots {
    static constexpr int value = KC ? ROWS * (BK / 8) / NT : (BK / 4) * (ROWS / 8) / NT;
    static_assert(value >= 1, "tile side too small for the workgroup");
};

// ---- register staging of one operand tile -------------------------------------------------------------------------
// Transposing side (!KC): the tile is cut into blocks of 4 k x 8 rows; block b = (rv, kg) covers rows 8 rv .. 8 rv + 7
// and k = 4 kg .. 4 kg + 3.  Lanes run over kg first (16 k-groups), then rv: the 8-byte LDS stores of a wave then fall
// on 32 distinct 8-byte bank groups (two lanes each, the minimum), where running over rv first would pile eight lanes on
// each group.  Global loads still cover 64 contiguous bytes per k-row per wave (4 lanes x 16 bytes).
template <int ROWS, bool KC, int NT = kThreads> struct Stage {
    static constexpr int NS = Slots<ROWS, KC, NT>::value;
    static constexpr int NV = KC ? NS : NS * 4;
    u32x4 r[NV];

    template <class L> static __device__ __forceinline__ void bind(L &ld, int row0)
    {
        const int tid = threadIdx.x;
        if constexpr (KC) {
#pragma unroll
            for (int i = 0; i < NS; ++i) ld.init(i, row0 + ((tid + i * NT) >> 3));
        } else {
#pragma unroll
            for (int i = 0; i < NS; ++i) ld.init(i, row0 + ((tid + i * NT) >> 4) * 8);
        }
    }

    // KMASK = false: K is a multiple of BK; a tile start beyond K (prefetch past the end) is pulled back to the last
    // tile (its data is never used).  KMASK = true: per-vector clamping and zeroing.
    template <bool KMASK, class L> __device__ __forceinline__ void load(L &ld, int k0)
    {
        const int tid = threadIdx.x;
        if constexpr (!KMASK) k0 = k0 < ld.K ? k0 : ld.K - BK;
        ld.begin_tile(k0);
        if constexpr (KC) {
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const int k = k0 + (((tid + i * NT) & 7) << 3);
                r[i] = KMASK ? ld.load_masked(i, k) : ld.load(i, k);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const int kg = (tid + i * NT) & 15;
                ld.template load4<KMASK>(i, k0 + kg * 4, &r[i * 4]);
            }
        }
    }

    __device__ __forceinline__ void store(uint16_t *lds) const
    {
        const int tid = threadIdx.x;
        if constexpr (KC) {
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const int v = tid + i * NT;
                *reinterpret_cast<u32x4 *>(lds + (v >> 3) * LDK + ((v & 7) << 3)) = r[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const int b = tid + i * NT;
                const int rv = b >> 4, kg = b & 15;
                uint16_t *dst = lds + (rv * 8) * LDK + kg * 4;
                const u32x4 &a = r[i * 4 + 0], &bq = r[i * 4 + 1], &c = r[i * 4 + 2], &d = r[i * 4 + 3];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // word j of each k-row holds rows (2j, 2j+1); collect the four k values of each row
                    u32x2 lo = {(a[j] & 0xffffu) | (bq[j] << 16), (c[j] & 0xffffu) | (d[j] << 16)};
                    u32x2 hi = {(a[j] >> 16) | (bq[j] & 0xffff0000u), (c[j] >> 16) | (d[j] & 0xffff0000u)};
                    *reinterpret_cast<u32x2 *>(dst + (2 * j) * LDK) = lo;
                    *reinterpret_cast<u32x2 *>(dst + (2 * j + 1) * LDK) = hi;
                }
            }
        }
    }
};

// DEPTH 1, 2: double-buffered LDS; DEPTH 0: one LDS buffer (two barriers per K tile), for two workgroups per CU
template <int BM, int BN, int DEPTH = 1> constexpr size_t smem_bytes()
{
    return (DEPTH == 0 ? 1 : 2) * (size_t)(BM + BN) * LDK * sizeof(uint16_t);
}

// ---- the tile product ---------------------------------------------------------------------------------------------
// C tile origin (m0, n0); C is row-major with leading dimension ldc, M x N valid.  KMASK: K is not a multiple of 64
// (else it must be).  relu: max(x, 0) before the store.  VEC_STORE: 16-byte stores are legal
// (ldc and the base address are multiples of 16 bytes); otherwise elements are stored one by one.
template <int BM, int BN, int WM, int WN, int DEPTH, bool KMASK, bool OUT_BF16, bool VEC_STORE, class LA, class LB>
__device__ __forceinline__ void tile_product(LA &la, LB &lb, void *Cv, int ldc, int M, int N, int K, int m0, int n0,
                                             bool relu, uint16_t *smem)
{
    static_assert(WM * WN == 4 || WM * WN == 8, "four or eight waves");
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_ELEMS = BM * LDK, B_ELEMS = BN * LDK, BUF = A_ELEMS + B_ELEMS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave / WN) * (TM * 32), wn0 = (wave % WN) * (TN * 32);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    using SA = Stage<BM, LA::KC, NT>;
    using SB = Stage<BN, LB::KC, NT>;
    SA sa0, sa1;
    SB sb0, sb1;
    SA::bind(la, m0);
    SB::bind(lb, n0);
    const int nk = (K + BK - 1) / BK;

    // Fragment reads run one k-step ahead of the MFMAs that consume them (two register sets), so the matrix pipe does
    // not idle behind LDS latency when a SIMD holds a single wave.
    auto compute = [&](const uint16_t *As, const uint16_t *Bs) {
        bf16x8 af[2][TM], bf[2][TN];
        const uint16_t *ap = As + (wm0 + (lane & 31)) * LDK + (lane >> 5) * 8;
        const uint16_t *bp = Bs + (wn0 + (lane & 31)) * LDK + (lane >> 5) * 8;
        auto fetch = [&](int ks, int set) {
#pragma unroll
            for (int i = 0; i < TM; ++i) af[set][i] = *reinterpret_cast<const bf16x8 *>(ap + i * 32 * LDK + ks * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[set][j] = *reinterpret_cast<const bf16x8 *>(bp + j * 32 * LDK + ks * 16);
        };
        fetch(0, 0);
        __builtin_amdgcn_iglp_opt(1); // scheduler hint: interleave the LDS fragment reads with the MFMAs
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) fetch(ks + 1, (ks + 1) & 1);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bf[ks & 1][j], acc[i][j], 0, 0, 0);
        }
    };

    if constexpr (DEPTH == 2) {
        // prologue: tiles 0 and 1 in flight, tile 0 into LDS buffer 0
        sa0.template load<KMASK>(la, 0);
        sb0.template load<KMASK>(lb, 0);
        sa1.template load<KMASK>(la, BK); // past the end the loaders clamp addresses and return zeros
        sb1.template load<KMASK>(lb, BK);
        sa0.store(smem);
        sb0.store(smem + A_ELEMS);
        __syncthreads();
        // iteration kt: registers of parity (kt+1)&1 hold tile kt+1; registers of parity kt&1 are free for tile kt+2
        for (int kt = 0; kt < nk; kt += 2) {
            {
                sa0.template load<KMASK>(la, (kt + 2) * BK);
                sb0.template load<KMASK>(lb, (kt + 2) * BK);
                if constexpr (LA::kFence && LB::kFence) __builtin_amdgcn_sched_barrier(0); // keep the prefetch ahead of the MFMAs (see below)
                compute(smem, smem + A_ELEMS);
                if constexpr (LA::kFence && LB::kFence) __builtin_amdgcn_sched_barrier(0);
                if (kt + 1 < nk) { sa1.store(smem + BUF); sb1.store(smem + BUF + A_ELEMS); }
                __syncthreads();
            }
            if (kt + 1 < nk) {
                sa1.template load<KMASK>(la, (kt + 3) * BK);
                sb1.template load<KMASK>(lb, (kt + 3) * BK);
                if constexpr (LA::kFence && LB::kFence) __builtin_amdgcn_sched_barrier(0);
                compute(smem + BUF, smem + BUF + A_ELEMS);
                if constexpr (LA::kFence && LB::kFence) __builtin_amdgcn_sched_barrier(0);
                if (kt + 2 < nk) { sa0.store(smem); sb0.store(smem + A_ELEMS); }
                __syncthreads();
            }
        }
    } else if constexpr (DEPTH == 0) {
        // One LDS buffer and one tile in registers: small enough (LDS and registers) for two workgroups per CU, whose
        // waves fill each other's barrier and memory waits.
        sa0.template load<KMASK>(la, 0);
        sb0.template load<KMASK>(lb, 0);
        for (int kt = 0; kt < nk; ++kt) {
            sa0.store(smem);
            sb0.store(smem + A_ELEMS);
            __syncthreads();
            sa0.template load<KMASK>(la, (kt + 1) * BK);
            sb0.template load<KMASK>(lb, (kt + 1) * BK);
            if constexpr (LA::kFence && LB::kFence) __builtin_amdgcn_sched_barrier(0);
            compute(smem, smem + A_ELEMS);
            if constexpr (LA::kFence && LB::kFence) __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
        }
    } else {
        // one tile in flight in registers (fewer registers: more workgroups per CU)
        sa0.template load<KMASK>(la, 0);
        sb0.template load<KMASK>(lb, 0);
        sa0.store(smem);
        sb0.store(smem + A_ELEMS);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            uint16_t *cur = smem + (kt & 1) * BUF, *nxt = smem + ((kt & 1) ^ 1) * BUF;
            const bool more = kt + 1 < nk;
            sa0.template load<KMASK>(la, (kt + 1) * BK);
            sb0.template load<KMASK>(lb, (kt + 1) * BK);
            // Scheduling fences (dense loaders): without them the compiler, short of registers, sinks the global
            // loads below the MFMA block and waits for them at once, so no memory latency is hidden.  Gather loaders
            // do better unfenced: their address arithmetic then interleaves with the MFMAs.
            if constexpr (LA::kFence && LB::kFence) __builtin_amdgcn_sched_barrier(0);
            compute(cur, cur + A_ELEMS);
            if constexpr (LA::kFence && LB::kFence) __builtin_amdgcn_sched_barrier(0);
            if (more) { sa0.store(nxt); sb0.store(nxt + A_ELEMS); }
            __syncthreads();
        }
    }

    // ---- epilogue.  A lane holds column (lane & 31) and rows 8*(e/4) + 4*(lane/32) + e%4 of each 32 x 32 block.
    if constexpr (!VEC_STORE) {
        const int col_l = lane & 31, row_l = (lane >> 5) * 4;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn0 + j * 32 + col_l;
                if (col >= N) continue;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wm0 + i * 32 + 8 * (e >> 2) + row_l + (e & 3);
                    if (row >= M) continue;
                    float v = acc[i][j][e];
                    if (relu) v = v > 0.0f ? v : 0.0f;
                    if (OUT_BF16) reinterpret_cast<uint16_t *>(Cv)[(size_t)row * ldc + col] = (uint16_t)f32_to_bf16_bits(v);
                    else reinterpret_cast<float *>(Cv)[(size_t)row * ldc + col] = v;
                }
            }
    } else {
        // Each wave turns its 32 x (TN*32) strip around in a private LDS area (fp32, padded rows), then writes whole
        // 16-byte vectors along C's rows.  The operand buffers are free: the last loop iteration ended with a barrier.
        constexpr int SW = TN * 32;        // strip width (elements)
        constexpr int SLD = SW + 4;        // padded fp32 row
        float *strip = reinterpret_cast<float *>(smem) + wave * (32 * SLD);
        static_assert(WM * WN * 32 * SLD * sizeof(float) <= smem_bytes<BM, BN, DEPTH>(), "strip staging fits in the operand buffers");
        constexpr int EPV = OUT_BF16 ? 8 : 4;            // elements per 16-byte output vector
        constexpr int VPR = SW / EPV;                    // vectors per strip row
        constexpr int RPI = 64 / VPR;                    // strip rows covered by one wave-wide store
        const int vr = lane / VPR, vc = (lane % VPR) * EPV;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float v = acc[i][j][e];
                    if (relu) v = fmaxf(v, 0.0f);
                    strip[(8 * (e >> 2) + (lane >> 5) * 4 + (e & 3)) * SLD + j * 32 + (lane & 31)] = v;
                }
            // Wave-private data: LDS operations of one wave execute in order, so the reads below see the writes above and the
            // next strip's writes cannot overtake them; no wait is needed, only a fence for the compiler's scheduler.
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int rr = 0; rr < 32; rr += RPI) {
                const int srow = rr + vr;
                const int row = m0 + wm0 + i * 32 + srow, col = n0 + wn0 + vc;
                const float *sp = strip + srow * SLD + vc;
                if (row < M && col < N) { // N is a multiple of EPV on this path: a vector is all in or all out
                    if constexpr (OUT_BF16) {
                        f32x4 x = *reinterpret_cast<const f32x4 *>(sp), y = *reinterpret_cast<const f32x4 *>(sp + 4);
                        u32x4 o = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(y[0], y[1]),
                                   pack_bf16x2(y[2], y[3])};
                        __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(reinterpret_cast<uint16_t *>(Cv) + (size_t)row * ldc + col));
                    } else {
                        __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(sp),
                                                    reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(Cv) + (size_t)row * ldc + col));
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// XCD-aware workgroup order: hardware workgroup numbers go round-robin over the 8 XCDs; hand every XCD a contiguous
// range of logical workgroups so tiles that share operands share an L2.  Returns -1 for padding workgroups.
__device__ __forceinline__ int logical_block(int per_xcd, int total)
{
    const int bid = blockIdx.x;
    const int logical = (bid % kXcds) * per_xcd + bid / kXcds;
    return logical < total ? logical : -1;
}

// Tile order inside one shard: column tiles are taken in groups of four; inside a group the row tiles run slowest and
// the group's columns fastest.  Workgroups that run at the same time then share a few column tiles of B and a few row
// tiles of A, and the A tiles are still in L2 when the next column group comes round.
__device__ __forceinline__ void grouped_tile(int t, int tiles_m, int tiles_n, int *tm, int *tn)
{
    constexpr int G = 4;
    const int per_group = tiles_m * G;
    const int g = t / per_group;
    const int r = t - g * per_group;
    const int width = tiles_n - g * G < G ? tiles_n - g * G : G;
    *tm = r / width;
    *tn = g * G + (r - *tm * width);
}

} // namespace core
} // namespace tt
