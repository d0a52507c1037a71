// Internal host-side helpers shared by the library's translation units.
#pragma once
#include <cstdlib>
#include <cstdint>
#include <cstddef>
#include "tensor_tiling.h"

namespace tt {

// Launch heuristics can be overridden through environment variables only in development builds (-DTT_TUNING); the
// product build reads no environment and every launch decision is a pure function of the call's arguments.
inline int tuning_int(const char *name, int dflt)
{
#ifdef TT_TUNING
    const char *e = std::getenv(name);
    return e ? std::atoi(e) : dflt;
#else
    (void)name;
    return dflt;
#endif
}


constexpr int kMaxShards = 1 << TT_MAX_K;

// Letter used internally for a cut whose shards hold different partial sums (output of form F3).
constexpr uint8_t kRed = 3;

inline bool valid_k(int k) { return k >= 0 && k <= TT_MAX_K; }

inline bool valid_tiling(const tt_tiling &t, int k)
{
    for (int j = 0; j < k; ++j)
        if (t.cut[j] > TT_REP) return false;
    return true;
}

// A k-cut tiling seen as a regular grid (flattening theorem, Sec. 4.4).
// Shard-id bit for cut j is bit (k-1-j).  maskR / maskC / maskX select the id bits of the R cuts, the C cuts and
// the remaining cuts (replicas, or partial-sum numbers for kRed).
struct Grid {
    int k = 0, kR = 0, kC = 0, kX = 0;
    uint32_t maskR = 0, maskC = 0, maskX = 0;
    int64_t rows = 0, cols = 0;   // full tensor
    int64_t srows = 0, scols = 0; // shard extent
};

// letters[j] in {TT_R, TT_C, anything else = extra}.  Returns false if the cut is uneven.
inline bool make_grid(const uint8_t *letters, int k, int64_t rows, int64_t cols, Grid *g)
{
    Grid out;
    out.k = k;
    out.rows = rows;
    out.cols = cols;
    for (int j = 0; j < k; ++j) {
        uint32_t b = 1u << (k - 1 - j);
        if (letters[j] == TT_R) { out.kR++; out.maskR |= b; }
        else if (letters[j] == TT_C) { out.kC++; out.maskC |= b; }
        else { out.kX++; out.maskX |= b; }
    }
    if (rows % (int64_t(1) << out.kR) || cols % (int64_t(1) << out.kC)) return false;
    out.srows = rows >> out.kR;
    out.scols = cols >> out.kC;
    *g = out;
    return true;
}

// bits of v scattered to the set positions of mask, most significant first (software pdep on <= 6 bits)
inline uint32_t deposit(uint32_t v, uint32_t mask, int k)
{
    uint32_t out = 0;
    int n = __builtin_popcount(mask);
    for (int b = k - 1; b >= 0; --b)
        if (mask & (1u << b)) { --n; if (v & (1u << n)) out |= 1u << b; }
    return out;
}
inline uint32_t extract(uint32_t s, uint32_t mask, int k)
{
    uint32_t out = 0;
    for (int b = k - 1; b >= 0; --b)
        if (mask & (1u << b)) out = (out << 1) | ((s >> b) & 1u);
    return out;
}

inline tt_tiling transpose_tiling(tt_tiling t, int k)
{
    for (int j = 0; j < k; ++j) t.cut[j] = t.cut[j] == TT_R ? TT_C : (t.cut[j] == TT_C ? TT_R : TT_REP);
    return t;
}

// aligned tilings of a form sequence (Sec. 4.2.1)
inline void aligned_tilings(const uint8_t *forms, int k, tt_tiling *aX, tt_tiling *aY, uint8_t *aZ /* k letters, kRed for F3 */)
{
    static const uint8_t ax[3] = {TT_R, TT_REP, TT_C}, ay[3] = {TT_REP, TT_C, TT_R}, az[3] = {TT_R, TT_C, kRed};
    for (int j = 0; j < k; ++j) {
        if (aX) aX->cut[j] = ax[forms[j]];
        if (aY) aY->cut[j] = ay[forms[j]];
        if (aZ) aZ[j] = az[forms[j]];
    }
}

inline bool same_tiling(const tt_tiling &a, const tt_tiling &b, int k)
{
    for (int j = 0; j < k; ++j) if (a.cut[j] != b.cut[j]) return false;
    return true;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- cost model (planner.cpp) used by the execute calls to pick default forms
// Matmul Z = X Y with tensors given as (rows, cols, mult) and tilings already expressed on the operands as multiplied.
struct CostTensor { int64_t rows, cols, mult; };
uint64_t matmul_cost(const CostTensor &X, const CostTensor &Y, const CostTensor &Z, int64_t M, int64_t K, int64_t N,
                     const uint8_t *tx, const uint8_t *ty, const uint8_t *tz, int k, uint8_t *forms_out,
                     uint64_t *level_out);

// ---- internal launchers (device pointers arrays are host arrays)
tt_status launch_convert(void *const *dst, const uint8_t *B, const void *const *src, const uint8_t *A,
                         const void *const *mask, const uint8_t *Am, int k, int64_t rows, int64_t cols,
                         int elem_bytes, int gate_dtype, bool dst_unique /* replicas of B alias one buffer */,
                         void *stream);
// ksplit > 1: every shard comes as ksplit partial buffers (partials[s * ksplit + c]) that are summed as well.
// per_block: the partial sums of an output block are not held shard by shard but as ksplit buffers per block (any
// ksplit >= 1), partials[b * ksplit + c] with b the block's shard id with zero bits at the kRed cuts.
tt_status launch_reduce(void *const *dst, const uint8_t *B, int out_dtype, const float *const *partials,
                        const uint8_t *zletters /* R, C or kRed per cut */, int k, int64_t rows, int64_t cols, int act,
                        int ksplit, void *stream, bool per_block = false);
// ksplit > 1: each shard's K range is cut into ksplit chunks; chunk c of shard s writes C[s * ksplit + c]
tt_status launch_gemm(int count, const void *const *A, const void *const *B, void *const *C, int64_t M, int64_t N,
                      int64_t K, int trans_a, int trans_b, int in_dtype, int out_dtype, int act, int ksplit,
                      void *stream);

// Persistent software-pipelined MFMA engine (gemm3.hip); bf16 operands.  a_kc / b_kc: the operand's rows (m / n) have
// K contiguous.  TT_EUNSUPPORTED when the shape does not meet the kernel's assumptions (the caller falls back).
tt_status launch_gemm_v3(int count, const void *const *A, const void *const *B, void *const *C, int64_t M, int64_t N,
                         int64_t K, int64_t lda, int64_t ldb, int64_t ldc, bool a_kc, bool b_kc, int out_dtype, int relu,
                         bool vec, int ksplit, int64_t kchunk, void *stream);

// Same contract for the 256 x 128 engine with two workgroups per CU (gemm_core4.h); K a multiple of 32.
tt_status launch_gemm_v5(int count, const void *const *A, const void *const *B, void *const *C, int64_t M, int64_t N,
                         int64_t K, int64_t lda, int64_t ldb, int64_t ldc, int relu, void *stream);
tt_status launch_gemm_v4(int count, const void *const *A, const void *const *B, void *const *C, int64_t M, int64_t N,
                         int64_t K, int64_t lda, int64_t ldb, int64_t ldc, bool a_kc, bool b_kc, int out_dtype, int relu,
                         bool vec, int ksplit, int64_t kchunk, void *stream);
// The same tile with K tiles of 64 and one workgroup per CU for products whose left operand has K contiguous
// (gemm_core6.h); K and a K chunk multiples of 64.
tt_status launch_gemm_v6(int count, const void *const *A, const void *const *B, void *const *C, int64_t M, int64_t N,
                         int64_t K, int64_t lda, int64_t ldb, int64_t ldc, bool b_kc, int out_dtype, int relu, bool vec,
                         int ksplit, int64_t kchunk, void *stream);

// Convolution shard products (conv.hip).  op TT_OP_FWD: A = X shards, B = filter shards, C = Y shards;
// TT_OP_DGRAD: A = dY, B = filters, C = dX;  TT_OP_WGRAD: A = dY, B = X, C = dW.  Ns images, Cs input channels and
// Ks output channels per shard; bf16 operands on the MFMA engines, fp32 operands (in_dtype TT_F32) on plain kernels
// that follow the definition term by term.
// flip_ws (TT_OP_DGRAD only, optional): per shard a 16-byte aligned scratch buffer of the filter shard's size; when
// given (and R == S, pad <= R - 1) the filters are flipped into it and the product runs on the forward kernel.
tt_status launch_conv(int op, int count, const void *const *A, const void *const *B, void *const *C, int64_t Ns,
                      int64_t Cs, int64_t Ks, int64_t H, int64_t W, int64_t R, int64_t S, int64_t pad, int out_dtype,
                      int act, void *stream, void *const *flip_ws = nullptr, int in_dtype = TT_BF16);

// Forward products (TT_OP_FWD) or data gradients (TT_OP_DGRAD, run as forward products of dY with flipped filters) of
// groups of `members` shards that share their left operand, one product per group with the members' columns side by side
// (conv.hip).  A[g]; B[g * members + m]; C[g * members + m]; cols: columns per member; red: contraction channels per pixel.
// TT_EUNSUPPORTED when the members' filter blocks do not lie one after the other or a shape does not fit (the caller runs
// launch_conv shard by shard).
tt_status launch_conv_fused(int op, int groups, int members, const void *const *A, const void *const *B, void *const *C,
                            int64_t Ns, int64_t cols, int64_t red, int64_t H, int64_t W, int64_t R, int64_t S, int64_t pad,
                            int out_dtype, int act, void *stream, void *const *flip_ws);

// Weight-gradient products with every output block's reduction over pixels (the pixels of all shards that an F3 cut
// makes add up into that block) cut into `parts` equal runs, one fp32 partial sum each (conv.hip).  A = dY shards and
// B = X shards by shard id; C[blk * parts + part]; blk_ids[b] / red_ids[q]: id bits of block b / of a block's q-th shard.
// TT_EUNSUPPORTED when the shapes do not fit (the caller takes launch_conv).
tt_status launch_conv_wgrad_split(int k, int nblk, int nred, const uint8_t *blk_ids, const uint8_t *red_ids, int parts,
                                  const void *const *A, const void *const *B, void *const *C, int64_t Ns, int64_t Cs,
                                  int64_t Ks, int64_t H, int64_t W, int64_t R, int64_t S, int64_t pad,
                                  int engine /* 1: 256 x 128 tiles, two workgroups per CU; 2: 256 x 256, straight into LDS */,
                                  void *stream);

// ---- optional kernel timing (profile.cpp).  A scope object brackets one launch with two events when the calling
// thread has recording switched on; otherwise it does nothing.
struct ProfileScope {
    ProfileScope(void *stream, int kernel, int count, int64_t d0, int64_t d1, int64_t d2, uint64_t bytes, uint64_t flops);
    ~ProfileScope();
    int slot;
    void *stream;
};

} // namespace tt
