// The step between a convolution and a fully-connected layer: the image tensor [batch][channel][pixel] changes from
// the convolutions' storage (per shard a row-major (batch * pixels) x channels matrix) to the fully-connected layers'
// storage (per shard a row-major batch x (channels * pixels) matrix, channel-major columns), or back for the gradient.
//
// Sec. 4.5 of arXiv 1805.04170 cuts a convolution's tensors along batch and channel only; with channel-major columns a
// column cut of the flattened matrix is a channel cut, so the k-cut tilings of both sides are tilings of the same
// [batch][channel] grid and the step is a tiling conversion (Sec. 5.2) whose pieces are also transposed per image.
// One launch covers all shards; a workgroup moves a 64-pixel x 64-channel tile of one image through LDS so that both
// sides are accessed along their contiguous dimension.
#include <cstdint>
#include "tt_device.h"
#include "tt_internal.h"

namespace tt {
namespace {

constexpr int kFlatThreads = 256;
constexpr int kFlatTile = 64;

struct SideGrid {
    uint32_t maskR, maskC, maskX;
    uint32_t simgs;  // images per shard
    uint32_t schans; // channels per shard
};

struct FlattenParams {
    const void *src[kMaxShards];
    void *dst[kMaxShards];
    uint8_t rep_ids[kMaxShards]; // id bits of the r-th destination replica
    SideGrid S, D;
    uint32_t k, nrep;
    uint32_t channels, pixels;
    uint32_t cchunks; // 64-channel chunks per image
};

__device__ __forceinline__ uint32_t deposit_dev(uint32_t v, uint32_t mask, uint32_t k)
{
    uint32_t out = 0;
    int n = __popc(mask);
    for (int b = (int)k - 1; b >= 0; --b)
        if (mask & (1u << b)) { --n; if ((v >> n) & 1u) out |= 1u << b; }
    return out;
}

struct ElemLoc { uint32_t shard; uint64_t off; };

// where element (image n, channel c, pixel px) lives under a side's grid; IMAGE: (images * pixels) x channels rows,
// otherwise images x (channels * pixels)
template <bool IMAGE>
__device__ __forceinline__ ElemLoc locate_elem(const SideGrid &g, uint32_t k, uint32_t pixels, uint32_t n, uint32_t c, uint32_t px)
{
    const uint32_t rb = n / g.simgs, ni = n - rb * g.simgs;
    const uint32_t cb = c / g.schans, ci = c - cb * g.schans;
    ElemLoc e;
    e.shard = deposit_dev(rb, g.maskR, k) | deposit_dev(cb, g.maskC, k);
    e.off = IMAGE ? ((uint64_t)ni * pixels + px) * g.schans + ci : ((uint64_t)ni * g.schans + ci) * pixels + px;
    return e;
}

// TO_MATRIX: source is the image side.  Lanes run along channels on the image side and along pixels on the matrix side.
template <typename T, bool TO_MATRIX>
__global__ __launch_bounds__(kFlatThreads) void flatten_kernel(const FlattenParams p)
{
    __shared__ T tile[kFlatTile][kFlatTile + 1]; // [pixel][channel]
    const uint32_t n = blockIdx.y;
    const uint32_t cc = blockIdx.x % p.cchunks, pc = blockIdx.x / p.cchunks;
    const uint32_t c0 = cc * kFlatTile, p0 = pc * kFlatTile;
    const uint32_t lane = threadIdx.x & 63u, grp = threadIdx.x >> 6;

    for (uint32_t i = grp; i < (uint32_t)kFlatTile; i += kFlatThreads / 64) {
        const uint32_t c = TO_MATRIX ? c0 + lane : c0 + i;
        const uint32_t px = TO_MATRIX ? p0 + i : p0 + lane;
        if (c < p.channels && px < p.pixels) {
            const ElemLoc e = locate_elem<TO_MATRIX>(p.S, p.k, p.pixels, n, c, px);
            const T v = reinterpret_cast<const T *>(p.src[e.shard])[e.off]; // replica with all other id bits zero
            if (TO_MATRIX) tile[i][lane] = v; else tile[lane][i] = v;
        }
    }
    __syncthreads();
    for (uint32_t i = grp; i < (uint32_t)kFlatTile; i += kFlatThreads / 64) {
        const uint32_t c = TO_MATRIX ? c0 + i : c0 + lane;
        const uint32_t px = TO_MATRIX ? p0 + lane : p0 + i;
        if (c < p.channels && px < p.pixels) {
            const ElemLoc e = locate_elem<!TO_MATRIX>(p.D, p.k, p.pixels, n, c, px);
            const T v = TO_MATRIX ? tile[lane][i] : tile[i][lane];
            for (uint32_t r = 0; r < p.nrep; ++r) reinterpret_cast<T *>(p.dst[e.shard | p.rep_ids[r]])[e.off] = v;
        }
    }
}

bool side_grid(const tt_tiling &t, int k, int64_t batch, int64_t channels, SideGrid *out, Grid *g)
{
    if (!make_grid(t.cut, k, batch, channels, g)) return false;
    out->maskR = g->maskR;
    out->maskC = g->maskC;
    out->maskX = g->maskX;
    out->simgs = (uint32_t)g->srows;
    out->schans = (uint32_t)g->scols;
    return true;
}

template <typename T> tt_status launch_flatten_t(const FlattenParams &p, dim3 grid, bool to_matrix, hipStream_t s)
{
    if (to_matrix) hipLaunchKernelGGL((flatten_kernel<T, true>), grid, dim3(kFlatThreads), 0, s, p);
    else hipLaunchKernelGGL((flatten_kernel<T, false>), grid, dim3(kFlatThreads), 0, s, p);
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

} // namespace
} // namespace tt

extern "C" tt_status tt_flatten(void *const *dst, tt_tiling B, const void *const *src, tt_tiling A, int k, int64_t batch,
                                int64_t channels, int64_t pixels, int elem_bytes, int to_matrix, void *stream)
{
    using namespace tt;
    if (!dst || !src || !valid_k(k) || !valid_tiling(A, k) || !valid_tiling(B, k)) return TT_EINVAL;
    if (batch < 0 || channels < 0 || pixels < 0 || (elem_bytes != 2 && elem_bytes != 4)) return TT_EINVAL;
    Grid ga, gb;
    FlattenParams p;
    if (!side_grid(A, k, batch, channels, &p.S, &ga) || !side_grid(B, k, batch, channels, &p.D, &gb)) return TT_EINFEASIBLE;
    if (batch == 0 || channels == 0 || pixels == 0) return TT_OK;
    // grid.y carries the image number; per-shard offsets are 64-bit, the coordinates themselves 32-bit
    if (batch > 65535 || channels >= (int64_t(1) << 31) || pixels >= (int64_t(1) << 31) ||
        batch * pixels >= (int64_t(1) << 32))
        return TT_EUNSUPPORTED;
    const int n = 1 << k;
    for (int s = 0; s < kMaxShards; ++s) {
        p.src[s] = s < n ? src[s] : nullptr;
        p.dst[s] = s < n ? dst[s] : nullptr;
        p.rep_ids[s] = 0;
        if (s < n && (!src[s] || !dst[s] || reinterpret_cast<uintptr_t>(src[s]) % elem_bytes ||
                      reinterpret_cast<uintptr_t>(dst[s]) % elem_bytes))
            return TT_EINVAL;
    }
    p.k = (uint32_t)k;
    p.nrep = 1u << gb.kX;
    for (uint32_t r = 0; r < p.nrep; ++r) p.rep_ids[r] = (uint8_t)deposit(r, gb.maskX, k);
    p.channels = (uint32_t)channels;
    p.pixels = (uint32_t)pixels;
    p.cchunks = (uint32_t)((channels + kFlatTile - 1) / kFlatTile);
    const uint64_t gx = (uint64_t)p.cchunks * (uint64_t)((pixels + kFlatTile - 1) / kFlatTile);
    if (gx >= (uint64_t(1) << 31)) return TT_EUNSUPPORTED;
    const uint64_t bytes = (uint64_t)batch * channels * pixels * elem_bytes;
    ProfileScope scope(stream, TT_K_CONVERT, n, batch * pixels, channels, elem_bytes, bytes * (1u + p.nrep), 0);
    const dim3 grid((uint32_t)gx, (uint32_t)batch);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    return elem_bytes == 2 ? launch_flatten_t<uint16_t>(p, grid, to_matrix != 0, s)
                           : launch_flatten_t<uint32_t>(p, grid, to_matrix != 0, s);
}
