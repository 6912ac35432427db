// Mask-side kernels: mask propagation (Sec. III-B), ordered compaction of the kept
// positions (Sec. III-A: which patches become columns) fused with it, zero-fill of
// the irrelevant output rows for the direct-convolution path, and the max-pool
// helper.  All of them are byte/row movers bound by HBM bandwidth or launch latency.
#include "fc_internal.hpp"

namespace fc {

// ---------------------------------------------------------------------------
// Mask propagation: one thread per output byte; the byte under the centre tap.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_mask_downsample(const uint8_t *__restrict__ mask_in, int n, int h,
                                                         int w, int ch0, int cw0, int sh, int sw, int ho,
                                                         int wo, uint8_t *__restrict__ mask_out)
{
    const int64_t total = (int64_t)n * ho * wo;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < total;
         p += (int64_t)gridDim.x * blockDim.x) {
        // (position counts fit 31 bits: 32-bit divisions)
        const uint32_t t = (uint32_t)p / (uint32_t)wo;
        const int ow = (int)((uint32_t)p - t * (uint32_t)wo);
        const int b = (int)(t / (uint32_t)ho);
        const int oh = (int)(t - (uint32_t)b * (uint32_t)ho);
        int ih = min(max(oh * sh + ch0, 0), h - 1);
        int iw = min(max(ow * sw + cw0, 0), w - 1);
        mask_out[p] = mask_in[(b * h + ih) * w + iw] ? 1 : 0;
    }
}

hipError_t launch_mask_downsample(const uint8_t *mask_in, int n, int h, int w, int kh, int kw, int sh,
                                  int sw, int ph, int pw, int dh, int dw, int ho, int wo,
                                  uint8_t *mask_out, hipStream_t s)
{
    const int64_t total = (int64_t)n * ho * wo;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 65536) blocks = 65536;
    const int ch0 = -ph + dh * ((kh - 1) / 2), cw0 = -pw + dw * ((kw - 1) / 2);
    hipLaunchKernelGGL(k_mask_downsample, dim3(blocks), dim3(256), 0, s, mask_in, n, h, w, ch0, cw0, sh, sw,
                       ho, wo, mask_out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Patch labels by a window rule (the other readings of "a patch labelled irrelevant",
// Sec. III-A): kept if ANY pixel of the window is relevant, or only if ALL are.  Pixels
// outside the image are not part of the window.  One thread per output byte; the
// window's mask bytes come through the cache (neighbouring positions share them).
// ---------------------------------------------------------------------------
template <bool ALL>
__global__ __launch_bounds__(256) void k_mask_window(const uint8_t *__restrict__ mask_in, int n, int h, int w,
                                                     int kh, int kw, int sh, int sw, int ph, int pw, int dh,
                                                     int dw, int ho, int wo, uint8_t *__restrict__ mask_out)
{
    const int64_t total = (int64_t)n * ho * wo;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < total;
         p += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t t = (uint32_t)p / (uint32_t)wo; // (position counts fit 31 bits)
        const int ow = (int)((uint32_t)p - t * (uint32_t)wo);
        const uint32_t b = t / (uint32_t)ho;
        const int oh = (int)(t - b * (uint32_t)ho);
        const uint8_t *img = mask_in + (int64_t)b * ((int64_t)h * w);
        int inside = 0, relevant = 0;
        for (int i = 0; i < kh; ++i) {
            const int ih = oh * sh - ph + i * dh;
            if (ih < 0 || ih >= h) continue;
            for (int j = 0; j < kw; ++j) {
                const int iw = ow * sw - pw + j * dw;
                if (iw < 0 || iw >= w) continue;
                ++inside;
                relevant += img[(int64_t)ih * w + iw] != 0;
            }
        }
        mask_out[p] = ALL ? (inside > 0 && relevant == inside) : (relevant > 0);
    }
}

hipError_t launch_mask_window(const uint8_t *mask_in, int n, int h, int w, int kh, int kw, int sh, int sw,
                              int ph, int pw, int dh, int dw, int ho, int wo, bool all, uint8_t *mask_out,
                              hipStream_t s)
{
    const int64_t total = (int64_t)n * ho * wo;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 65536) blocks = 65536;
    if (all)
        hipLaunchKernelGGL(k_mask_window<true>, dim3(blocks), dim3(256), 0, s, mask_in, n, h, w, kh, kw, sh, sw, ph,
                           pw, dh, dw, ho, wo, mask_out);
    else
        hipLaunchKernelGGL(k_mask_window<false>, dim3(blocks), dim3(256), 0, s, mask_in, n, h, w, kh, kw, sh, sw, ph,
                           pw, dh, dw, ho, wo, mask_out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Ordered compaction, fused with the mask propagation.  A block owns 4096
// consecutive output positions, a lane 16 of them.  The output-resolution mask is
// never needed as an input: every kernel recomputes a position's flag from the
// input mask (centre tap), which for a stride-1 "same" layer is one 128-bit load
// per lane.  Ranks inside a block come from a wave prefix sum (shuffles inside a
// wave, LDS across the four waves); the indices are staged in LDS in order and
// copied out coalesced.  No block ever waits on another block, so every grid drains:
//   - small inputs (up to 16 blocks): ONE launch; a block counts the kept
//     positions of all blocks before it by itself (at most 60 KB of mask re-read
//     per block, out of L2, all loads in flight together);
//   - larger inputs: two launches, per-block counts first, then prefix + scatter.
// ---------------------------------------------------------------------------

// sum of v over the block (all threads get it); scratch holds one int per wave
__device__ __forceinline__ int block_sum(int v, int *scratch)
{
    // wave total through ballots of the value's bits would need its width; use the scan
    const int incl = wave_inclusive_scan(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 63) scratch[threadIdx.x >> 6] = incl;
    __syncthreads();
    int s = 0;
#pragma unroll
    for (int i = 0; i < kCompactBlockThreads / 64; ++i) s += scratch[i];
    return s;
}

__global__ __launch_bounds__(kCompactBlockThreads) void k_compact_count(MaskGeom g,
                                                                         const uint8_t *__restrict__ mask_in,
                                                                         int32_t *__restrict__ block_counts)
{
    __shared__ int wave_sum[kCompactBlockThreads / 64];
    const int64_t p0 = (int64_t)blockIdx.x * kCompactBlockElems + (int64_t)threadIdx.x * kCompactBytesPerThread;
    const int c = __popc(kept_flags16(g, mask_in, p0));
    // wave total through ballots of the count's bits (counts are 0..16: 5 bits)
    int total = 0;
#pragma unroll
    for (int b = 0; b < 5; ++b) total += __popcll(__ballot((c >> b) & 1)) << b;
    if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = total;
    __syncthreads();
    if (threadIdx.x == 0) {
        int s = 0;
#pragma unroll
        for (int i = 0; i < kCompactBlockThreads / 64; ++i) s += wave_sum[i];
        block_counts[blockIdx.x] = s;
    }
}

// SELF = true: the block counts everything before it by itself (single launch);
// otherwise it sums the per-block counts of the first launch.
template <bool SELF>
__global__ __launch_bounds__(kCompactBlockThreads) void k_compact_scatter(MaskGeom g,
                                                                           const uint8_t *__restrict__ mask_in,
                                                                           const int32_t *__restrict__ block_counts,
                                                                           uint8_t *__restrict__ mask_out,
                                                                           int32_t *__restrict__ idx,
                                                                           int32_t *__restrict__ count,
                                                                           CompactExtras ex)
{
    __shared__ int wave_sum[kCompactBlockThreads / 64];
    __shared__ int scratch[kCompactBlockThreads / 64];
    __shared__ int32_t stage[kCompactBlockElems];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // offset of this block = number of kept positions in all blocks before it
    int part = 0;
    if (SELF) {
        // all loads of the (at most kCompactSingleLaunchBlocks - 1) earlier chunks are
        // independent: unrolled, so that they are in flight together
#pragma unroll
        for (int pb = 0; pb < kCompactSingleLaunchBlocks - 1; ++pb)
            if (pb < (int)blockIdx.x)
                part += __popc(kept_flags16(g, mask_in, (int64_t)pb * kCompactBlockElems + (int64_t)tid * 16));
    } else {
        for (int i = tid; i < (int)blockIdx.x; i += kCompactBlockThreads) part += block_counts[i];
    }
    const int block_base = block_sum(part, scratch);

    const int64_t p0 = (int64_t)blockIdx.x * kCompactBlockElems + (int64_t)tid * kCompactBytesPerThread;
    const uint32_t flags = kept_flags16(g, mask_in, p0);
    if (mask_out && g.packed_out) {
        // sixteen labels = one 16-bit piece of the packed mask (zeros past the end, up to a whole word)
        if (p0 < ((g.m + 63) & ~(int64_t)63)) reinterpret_cast<uint16_t *>(mask_out)[p0 >> 4] = (uint16_t)flags;
    } else if (mask_out) {
        if (p0 + 16 <= g.m) {
            uint32_t wds[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                wds[q] = ((flags >> (4 * q)) & 1u) | (((flags >> (4 * q + 1)) & 1u) << 8) |
                         (((flags >> (4 * q + 2)) & 1u) << 16) | (((flags >> (4 * q + 3)) & 1u) << 24);
            *reinterpret_cast<uint4 *>(mask_out + p0) = make_uint4(wds[0], wds[1], wds[2], wds[3]);
        } else {
            for (int j = 0; j < 16 && p0 + j < g.m; ++j) mask_out[p0 + j] = (flags >> j) & 1u;
        }
    }
    const int c = __popc(flags);
    const int incl = wave_inclusive_scan(c);
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();

    int before = 0, block_total = 0;
#pragma unroll
    for (int i = 0; i < kCompactBlockThreads / 64; ++i) {
        if (i < wave) before += wave_sum[i];
        block_total += wave_sum[i];
    }
    int pos = before + incl - c;
    uint32_t f = flags;
    while (f) {
        const int j = __ffs(f) - 1;
        f &= f - 1;
        stage[pos++] = (int32_t)(p0 + j);
    }
    __syncthreads();
    for (int i = tid; i < block_total; i += kCompactBlockThreads) idx[(int64_t)block_base + i] = stage[i];
    if (blockIdx.x == gridDim.x - 1 && tid == 0) *count = block_base + block_total;

    // on the side, for the convolution that follows: clear its split-K tile counters
    if (ex.zero && blockIdx.x == 0)
        for (int i = tid; i < ex.zero_n; i += kCompactBlockThreads) ex.zero[i] = 0;
}

hipError_t launch_compact(const MaskGeom &g_in, const uint8_t *mask_in, uint8_t *mask_out, int32_t *idx,
                          int32_t *count, int32_t *block_counts, const CompactExtras &extras, hipStream_t s)
{
    MaskGeom g = g_in;
    if (!g.packed_in && (reinterpret_cast<uintptr_t>(mask_in) & 15u)) g.identity = 0; // the 128-bit path needs alignment
    const int nb = (int)compact_blocks(g.m);
    if (nb <= kCompactSingleLaunchBlocks) {
        hipLaunchKernelGGL(k_compact_scatter<true>, dim3(nb), dim3(kCompactBlockThreads), 0, s, g, mask_in,
                           (const int32_t *)nullptr, mask_out, idx, count, extras);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_compact_count, dim3(nb), dim3(kCompactBlockThreads), 0, s, g, mask_in, block_counts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_compact_scatter<false>, dim3(nb), dim3(kCompactBlockThreads), 0, s, g, mask_in,
                       (const int32_t *)block_counts, mask_out, idx, count, extras);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Kept positions in tile order (Sec. III-A fixes which patches become columns, not their
// order): tiles of tile_h x tile_w positions, row-major over the tiles of an image, row-major
// inside a tile.  A thread owns one row of one tile (up to 32 positions), a block 256 such rows
// in list order; two launches: per-block counts, then offsets + ordered scatter.
// ---------------------------------------------------------------------------
struct TiledGeom {
    int32_t n, ho, wo, th, tw, tiles_y, tiles_x;
    int32_t rows; // n * tiles_y * tiles_x * th tile rows (those below the image are empty)
};

// bit j = position (row of a tile, column j) is kept; *first = flat position of column 0
__device__ __forceinline__ uint32_t tiled_row_flags(const TiledGeom &g, const uint8_t *__restrict__ mask, int r,
                                                    int *first)
{
    *first = 0;
    if (r >= g.rows) return 0;
    const uint32_t t = (uint32_t)r / (uint32_t)g.th;
    const int dy = (int)((uint32_t)r - t * (uint32_t)g.th);
    const uint32_t t2 = t / (uint32_t)g.tiles_x;
    const int tx = (int)(t - t2 * (uint32_t)g.tiles_x);
    const int b = (int)(t2 / (uint32_t)g.tiles_y);
    const int ty = (int)(t2 - (uint32_t)b * (uint32_t)g.tiles_y);
    const int y = ty * g.th + dy, x0 = tx * g.tw;
    if (y >= g.ho) return 0;
    const int p = (b * g.ho + y) * g.wo + x0;
    *first = p;
    const int nx = min(g.tw, g.wo - x0);
    uint32_t flags = 0;
    if (nx == 16 && ((reinterpret_cast<uintptr_t>(mask) + (uintptr_t)p) & 15u) == 0) {
        const uint4 v = *reinterpret_cast<const uint4 *>(mask + p);
        const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) flags |= ((wds[q] >> (8 * bb)) & 0xffu) ? (1u << (4 * q + bb)) : 0u;
    } else {
        uint8_t got[32];
#pragma unroll
        for (int j = 0; j < 32; ++j) got[j] = j < nx ? mask[p + j] : (uint8_t)0;
#pragma unroll
        for (int j = 0; j < 32; ++j) flags |= got[j] ? (1u << j) : 0u;
    }
    return flags;
}

__global__ __launch_bounds__(kCompactBlockThreads) void k_tiled_count(TiledGeom g, const uint8_t *__restrict__ mask,
                                                                       int32_t *__restrict__ block_counts)
{
    __shared__ int scratch[kCompactBlockThreads / 64];
    int first;
    const uint32_t flags = tiled_row_flags(g, mask, (int)(blockIdx.x * kCompactBlockThreads + threadIdx.x), &first);
    const int total = block_sum(__popc(flags), scratch);
    if (threadIdx.x == 0) block_counts[blockIdx.x] = total;
}

__global__ __launch_bounds__(kCompactBlockThreads) void k_tiled_scatter(TiledGeom g, const uint8_t *__restrict__ mask,
                                                                         const int32_t *__restrict__ block_counts,
                                                                         int32_t *__restrict__ idx,
                                                                         int32_t *__restrict__ count)
{
    __shared__ int wave_sum[kCompactBlockThreads / 64];
    __shared__ int scratch[kCompactBlockThreads / 64];
    __shared__ int32_t stage[kCompactBlockThreads * 32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int part = 0;
    for (int i = tid; i < (int)blockIdx.x; i += kCompactBlockThreads) part += block_counts[i];
    const int block_base = block_sum(part, scratch);
    int first;
    const uint32_t flags = tiled_row_flags(g, mask, (int)(blockIdx.x * kCompactBlockThreads + tid), &first);
    const int c = __popc(flags);
    const int incl = wave_inclusive_scan(c);
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int before = 0, block_total = 0;
#pragma unroll
    for (int i = 0; i < kCompactBlockThreads / 64; ++i) {
        if (i < wave) before += wave_sum[i];
        block_total += wave_sum[i];
    }
    int pos = before + incl - c;
    uint32_t f = flags;
    while (f) {
        const int j = __ffs(f) - 1;
        f &= f - 1;
        stage[pos++] = first + j;
    }
    __syncthreads();
    for (int i = tid; i < block_total; i += kCompactBlockThreads) idx[(int64_t)block_base + i] = stage[i];
    if (blockIdx.x == gridDim.x - 1 && tid == 0) *count = block_base + block_total;
}

hipError_t launch_compact_tiled(const uint8_t *mask, int n, int ho, int wo, int tile_h, int tile_w, int32_t *idx,
                                int32_t *count, int32_t *block_counts, hipStream_t s)
{
    TiledGeom g;
    g.n = n; g.ho = ho; g.wo = wo; g.th = tile_h; g.tw = tile_w;
    g.tiles_y = (ho + tile_h - 1) / tile_h;
    g.tiles_x = (wo + tile_w - 1) / tile_w;
    g.rows = n * g.tiles_y * g.tiles_x * tile_h;
    const int nb = (g.rows + kCompactBlockThreads - 1) / kCompactBlockThreads;
    hipLaunchKernelGGL(k_tiled_count, dim3(nb), dim3(kCompactBlockThreads), 0, s, g, mask, block_counts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_tiled_scatter, dim3(nb), dim3(kCompactBlockThreads), 0, s, g, mask,
                       (const int32_t *)block_counts, idx, count);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Mask pyramid (Sec. III-B: one mask, rescaled to every layer's size): the masks and
// the kept-position lists of all levels from the input mask, in two launches.
// Level l is the centre-tap rescaling of level l - 1, so a position of level l reads
// the input mask through the composition of the levels' index maps; no level waits for
// another.  Launch 1 writes every level's 0/1 mask and per-block counts, launch 2 turns
// the counts into offsets and writes the ordered lists.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int pyramid_level_of(const PyramidArgs &a, int block)
{
    int l = 0;
#pragma unroll
    for (int i = 1; i < kMaxPyramidLevels; ++i)
        if (i < a.levels && block >= a.block0[i]) l = i;
    return l;
}

__global__ __launch_bounds__(kCompactBlockThreads) void k_pyramid_masks(PyramidArgs a,
                                                                         const uint8_t *__restrict__ mask_in,
                                                                         int32_t *__restrict__ block_counts)
{
    __shared__ int scratch[kCompactBlockThreads / 64];
    const int l = pyramid_level_of(a, blockIdx.x);
    const int64_t m = a.m[l];
    const int64_t p0 = (int64_t)(blockIdx.x - a.block0[l]) * kCompactBlockElems +
                       (int64_t)threadIdx.x * kCompactBytesPerThread;
    uint32_t flags = 0;
    if (l == 0 && a.identity0 && a.packed_in) {
        if (p0 < m) {
            flags = reinterpret_cast<const uint16_t *>(mask_in)[p0 >> 4];
            if (p0 + 16 > m) flags &= (1u << (uint32_t)(m - p0)) - 1u;
        }
    } else if (l == 0 && a.identity0 && p0 + 16 <= m) {
        // the first level keeps the resolution of an aligned input mask: one 128-bit load
        const uint4 v = *reinterpret_cast<const uint4 *>(mask_in + p0);
        const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int b = 0; b < 4; ++b) flags |= ((wds[q] >> (8 * b)) & 0xffu) ? (1u << (4 * q + b)) : 0u;
    } else if (p0 < m) {
        // (positions fit 31 bits; the level's parameters are read with constant indices, so they
        // sit in scalar registers instead of being fetched again for every position)
        const int wl = a.w[l + 1], hl = a.h[l + 1];
        const uint32_t t = fast_div((uint32_t)p0, a.div_w[l]);
        int ow = (int)((uint32_t)p0 - t * (uint32_t)wl);
        int b = (int)fast_div(t, a.div_h[l]);
        int oh = (int)(t - (uint32_t)b * (uint32_t)hl);
        // a row / column of level l seen through all levels down to the input mask
        auto row_in = [&](int v) {
#pragma unroll
            for (int q = kMaxPyramidLevels - 1; q >= 0; --q)
                if (q <= l) v = min(max(v * a.sh[q] + a.ch0[q], 0), a.h[q] - 1);
            return v;
        };
        auto col_in = [&](int v) {
#pragma unroll
            for (int q = kMaxPyramidLevels - 1; q >= 0; --q)
                if (q <= l) v = min(max(v * a.sw[q] + a.cw0[q], 0), a.w[q] - 1);
            return v;
        };
        int row_at = (b * a.h[0] + row_in(oh)) * a.w[0];
        // addresses first, then all sixteen bytes in flight together
        int at[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            at[j] = p0 + j < m ? row_at + col_in(ow) : -1;
            if (++ow == wl) {
                ow = 0;
                if (++oh == hl) {
                    oh = 0;
                    ++b;
                }
                row_at = (b * a.h[0] + row_in(oh)) * a.w[0];
            }
        }
        if (a.packed_in) {
            uint32_t got[16];
#pragma unroll
            for (int j = 0; j < 16; ++j)
                got[j] = at[j] >= 0 ? reinterpret_cast<const uint32_t *>(mask_in)[at[j] >> 5] : 0u;
#pragma unroll
            for (int j = 0; j < 16; ++j) flags |= ((got[j] >> (at[j] & 31)) & 1u) << j;
        } else {
            uint8_t got[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) got[j] = at[j] >= 0 ? mask_in[at[j]] : (uint8_t)0;
#pragma unroll
            for (int j = 0; j < 16; ++j) flags |= got[j] ? (1u << j) : 0u;
        }
    }
    if (a.packed_out) {
        if (p0 < ((m + 63) & ~(int64_t)63)) reinterpret_cast<uint16_t *>(a.mask_out[l])[p0 >> 4] = (uint16_t)flags;
    } else if (p0 < m) {
        uint8_t *mo = a.mask_out[l];
        if (p0 + 16 <= m && (reinterpret_cast<uintptr_t>(mo) & 15u) == 0) {
            uint32_t wds[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                wds[q] = ((flags >> (4 * q)) & 1u) | (((flags >> (4 * q + 1)) & 1u) << 8) |
                         (((flags >> (4 * q + 2)) & 1u) << 16) | (((flags >> (4 * q + 3)) & 1u) << 24);
            *reinterpret_cast<uint4 *>(mo + p0) = make_uint4(wds[0], wds[1], wds[2], wds[3]);
        } else {
            for (int j = 0; j < 16 && p0 + j < m; ++j) mo[p0 + j] = (flags >> j) & 1u;
        }
    }
    const int total = block_sum(__popc(flags), scratch);
    if (threadIdx.x == 0) block_counts[blockIdx.x] = total;
}

__global__ __launch_bounds__(kCompactBlockThreads) void k_pyramid_lists(PyramidArgs a,
                                                                         const int32_t *__restrict__ block_counts)
{
    __shared__ int wave_sum[kCompactBlockThreads / 64];
    __shared__ int scratch[kCompactBlockThreads / 64];
    __shared__ int32_t stage[kCompactBlockElems];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l = pyramid_level_of(a, blockIdx.x);
    const int64_t m = a.m[l];
    const int first = a.block0[l], last = a.block0[l + 1] - 1;

    int part = 0;
    for (int i = first + tid; i < (int)blockIdx.x; i += kCompactBlockThreads) part += block_counts[i];
    const int block_base = block_sum(part, scratch);

    // the level's own 0/1 mask, written by the first launch
    const int64_t p0 = (int64_t)(blockIdx.x - first) * kCompactBlockElems + (int64_t)tid * kCompactBytesPerThread;
    const uint8_t *mo = a.mask_out[l];
    uint32_t flags = 0;
    if (a.packed_out) {
        if (p0 < m) flags = reinterpret_cast<const uint16_t *>(mo)[p0 >> 4]; // (zeros past the end)
    } else if (p0 + 16 <= m && (reinterpret_cast<uintptr_t>(mo) & 15u) == 0) {
        const uint4 v = *reinterpret_cast<const uint4 *>(mo + p0);
        const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int b = 0; b < 4; ++b) flags |= ((wds[q] >> (8 * b)) & 0xffu) ? (1u << (4 * q + b)) : 0u;
    } else {
        for (int j = 0; j < 16 && p0 + j < m; ++j)
            if (mo[p0 + j]) flags |= 1u << j;
    }
    const int c = __popc(flags);
    const int incl = wave_inclusive_scan(c);
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int before = 0, block_total = 0;
#pragma unroll
    for (int i = 0; i < kCompactBlockThreads / 64; ++i) {
        if (i < wave) before += wave_sum[i];
        block_total += wave_sum[i];
    }
    int pos = before + incl - c;
    uint32_t f = flags;
    while (f) {
        const int j = __ffs(f) - 1;
        f &= f - 1;
        stage[pos++] = (int32_t)(p0 + j);
    }
    __syncthreads();
    int32_t *idx = a.idx[l];
    for (int i = tid; i < block_total; i += kCompactBlockThreads) idx[(int64_t)block_base + i] = stage[i];
    if ((int)blockIdx.x == last && tid == 0) *a.count[l] = block_base + block_total;
}

hipError_t launch_mask_pyramid(const PyramidArgs &a, const uint8_t *mask_in, int32_t *block_counts, hipStream_t s)
{
    const int nb = a.block0[a.levels];
    hipLaunchKernelGGL(k_pyramid_masks, dim3(nb), dim3(kCompactBlockThreads), 0, s, a, mask_in, block_counts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_pyramid_lists, dim3(nb), dim3(kCompactBlockThreads), 0, s, a,
                       (const int32_t *)block_counts);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Packed masks: one bit per pixel.  Packing: a thread turns sixteen bytes into sixteen bits.
// Rescaling (centre tap) between the two forms: sixteen output labels per thread.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_mask_rescale(MaskGeom g, const uint8_t *__restrict__ mask_in,
                                                      uint8_t *__restrict__ mask_out)
{
    const int64_t padded = g.packed_out ? ((g.m + 63) & ~(int64_t)63) : g.m;
    for (int64_t p0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 16; p0 < padded; p0 += (int64_t)gridDim.x * 256 * 16) {
        const uint32_t flags = kept_flags16(g, mask_in, p0);
        if (g.packed_out) {
            reinterpret_cast<uint16_t *>(mask_out)[p0 >> 4] = (uint16_t)flags;
        } else {
            for (int j = 0; j < 16 && p0 + j < g.m; ++j) mask_out[p0 + j] = (flags >> j) & 1u;
        }
    }
}

hipError_t launch_mask_rescale(const MaskGeom &g_in, const uint8_t *mask_in, uint8_t *mask_out, hipStream_t s)
{
    MaskGeom g = g_in;
    if (!g.packed_in && (reinterpret_cast<uintptr_t>(mask_in) & 15u)) g.identity = 0; // the 128-bit path needs alignment
    const int64_t threads = (g.m + 15) / 16 + 4;
    int64_t blocks = (threads + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_mask_rescale, dim3((unsigned)blocks), dim3(256), 0, s, g, mask_in, mask_out);
    return hipGetLastError();
}

hipError_t launch_mask_pack(const uint8_t *mask, int64_t m, uint64_t *bits, hipStream_t s)
{
    // a flat mask is a 1 x 1 x m image seen through a 1x1 stride-1 window
    MaskGeom g = mask_geom(1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1, 1, 1);
    g.w = g.wo = (int32_t)m;
    g.m = m;
    g.packed_out = 1;
    return launch_mask_rescale(g, mask, reinterpret_cast<uint8_t *>(bits), s);
}

// ---------------------------------------------------------------------------
// Zero-fill of the irrelevant output rows: a lane owns 16 bytes of one row.
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool position_kept(const Geom &g, const uint8_t *__restrict__ mask_in,
                                              const uint8_t *__restrict__ mask_out, int64_t p)
{
    const bool packed = (g.flags & FC_PACKED_MASKS) != 0;
    if (mask_out) return mask_at(mask_out, p, packed);
    const uint32_t t = (uint32_t)p / (uint32_t)g.wo; // (position counts fit 31 bits)
    const int ow = (int)((uint32_t)p - t * (uint32_t)g.wo);
    const int b = (int)(t / (uint32_t)g.ho);
    const int oh = (int)(t - (uint32_t)b * (uint32_t)g.ho);
    int ih = min(max(oh * g.sh - g.ph + g.dh * ((g.kh - 1) / 2), 0), g.h - 1);
    int iw = min(max(ow * g.sw - g.pw + g.dw * ((g.kw - 1) / 2), 0), g.w - 1);
    return mask_at(mask_in, (int64_t)(b * g.h + ih) * g.w + iw, packed);
}

// Rows of whole 16-byte pieces: a wave looks at 64 positions at a time (one label each), lists
// the irrelevant ones in LDS in order, and then all its lanes store 16-byte pieces of those
// rows, so the stores are dense and none of them waits for a label.  The labels of the next 64
// positions are requested before the stores of the current ones.
__global__ __launch_bounds__(256) void k_zero_fill16(Geom g, const uint8_t *__restrict__ mask_in,
                                                     const uint8_t *__restrict__ mask_out,
                                                     uint4 *__restrict__ out, int chunks_per_row)
{
    __shared__ int32_t dropped_s[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t *dropped = dropped_s[wave];
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int64_t step = nwaves * 64;
    typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));
    const u32x4_nt zero4 = {0u, 0u, 0u, 0u};
    u32x4_nt *o4 = reinterpret_cast<u32x4_nt *>(out);
    int64_t p0 = ((int64_t)blockIdx.x * 4 + wave) * 64;
    bool kept = p0 + lane >= g.m || position_kept(g, mask_in, mask_out, p0 + lane);
    for (; p0 < g.m; p0 += step) {
        const uint64_t drop = __ballot(!kept);
        const int nd = __popcll(drop);
        if (!kept) dropped[__popcll(drop & ((1ull << lane) - 1ull))] = (int32_t)(p0 + lane); // in position order
        // (same wave wrote and reads the list: program order suffices)
        const int64_t pn = p0 + step + lane;
        kept = pn >= g.m || position_kept(g, mask_in, mask_out, pn);
        const int total = nd * chunks_per_row;
        for (int c = lane; c < total; c += 64) {
            const int rk = c / chunks_per_row, pc = c - rk * chunks_per_row;
            __builtin_nontemporal_store(zero4, o4 + (int64_t)dropped[rk] * chunks_per_row + pc);
        }
    }
}

__global__ __launch_bounds__(256) void k_zero_fill_bytes(Geom g, const uint8_t *__restrict__ mask_in,
                                                         const uint8_t *__restrict__ mask_out,
                                                         uint8_t *__restrict__ out, int row_bytes)
{
    const int64_t total = (int64_t)g.m * row_bytes;
    for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < total;
         c += (int64_t)gridDim.x * blockDim.x) {
        const int64_t p = c / row_bytes;
        if (!position_kept(g, mask_in, mask_out, p)) out[c] = 0;
    }
}

hipError_t launch_zero_fill(const Geom &g, const uint8_t *mask_in, const uint8_t *mask_out, void *out,
                            int out_dtype, hipStream_t s)
{
    const int esz = out_dtype == FC_F32 ? 4 : (out_dtype == FC_FP8 ? 1 : 2);
    const int row_bytes = g.c_out * esz;
    if (row_bytes % 16 == 0) {
        const int cpr = row_bytes / 16;
        const int64_t groups = ((int64_t)g.m + 255) / 256; // 64 positions per wave, 4 waves per workgroup
        const int blocks = (int)(groups > 4096 ? 4096 : groups);
        hipLaunchKernelGGL(k_zero_fill16, dim3(blocks), dim3(256), 0, s, g, mask_in, mask_out, (uint4 *)out, cpr);
    } else {
        int64_t total = (int64_t)g.m * row_bytes;
        int blocks = (int)((total + 255) / 256 > 16384 ? 16384 : (total + 255) / 256);
        hipLaunchKernelGGL(k_zero_fill_bytes, dim3(blocks), dim3(256), 0, s, g, mask_in, mask_out, (uint8_t *)out,
                           row_bytes);
    }
    return hipGetLastError();
}

// Small fill kernel (a kernel rather than a memset node, so that callers can record it
// into HIP graphs).
__global__ __launch_bounds__(256) void k_zero_i32(int32_t *__restrict__ p, int n)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}

hipError_t launch_zero_i32(int32_t *p, int n, hipStream_t s)
{
    hipLaunchKernelGGL(k_zero_i32, dim3((n + 255) / 256), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Max-pool helper (NHWC, whole tensor).  Padding never wins.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_maxpool(const T *__restrict__ x, int n, int h, int w, int c, int k,
                                                 int stride, int pad, int ho, int wo,
                                                 const uint8_t *__restrict__ keep, T *__restrict__ out)
{
    const int64_t total = (int64_t)n * ho * wo * c;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        int ch = (int)(i % c);
        int64_t t = i / c;
        int ow = (int)(t % wo);
        t /= wo;
        int oh = (int)(t % ho);
        int b = (int)(t / ho);
        if (keep && !keep[((int64_t)b * ho + oh) * wo + ow]) {
            // a position the mask drops: no feature is computed for it (Sec. III-A); its window is not read
            T zero;
            __builtin_memset(&zero, 0, sizeof(T));
            out[i] = zero;
            continue;
        }
        bool have = false;
        float best = 0.f;
        T best_raw = x[0];
        for (int a = 0; a < k; ++a) {
            int ih = oh * stride - pad + a;
            if (ih < 0 || ih >= h) continue;
            for (int q = 0; q < k; ++q) {
                int iw = ow * stride - pad + q;
                if (iw < 0 || iw >= w) continue;
                T raw = x[(((int64_t)b * h + ih) * w + iw) * c + ch];
                float v = to_float(raw);
                if (!have || v > best) {
                    best = v;
                    best_raw = raw;
                    have = true;
                }
            }
        }
        out[i] = best_raw;
    }
}

// 16-bit types, channel count a multiple of 8: one lane owns 8 consecutive channels of an
// output position (16-byte loads and one 16-byte store).  IDX: the type the flat index is split
// in (32 bits whenever the tensor allows: the three divisions are most of the arithmetic).
template <typename T, typename IDX>
__global__ __launch_bounds__(256) void k_maxpool_x8(const T *__restrict__ x, int n, int h, int w, int c, int k,
                                                    int stride, int pad, int ho, int wo,
                                                    const uint8_t *__restrict__ keep, T *__restrict__ out)
{
    const int cg = c / 8;
    const int64_t total = (int64_t)n * ho * wo * cg;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        IDX t = (IDX)i / (IDX)cg;
        const int g8 = (int)((IDX)i - t * (IDX)cg);
        const IDX pos = t; // (b * ho + oh) * wo + ow
        const IDX t2 = t / (IDX)wo;
        const int ow = (int)(t - t2 * (IDX)wo);
        const int b = (int)(t2 / (IDX)ho);
        const int oh = (int)(t2 - (IDX)b * (IDX)ho);
        if (keep && !keep[pos]) {
            *reinterpret_cast<uint4 *>(out + i * 8) = make_uint4(0, 0, 0, 0);
            continue;
        }
        bool have = false;
        float best[8];
        uint16_t raw[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            best[e] = 0.f;
            raw[e] = 0;
        }
        for (int a = 0; a < k; ++a) {
            const int ih = oh * stride - pad + a;
            if (ih < 0 || ih >= h) continue;
            for (int q = 0; q < k; ++q) {
                const int iw = ow * stride - pad + q;
                if (iw < 0 || iw >= w) continue;
                const uint4 v = *reinterpret_cast<const uint4 *>(x + (((int64_t)b * h + ih) * w + iw) * c + g8 * 8);
                const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    T one;
                    one.bits = (uint16_t)(wd[e >> 1] >> (16 * (e & 1)));
                    const float f = to_float(one);
                    if (!have || f > best[e]) {
                        best[e] = f;
                        raw[e] = one.bits;
                    }
                }
                have = true;
            }
        }
        uint4 o;
        o.x = raw[0] | ((uint32_t)raw[1] << 16);
        o.y = raw[2] | ((uint32_t)raw[3] << 16);
        o.z = raw[4] | ((uint32_t)raw[5] << 16);
        o.w = raw[6] | ((uint32_t)raw[7] << 16);
        *reinterpret_cast<uint4 *>(out + i * 8) = o;
    }
}

// Grouped weights [c_out][taps][c_in / groups] written as the block-diagonal weights
// [c_out][taps][c_in] of the full layer that computes the same thing (zeros outside the
// blocks); esize = bytes per value.  One thread per output value.
__global__ __launch_bounds__(256) void k_expand_group_weights(const uint8_t *__restrict__ wg, int c_in, int c_out,
                                                              int taps, int groups, int esize,
                                                              uint8_t *__restrict__ wd)
{
    const int cig = c_in / groups, cog = c_out / groups;
    const int64_t total = (int64_t)c_out * taps * c_in;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int ci = (int)(i % c_in);
        const int64_t ct = i / c_in; // co * taps + tap
        const int co = (int)(ct / taps);
        const int grp = co / cog;
        const int cl = ci - grp * cig;
        const bool inside = cl >= 0 && cl < cig;
        for (int b = 0; b < esize; ++b) wd[i * esize + b] = inside ? wg[(ct * cig + cl) * esize + b] : (uint8_t)0;
    }
}

hipError_t launch_expand_group_weights(const void *wg, int c_in, int c_out, int taps, int groups, int esize,
                                       void *wd, hipStream_t s)
{
    const int64_t total = (int64_t)c_out * taps * c_in;
    const int blocks = (int)((total + 255) / 256 > 65536 ? 65536 : (total + 255) / 256);
    hipLaunchKernelGGL(k_expand_group_weights, dim3(blocks), dim3(256), 0, s, (const uint8_t *)wg, c_in, c_out, taps,
                       groups, esize, (uint8_t *)wd);
    return hipGetLastError();
}

hipError_t launch_maxpool(const void *x, int n, int h, int w, int c, int dtype, int k, int stride, int pad,
                          int ho, int wo, const uint8_t *keep, void *out, hipStream_t s)
{
    if (dtype != FC_F32 && c % 8 == 0) {
        const int64_t total8 = (int64_t)n * ho * wo * (c / 8);
        const int blocks8 = (int)((total8 + 255) / 256 > 65536 ? 65536 : (total8 + 255) / 256);
        const bool small = total8 < (int64_t)INT32_MAX;
        if (dtype == FC_BF16) {
            if (small)
                hipLaunchKernelGGL((k_maxpool_x8<bf16_t, uint32_t>), dim3(blocks8), dim3(256), 0, s, (const bf16_t *)x, n,
                                   h, w, c, k, stride, pad, ho, wo, keep, (bf16_t *)out);
            else
                hipLaunchKernelGGL((k_maxpool_x8<bf16_t, int64_t>), dim3(blocks8), dim3(256), 0, s, (const bf16_t *)x, n,
                                   h, w, c, k, stride, pad, ho, wo, keep, (bf16_t *)out);
        } else {
            if (small)
                hipLaunchKernelGGL((k_maxpool_x8<f16_t, uint32_t>), dim3(blocks8), dim3(256), 0, s, (const f16_t *)x, n, h,
                                   w, c, k, stride, pad, ho, wo, keep, (f16_t *)out);
            else
                hipLaunchKernelGGL((k_maxpool_x8<f16_t, int64_t>), dim3(blocks8), dim3(256), 0, s, (const f16_t *)x, n, h,
                                   w, c, k, stride, pad, ho, wo, keep, (f16_t *)out);
        }
        return hipGetLastError();
    }
    const int64_t total = (int64_t)n * ho * wo * c;
    int blocks = (int)((total + 255) / 256 > 65536 ? 65536 : (total + 255) / 256);
    if (dtype == FC_F32)
        hipLaunchKernelGGL(k_maxpool<float>, dim3(blocks), dim3(256), 0, s, (const float *)x, n, h, w, c, k, stride,
                           pad, ho, wo, keep, (float *)out);
    else if (dtype == FC_BF16)
        hipLaunchKernelGGL(k_maxpool<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t *)x, n, h, w, c, k,
                           stride, pad, ho, wo, keep, (bf16_t *)out);
    else
        hipLaunchKernelGGL(k_maxpool<f16_t>, dim3(blocks), dim3(256), 0, s, (const f16_t *)x, n, h, w, c, k, stride,
                           pad, ho, wo, keep, (f16_t *)out);
    return hipGetLastError();
}

} // namespace fc
