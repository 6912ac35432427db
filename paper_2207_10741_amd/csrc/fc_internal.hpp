// Internal declarations shared by the library's translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "focused_conv.h"

namespace fc {

// Geometry handed to every kernel (plain ints, passed by value).
struct Geom {
    int32_t n, h, w, c_in, c_out, kh, kw;
    int32_t sh, sw, ph, pw, dh, dw;
    int32_t ho, wo;
    int32_t m;        // n*ho*wo
    uint32_t flags;
};

// 16-bit storage types are carried as raw bit patterns.
struct bf16_t { uint16_t bits; };
struct f16_t { uint16_t bits; };

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }
__device__ __forceinline__ float to_float(f16_t v)
{
    _Float16 h;
    __builtin_memcpy(&h, &v.bits, 2);
    return (float)h;
}

// float -> storage, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint16_t bf16_bits_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ uint16_t f16_bits_rne(float f)
{
    _Float16 h = (_Float16)f;
    uint16_t b;
    __builtin_memcpy(&b, &h, 2);
    return b;
}
__device__ __forceinline__ void from_float(float f, float *o) { *o = f; }
__device__ __forceinline__ void from_float(float f, bf16_t *o) { o->bits = bf16_bits_rne(f); }
__device__ __forceinline__ void from_float(float f, f16_t *o) { o->bits = f16_bits_rne(f); }

// n / d for n < 2^31 as a multiply and a shift: s = ceil(log2 d), m = ceil(2^(31+s) / d);
// m*d = 2^(31+s) + e with e < d <= 2^s, so the estimate is off by less than 1/d.
struct FastDiv {
    uint32_t m, s;
};

static inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.s = 0;
    while ((1ull << f.s) < d) ++f.s;
    f.m = (uint32_t)(((1ull << (31 + f.s)) + d - 1) / d);
    return f;
}

__device__ __forceinline__ uint32_t fast_div(uint32_t n, FastDiv f)
{
    return (uint32_t)(((uint64_t)n * f.m) >> (31 + f.s));
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int kCompactBlockThreads = 256;
constexpr int kCompactBytesPerThread = 16;
constexpr int kCompactBlockElems = kCompactBlockThreads * kCompactBytesPerThread; // 4096

constexpr int kCompactSingleLaunchBlocks = 16; // up to this many blocks the compaction is one launch

static inline int64_t compact_blocks(int64_t m) { return (m + kCompactBlockElems - 1) / kCompactBlockElems; }

// How output positions map to input-mask pixels (centre tap of the receptive field).
struct MaskGeom {
    int32_t n, h, w, ho, wo, sh, sw, ch0, cw0;
    int32_t identity; // output position p reads input pixel p (stride 1, same size, centred)
    int32_t packed_in, packed_out; // the mask read / written is one bit per pixel (see mask_at)
    int64_t m;        // n*ho*wo
};

// A mask is one byte per pixel (nonzero = relevant) or, packed, one bit per pixel: bit p & 31
// of the 32-bit word p >> 5 (little-endian, so the same bits as bit p & 63 of the 64-bit word
// p >> 6, one wave ballot); bits past the last pixel are zero.
__device__ __forceinline__ bool mask_at(const uint8_t *__restrict__ m, int64_t p, bool packed)
{
    if (packed) return (reinterpret_cast<const uint32_t *>(m)[p >> 5] >> (uint32_t)(p & 31)) & 1u;
    return m[p] != 0;
}

__host__ __device__ static inline MaskGeom mask_geom(int n, int h, int w, int kh, int kw, int sh, int sw, int ph, int pw, int dh,
                                 int dw, int ho, int wo)
{
    MaskGeom g;
    g.n = n; g.h = h; g.w = w; g.ho = ho; g.wo = wo; g.sh = sh; g.sw = sw;
    g.ch0 = -ph + dh * ((kh - 1) / 2);
    g.cw0 = -pw + dw * ((kw - 1) / 2);
    g.identity = (sh == 1 && sw == 1 && ho == h && wo == w && g.ch0 == 0 && g.cw0 == 0) ? 1 : 0;
    g.packed_in = g.packed_out = 0;
    g.m = (int64_t)n * ho * wo;
    return g;
}

// bit j = output position p0 + j is kept (positions at or past g.m read as 0)
__device__ __forceinline__ uint32_t kept_flags16(const MaskGeom &g, const uint8_t *__restrict__ mask_in,
                                                 int64_t p0)
{
    uint32_t flags = 0;
    if (p0 >= g.m) return 0;
    if (g.identity && g.packed_in) {
        // p0 is a multiple of 16: the labels are one 16-bit piece of the packed mask
        flags = reinterpret_cast<const uint16_t *>(mask_in)[p0 >> 4];
        if (p0 + 16 > g.m) flags &= (1u << (uint32_t)(g.m - p0)) - 1u;
        return flags;
    }
    if (g.identity && p0 + 16 <= g.m) {
        const uint4 v = *reinterpret_cast<const uint4 *>(mask_in + p0);
        const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                flags |= ((wds[q] >> (8 * b)) & 0xffu) ? (1u << (4 * q + b)) : 0u;
        return flags;
    }
    // (positions fit 31 bits: 32-bit divisions; addresses first, then all sixteen bytes in
    // flight together)
    const uint32_t t = (uint32_t)p0 / (uint32_t)g.wo;
    int ow = (int)((uint32_t)p0 - t * (uint32_t)g.wo);
    int b = (int)(t / (uint32_t)g.ho);
    int oh = (int)(t - (uint32_t)b * (uint32_t)g.ho);
    int row_at = (b * g.h + min(max(oh * g.sh + g.ch0, 0), g.h - 1)) * g.w;
    int at[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        at[j] = p0 + j < g.m ? row_at + min(max(ow * g.sw + g.cw0, 0), g.w - 1) : -1;
        if (++ow == g.wo) {
            ow = 0;
            if (++oh == g.ho) {
                oh = 0;
                ++b;
            }
            row_at = (b * g.h + min(max(oh * g.sh + g.ch0, 0), g.h - 1)) * g.w;
        }
    }
    if (g.packed_in) {
        uint32_t got[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) got[j] = at[j] >= 0 ? reinterpret_cast<const uint32_t *>(mask_in)[at[j] >> 5] : 0u;
#pragma unroll
        for (int j = 0; j < 16; ++j) flags |= ((got[j] >> (at[j] & 31)) & 1u) << j;
        return flags;
    }
    uint8_t got[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) got[j] = at[j] >= 0 ? mask_in[at[j]] : (uint8_t)0;
#pragma unroll
    for (int j = 0; j < 16; ++j) flags |= got[j] ? (1u << j) : 0u;
    return flags;
}

// inclusive prefix sum over the 64 lanes of a wave, on the cross-lane data path of the
// vector ALU (no LDS traffic): shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last
// lane of row 0 / row 2 is broadcast into row 1 / row 3, then lane 31 into rows 2 and 3.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    // row_shr:n = 0x110 + n (a lane with no source inside its row adds 0)
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);
    // row_bcast:15 into rows 1 and 3 (row mask 0b1010), row_bcast:31 into rows 2 and 3 (0b1100)
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);
    return v;
}

// ---- launchers (each enqueues on `s`, returns a hipError_t) ----------------
hipError_t launch_mask_downsample(const uint8_t *mask_in, int n, int h, int w, int kh, int kw,
                                  int sh, int sw, int ph, int pw, int dh, int dw, int ho, int wo,
                                  uint8_t *mask_out, hipStream_t s);
// Patch labels by a window rule: any pixel of the window relevant, or all of them.
hipError_t launch_mask_window(const uint8_t *mask_in, int n, int h, int w, int kh, int kw, int sh, int sw,
                              int ph, int pw, int dh, int dw, int ho, int wo, bool all, uint8_t *mask_out,
                              hipStream_t s);
// What the compaction can do on the side for the convolution that follows it.
struct CompactExtras {
    int32_t *zero = nullptr; // zero_n ints to clear (the split-K tile counters)
    int32_t zero_n = 0;
};

// Kept positions of the layer whose mask geometry is g: writes mask_out (0/1 bytes;
// may be NULL), the ascending index list and its length.
hipError_t launch_compact(const MaskGeom &g, const uint8_t *mask_in, uint8_t *mask_out, int32_t *idx,
                          int32_t *count, int32_t *block_counts, const CompactExtras &extras, hipStream_t s);
// Mask pyramid: level l (1-based here; index 0 of h/w is the input mask) is the centre-tap
// rescaling of level l - 1 with vertical/horizontal step sh/sw and first-tap offset ch0/cw0.
constexpr int kMaxPyramidLevels = 8;
struct PyramidArgs {
    int32_t levels, n;
    int32_t packed_in, packed_out; // the input mask / the levels' masks are one bit per pixel
    int32_t identity0; // level 0 has the input's resolution, centred window, and the input is 16-byte aligned
    int32_t h[kMaxPyramidLevels + 1], w[kMaxPyramidLevels + 1]; // [0] = input mask, [l + 1] = level l
    int32_t sh[kMaxPyramidLevels], sw[kMaxPyramidLevels], ch0[kMaxPyramidLevels], cw0[kMaxPyramidLevels];
    int64_t m[kMaxPyramidLevels];          // positions of level l
    FastDiv div_w[kMaxPyramidLevels], div_h[kMaxPyramidLevels]; // by the level's width and height
    int32_t block0[kMaxPyramidLevels + 1]; // first block of level l; [levels] = total
    uint8_t *mask_out[kMaxPyramidLevels];
    int32_t *idx[kMaxPyramidLevels];
    int32_t *count[kMaxPyramidLevels];
};
// kept positions of a [n][ho][wo] mask in tile order; block_counts: one int per 256 tile rows
hipError_t launch_compact_tiled(const uint8_t *mask, int n, int ho, int wo, int tile_h, int tile_w, int32_t *idx,
                                int32_t *count, int32_t *block_counts, hipStream_t s);
constexpr int kMaxListTileWidth = 32; // a tile row's labels are one 32-bit word
static inline int64_t tiled_rows(int n, int ho, int wo, int tile_h, int tile_w)
{
    return (int64_t)n * ((ho + tile_h - 1) / tile_h) * ((wo + tile_w - 1) / tile_w) * tile_h;
}
hipError_t launch_mask_pyramid(const PyramidArgs &a, const uint8_t *mask_in, int32_t *block_counts, hipStream_t s);
// bytes -> bits (nonzero byte = 1; the bits of the last word past m are zero), and the
// centre-tap rescaling of a mask in either form into either form
hipError_t launch_mask_pack(const uint8_t *mask, int64_t m, uint64_t *bits, hipStream_t s);
hipError_t launch_mask_rescale(const MaskGeom &g, const uint8_t *mask_in, uint8_t *mask_out, hipStream_t s);
hipError_t launch_zero_fill(const Geom &g, const uint8_t *mask_in, const uint8_t *mask_out, void *out,
                            int out_dtype, hipStream_t s);
hipError_t launch_expand_group_weights(const void *wg, int c_in, int c_out, int taps, int groups, int esize,
                                       void *wd, hipStream_t s);
// keep: [n][ho][wo] bytes or NULL; positions with a zero byte are written as +0 and not computed
hipError_t launch_maxpool(const void *x, int n, int h, int w, int c, int dtype, int k, int stride,
                          int pad, int ho, int wo, const uint8_t *keep, void *out, hipStream_t s);

// Direct convolution over the active rows; any shape, any dtype.  groups > 1: g.c_in / g.c_out
// are the channels of one group, x and out hold all groups side by side.
hipError_t launch_conv_direct(const Geom &g, int in_dtype, int out_dtype, const void *x,
                              const uint8_t *mask_in, const void *w, const float *bias,
                              const int32_t *idx, const int32_t *count, void *out, hipStream_t s, int groups = 1);

// Depthwise layer (one filter per channel); labels positions from mask_in itself and clears
// the irrelevant rows.
bool conv_depthwise_supported(const Geom &g, int in_dtype);
hipError_t launch_conv_depthwise(const Geom &g, int in_dtype, int out_dtype, const void *x, const uint8_t *mask_in,
                                 const void *w, const float *bias, void *out, hipStream_t s);

// Matrix-core path for layers with at most 4 input channels (RGB stems); the caller clears the
// irrelevant rows with launch_zero_fill.
bool conv_stem_supported(const Geom &g, int in_dtype, int out_dtype);
hipError_t launch_conv_stem(const Geom &g, int in_dtype, int out_dtype, const void *x, const uint8_t *mask_in,
                            const void *w, const float *bias, const int32_t *idx, const int32_t *count,
                            void *out, hipStream_t s);

// Split-K scratch of the matrix-core path (optional): fp32 partial tiles and one counter
// per tile.  Only layers with few tiles use it; for the others the sizes are zero.
constexpr int kInlineRankPositions = 4096;                  // layers up to this many positions rank their kept rows in the conv kernel (16 per thread of a 256-thread workgroup)
constexpr int kSplitGrid = 512;                          // workgroups launched when split-K may run
constexpr size_t kSplitTileFloats = 128 * 128;           // largest tile
static inline bool split_k_possible(const Geom &g)
{
    const int64_t tiles64 = (int64_t)((g.m + 127) / 128) * ((g.c_out + 63) / 64);
    return tiles64 < kSplitGrid; // fewer tiles than workgroups even for the dense row count
}
static inline size_t split_k_counter_bytes(const Geom &g) { return split_k_possible(g) ? align_up(kSplitGrid * sizeof(int32_t), 256) : 0; }
static inline size_t split_k_partial_bytes(const Geom &g)
{
    return split_k_possible(g) ? (size_t)kSplitGrid * kSplitTileFloats * sizeof(float) : 0;
}
hipError_t launch_zero_i32(int32_t *p, int n, hipStream_t s);

// Matrix-core path (only for shapes conv_mfma_supported accepts).  It also clears
// the irrelevant output rows unless FC_SKIP_ZERO_FILL is set; mask_out may be NULL.
bool conv_mfma_supported(const Geom &g, int in_dtype, int out_dtype);
hipError_t launch_conv_mfma(const Geom &g, int in_dtype, int out_dtype, const void *x,
                            const uint8_t *mask_in, const uint8_t *mask_out, const void *w,
                            const float *bias, const int32_t *idx, const int32_t *count, void *out,
                            float *partials, int32_t *tile_counters, hipStream_t s);

// Calibration launches (see fc_calibrate.hip): `blocks` workgroups of four waves each run
// `iters` rounds of eight matrix instructions; a streaming copy of `bytes` bytes.
hipError_t launch_calibrate_mfma(int dtype, int iters, int blocks, float *sink, hipStream_t s);
hipError_t launch_calibrate_copy(const void *src, void *dst, size_t bytes, hipStream_t s);
// `steps` steps of two matrix instructions plus item `mode` per wave, 1, 2 or 4 waves per SIMD;
// cycles[block] = shader cycles of the loop.
hipError_t launch_calibrate_issue(int mode, int waves_per_simd, int steps, int blocks, const void *src,
                                  long long *cycles, float *sink, hipStream_t s);

// One-workgroup-per-CU matrix-core path for 3x3 layers (see fc_conv_line.hip): 128 output
// channels per tile.  Needs the kept list (or no mask at all).
bool conv_line_supported(const Geom &g, int in_dtype, int out_dtype);
hipError_t launch_conv_line(const Geom &g, int in_dtype, int out_dtype, const void *x,
                            const uint8_t *mask_in, const uint8_t *mask_out, const void *w, const float *bias,
                            const int32_t *idx, const int32_t *count, void *out, hipStream_t s);

// Resident-weights matrix-core path (see fc_conv_pw.hip): 1x1 layers without padding whose rows
// are whole 16-byte pieces and whose weights, cut into slices of output channels, stay in LDS,
// and 3x3 layers whose pixels are 128 bytes (bf16, f16 or E4M3 storage).  Needs the kept list
// (or no mask at all).
bool conv_pw_supported(const Geom &g, int in_dtype, int out_dtype);
hipError_t launch_conv_pw(const Geom &g, int in_dtype, int out_dtype, const void *x, const uint8_t *mask_in,
                          const uint8_t *mask_out, const void *w, const float *bias, const int32_t *idx,
                          const int32_t *count, void *out, hipStream_t s);

} // namespace fc
