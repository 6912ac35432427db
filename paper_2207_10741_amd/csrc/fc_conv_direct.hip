// Direct focused convolution for shapes the matrix-core path does not take
// (odd channel counts such as RGB stems, fp32 storage, very large kernels).
// Sec. III-A: only the kept patches are evaluated.
//
// One lane owns one kept position and CO_T of its output channels, held as fp32
// accumulators in registers; it walks the taps in the order kh, kw, ci.  The
// weights of those CO_T channels are staged once per workgroup in LDS as fp32,
// transposed to [k][channel], so that the inner loop reads them as broadcasts
// (every lane the same address) and does CO_T fused multiply-adds per loaded input
// value.  Lanes of a wave hold consecutive kept positions, so for an RGB stem their
// input loads fall on neighbouring pixels.  A gated tap (padding, irrelevant input
// pixel) is skipped, not multiplied.
#include "fc_internal.hpp"

namespace fc {

constexpr int kRowsThreads = 256;
constexpr int kRowsLdsFloats = 12288; // 48 KB of staged weights per workgroup

template <typename TI, typename TO, int CO_T>
__global__ __launch_bounds__(kRowsThreads) void k_conv_rows(Geom g, const TI *__restrict__ x,
                                                            const uint8_t *__restrict__ mask_in,
                                                            const TI *__restrict__ w,
                                                            const float *__restrict__ bias,
                                                            const int32_t *__restrict__ idx,
                                                            const int32_t *__restrict__ count,
                                                            TO *__restrict__ out, int groups)
{
    // Grouped layers: g.c_in and g.c_out are the channels of ONE group, blockIdx.z is the group;
    // a pixel of x holds groups * g.c_in channels and a row of out groups * g.c_out, group by
    // group; w is [groups * g.c_out][kh][kw][g.c_in].  groups = 1 is the plain layer.
    const int grp = blockIdx.z;
    const int x_pitch = groups * g.c_in, out_pitch = groups * g.c_out;
    x += grp * g.c_in;
    w += (int64_t)grp * g.c_out * (g.kh * g.kw * g.c_in);
    if (bias) bias += grp * g.c_out;
    out += grp * g.c_out;
    constexpr int KC = kRowsLdsFloats / CO_T; // reduction elements staged at a time
    __shared__ float wt[KC * CO_T];           // [k][channel]
    const int tid = threadIdx.x;
    const int rows = idx ? *count : g.m;
    const int K = g.kh * g.kw * g.c_in;
    const int co0 = blockIdx.y * CO_T;
    const int nchunks = (K + KC - 1) / KC;
    bool staged = false; // with a single chunk the weights are staged once for all row blocks

    for (int r0 = blockIdx.x * kRowsThreads; r0 < rows; r0 += gridDim.x * kRowsThreads) {
        const int r = r0 + tid;
        const bool live = r < rows;
        int p = 0, ih0 = 0, iw0 = 0, b = 0;
        if (live) {
            p = idx ? idx[r] : r;
            const int ow = p % g.wo;
            const int q = p / g.wo;
            const int oh = q % g.ho;
            b = q / g.ho;
            ih0 = oh * g.sh - g.ph;
            iw0 = ow * g.sw - g.pw;
        }
        float acc[CO_T];
#pragma unroll
        for (int j = 0; j < CO_T; ++j) acc[j] = 0.f;

        // cursor over the reduction index k = (kh, kw, ci), carried across chunks
        int kh = 0, kw = 0, ci = 0;
        bool tap_ok = false;
        const TI *xp = x;
        bool new_tap = true;
        for (int c = 0; c < nchunks; ++c) {
            const int k0 = c * KC;
            const int kc = K - k0 < KC ? K - k0 : KC;
            if (!staged) {
                __syncthreads(); // the previous chunk has been consumed
                for (int i = tid; i < CO_T * kc; i += kRowsThreads) {
                    const int j = i / kc, k = i - j * kc; // k fastest: contiguous global reads
                    const int co = co0 + j;
                    wt[k * CO_T + j] = co < g.c_out ? to_float(w[(int64_t)co * K + k0 + k]) : 0.f;
                }
                __syncthreads();
                staged = nchunks == 1;
            }
            // four input channels at a time where the layout allows (channel count a multiple of
            // four: a group of four never straddles a tap or a staged chunk), so that a lane has one
            // 16-byte (fp32) or 8-byte (16-bit types) load in flight per 4 x CO_T multiply-adds
            // instead of four dependent narrow loads
            const bool by4 = g.c_in % 4 == 0;
            for (int k = 0; k < kc; k += by4 ? 4 : 1) {
                if (new_tap) {
                    const int ih = ih0 + kh * g.dh, iw = iw0 + kw * g.dw;
                    tap_ok = live && ih >= 0 && ih < g.h && iw >= 0 && iw < g.w;
                    if (tap_ok) {
                        const int64_t pix = ((int64_t)b * g.h + ih) * g.w + iw;
                        tap_ok = !mask_in || mask_at(mask_in, pix, (g.flags & FC_PACKED_MASKS) != 0);
                        xp = x + pix * x_pitch;
                    }
                    new_tap = false;
                }
                if (tap_ok) {
                    if (by4) {
                        float xs[4];
                        if constexpr (sizeof(TI) == 4) {
                            const float4 xq = *reinterpret_cast<const float4 *>(xp + ci);
                            xs[0] = xq.x; xs[1] = xq.y; xs[2] = xq.z; xs[3] = xq.w;
                        } else {
                            const uint2 xq = *reinterpret_cast<const uint2 *>(xp + ci);
                            TI t;
                            t.bits = (uint16_t)(xq.x & 0xffffu); xs[0] = to_float(t);
                            t.bits = (uint16_t)(xq.x >> 16);     xs[1] = to_float(t);
                            t.bits = (uint16_t)(xq.y & 0xffffu); xs[2] = to_float(t);
                            t.bits = (uint16_t)(xq.y >> 16);     xs[3] = to_float(t);
                        }
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float *wk = wt + (k + e) * CO_T;
#pragma unroll
                            for (int j = 0; j < CO_T; ++j) acc[j] = fmaf(xs[e], wk[j], acc[j]);
                        }
                    } else {
                        const float xv = to_float(xp[ci]);
                        const float *wk = wt + k * CO_T;
#pragma unroll
                        for (int j = 0; j < CO_T; ++j) acc[j] = fmaf(xv, wk[j], acc[j]);
                    }
                }
                ci += by4 ? 3 : 0;
                if (++ci == g.c_in) {
                    ci = 0;
                    new_tap = true;
                    if (++kw == g.kw) {
                        kw = 0;
                        ++kh;
                    }
                }
            }
        }
        if (live) {
            TO *orow = out + (int64_t)p * out_pitch + co0;
            // elements per store: 16 bytes' worth, or the whole (narrow) channel block
            constexpr int EPV = 16 / (int)sizeof(TO) < CO_T ? 16 / (int)sizeof(TO) : CO_T;
            constexpr int PIECE_BYTES = EPV * (int)sizeof(TO);
            const bool whole_pieces = g.c_out % EPV == 0;
#pragma unroll
            for (int j0 = 0; j0 < CO_T; j0 += EPV) {
                if (co0 + j0 >= g.c_out) break;
                __align__(16) TO piece[EPV];
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const int co = co0 + j0 + e;
                    float v = acc[j0 + e] + ((bias && co < g.c_out) ? bias[co] : 0.f);
                    if ((g.flags & FC_RELU) && !(v > 0.f)) v = (v != v) ? v : 0.f;
                    from_float(v, &piece[e]);
                }
                if (whole_pieces) {
                    if constexpr (PIECE_BYTES == 16)
                        *reinterpret_cast<uint4 *>(orow + j0) = *reinterpret_cast<const uint4 *>(piece);
                    else if constexpr (PIECE_BYTES == 8)
                        *reinterpret_cast<uint2 *>(orow + j0) = *reinterpret_cast<const uint2 *>(piece);
                    else
                        *reinterpret_cast<uint32_t *>(orow + j0) = *reinterpret_cast<const uint32_t *>(piece);
                } else {
#pragma unroll
                    for (int e = 0; e < EPV; ++e)
                        if (co0 + j0 + e < g.c_out) orow[j0 + e] = piece[e];
                }
            }
        }
    }
}

template <typename TI, typename TO, int CO_T>
static hipError_t launch_rows(const Geom &g, const void *x, const uint8_t *mask_in, const void *w,
                              const float *bias, const int32_t *idx, const int32_t *count, void *out,
                              int groups, hipStream_t s)
{
    // grid sized for the dense row count: the kept count is only known on the device
    const int64_t row_blocks = ((int64_t)g.m + kRowsThreads - 1) / kRowsThreads;
    const int gx = (int)(row_blocks > 8192 ? 8192 : row_blocks);
    const int gy = (g.c_out + CO_T - 1) / CO_T;
    hipLaunchKernelGGL((k_conv_rows<TI, TO, CO_T>), dim3(gx, gy, groups), dim3(kRowsThreads), 0, s, g, (const TI *)x,
                       mask_in, (const TI *)w, bias, idx, count, (TO *)out, groups);
    return hipGetLastError();
}

template <typename TI, typename TO>
static hipError_t launch_t(const Geom &g, const void *x, const uint8_t *mask_in, const void *w,
                           const float *bias, const int32_t *idx, const int32_t *count, void *out,
                           int groups, hipStream_t s)
{
    // wide accumulator blocks when the layer is wide enough to use them and has enough rows to
    // fill the chip with them; a small layer is cut into narrow channel blocks instead (more
    // workgroups, a four times shorter serial loop per lane; the input is re-read per block,
    // which a small layer can afford)
    const int64_t wide_blocks = (((int64_t)g.m + kRowsThreads - 1) / kRowsThreads) * ((g.c_out + 63) / 64) * groups;
    if (g.c_out > 32 && wide_blocks >= 512) return launch_rows<TI, TO, 64>(g, x, mask_in, w, bias, idx, count, out, groups, s);
    // few output channels (per group): accumulator blocks no wider than the layer
    if (g.c_out <= 4) return launch_rows<TI, TO, 4>(g, x, mask_in, w, bias, idx, count, out, groups, s);
    if (g.c_out <= 8) return launch_rows<TI, TO, 8>(g, x, mask_in, w, bias, idx, count, out, groups, s);
    return launch_rows<TI, TO, 16>(g, x, mask_in, w, bias, idx, count, out, groups, s);
}

hipError_t launch_conv_direct(const Geom &g, int in_dtype, int out_dtype, const void *x,
                              const uint8_t *mask_in, const void *w, const float *bias, const int32_t *idx,
                              const int32_t *count, void *out, hipStream_t s, int groups)
{
    if (in_dtype == FC_F32) return launch_t<float, float>(g, x, mask_in, w, bias, idx, count, out, groups, s);
    if (in_dtype == FC_BF16) {
        if (out_dtype == FC_F32) return launch_t<bf16_t, float>(g, x, mask_in, w, bias, idx, count, out, groups, s);
        return launch_t<bf16_t, bf16_t>(g, x, mask_in, w, bias, idx, count, out, groups, s);
    }
    if (out_dtype == FC_F32) return launch_t<f16_t, float>(g, x, mask_in, w, bias, idx, count, out, groups, s);
    return launch_t<f16_t, f16_t>(g, x, mask_in, w, bias, idx, count, out, groups, s);
}

} // namespace fc
