// Depthwise focused convolution: channel c of the output sees channel c of the input only,
// through its own KH x KW filter (the layer type most of the networks of Sec. IV consist of).
// Sec. III-A unchanged otherwise: a position whose centre-tap mask byte is zero gets no
// features (+0.0 in every channel), a kept position sees zero at irrelevant input pixels and
// outside the image, weights and bias are the dense layer's.
//
// There is no contraction here (KH*KW multiply-adds per output value, 2 bytes in and 2 bytes
// out), so the kernel is bound by memory traffic and vector ALU work, not by the matrix cores.
//
// Mapping.  A lane owns VEC consecutive channels (16 bytes of a pixel) for the whole launch.
// The lanes of a workgroup are laid out [position][channel chunk]: consecutive lanes read and
// write consecutive 16-byte pieces of a pixel, then the next pixel, and the workgroup walks the
// positions of one image with a grid stride.  Pixels are not staged in LDS; taps shared by
// neighbouring positions are served by the caches.  The filters and the bias of a lane's
// channels live in its registers, or, for 3 x 3 layers whose filters are small enough, in LDS
// (which halves the register count and doubles the waves in flight).
//
// Gating without branches.  The image and its mask are addressed through buffer descriptors
// that cover exactly one image: a tap outside the image or at an irrelevant pixel is given an
// out-of-range offset, for which the hardware returns zero and touches no memory, so NaN at an
// irrelevant pixel is never loaded.  The mask bytes of all taps are requested first, then the
// pixels of the taps that survive, then the arithmetic (fp32 sums over the taps in the order
// kh, kw, two taps at a time for 16-bit 3 x 3 layers; one rounding to the output type).
//
// The position's own label is read from the input mask under the centre tap (Sec. III-B), so
// no kept-position list is needed, and irrelevant positions are cleared by the lanes that
// would have computed them (unless the caller asked to leave them untouched).
#include "fc_internal.hpp"

namespace fc {

namespace {

constexpr int kDwThreads = 256;
constexpr uint32_t kDwBufferLimit = 0xF0000000u; // one image (and its mask) stays below this many bytes
constexpr uint32_t kDwOutOfRange = kDwBufferLimit;
constexpr int kDwTargetBlocks = 1024;            // four workgroups per CU

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct DwArgs {
    Geom g;
    int32_t lanes_per_pos; // channel chunks of one position handled by one workgroup
    int32_t pos_per_block; // positions a workgroup handles per step
    int32_t chunks;        // channel chunks in all: C / VEC
    FastDiv div_wo;
};

template <int BYTES>
struct RawWords {
    static constexpr int N = (BYTES + 3) / 4;
    uint32_t v[N];
};

template <int BYTES>
__device__ __forceinline__ RawWords<BYTES> buffer_load(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    RawWords<BYTES> o;
    if constexpr (BYTES == 16) {
        const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
        o.v[0] = t.x; o.v[1] = t.y; o.v[2] = t.z; o.v[3] = t.w;
    } else if constexpr (BYTES == 4) {
        o.v[0] = __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0);
    } else {
        static_assert(BYTES == 2, "16-, 4- or 2-byte pieces");
        o.v[0] = __builtin_amdgcn_raw_buffer_load_b16(r, off, 0, 0);
    }
    return o;
}

// element e of a piece of VEC values of type TI held as raw words
template <typename TI>
__device__ __forceinline__ float piece_elem(const uint32_t *words, int e)
{
    if constexpr (sizeof(TI) == 4) {
        return __uint_as_float(words[e]);
    } else {
        const uint32_t wd = words[e >> 1];
        if constexpr (__is_same(TI, bf16_t)) {
            return __uint_as_float((e & 1) ? (wd & 0xffff0000u) : (wd << 16));
        } else {
            f16_t h;
            h.bits = (uint16_t)((e & 1) ? (wd >> 16) : (wd & 0xffffu));
            return to_float(h);
        }
    }
}

// VEC values rounded once and written as 16-byte pieces where the count allows
template <typename TO, int VEC>
__device__ __forceinline__ void store_piece(TO *dst, const float *v)
{
    if constexpr (sizeof(TO) == 4) {
        if constexpr (VEC % 4 == 0) {
#pragma unroll
            for (int k = 0; k < VEC / 4; ++k)
                reinterpret_cast<float4 *>(dst)[k] = make_float4(v[4 * k], v[4 * k + 1], v[4 * k + 2], v[4 * k + 3]);
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) dst[e] = v[e];
        }
    } else {
        if constexpr (VEC == 8) {
            uint32_t wds[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                TO lo, hi;
                from_float(v[2 * k], &lo);
                from_float(v[2 * k + 1], &hi);
                wds[k] = (uint32_t)lo.bits | ((uint32_t)hi.bits << 16);
            }
            u32x4 p;
            p.x = wds[0]; p.y = wds[1]; p.z = wds[2]; p.w = wds[3];
            *reinterpret_cast<u32x4 *>(dst) = p;
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) from_float(v[e], &dst[e]);
        }
    }
}

// a.lo * b.lo + a.hi * b.hi + c for two packed 16-bit floats per operand, summed in fp32
// (v_dot2c_f32_bf16 / v_dot2c_f32_f16)
typedef __bf16 bf16x2_native __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_native __attribute__((ext_vector_type(2)));
template <typename TI>
__device__ __forceinline__ float dot2_acc(uint32_t a, uint32_t b, float c)
{
    if constexpr (__is_same(TI, bf16_t))
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_native, a),
                                               __builtin_bit_cast(bf16x2_native, b), c, false);
    else
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_native, a), __builtin_bit_cast(f16x2_native, b), c,
                                      false);
}

// 3 x 3 layers of the 16-bit types pair their taps: (0,1) (2,3) (4,5) (6,7) and tap 8 with a
// zero.  The two pixels of a pair are interleaved channel by channel (one byte permute per
// output channel) and multiplied against the packed pair of filter values by one 2-element dot
// product, instead of two unpacks and two multiply-adds; the filters take 5 words per channel
// instead of 9.
constexpr int kDwPairRows = 5;

// KS: compile-time square kernel size (filters in registers), or 0 for any KH x KW (filters
// re-read through the cache at every tap).
// WLDS: the workgroup's filters and bias sit in LDS as fp32 [tap][channel] instead of in every
// lane's registers; lanes with the same channel chunk read the same addresses.  The kernel then
// needs about 60 registers instead of 128, twice as many waves fit a SIMD, and it is the number
// of waves in flight that hides the dependent memory round trips of a position.
template <typename TI, typename TO, int VEC, int KS, bool WLDS>
__global__ __launch_bounds__(kDwThreads, (WLDS ? 8 : (KS > 3 ? 2 : 4))) void k_dwconv(DwArgs a, const TI *__restrict__ x,
                                                       const uint8_t *__restrict__ mask_in,
                                                       const TI *__restrict__ w, const float *__restrict__ bias,
                                                       TO *__restrict__ out)
{
    constexpr int PIECE = VEC * (int)sizeof(TI); // bytes of a pixel one lane owns
    constexpr int TAPS_C = KS * KS;
    constexpr bool PAIR = KS == 3 && sizeof(TI) == 2 && VEC == 8;
    constexpr int WROWS = PAIR ? kDwPairRows : TAPS_C; // filter words per channel (LDS rows before the bias)
    const Geom &g = a.g;
    const int b = blockIdx.y;
    const int j = threadIdx.x % a.lanes_per_pos;
    const int pp = threadIdx.x / a.lanes_per_pos;
    const int chunk = blockIdx.z * a.lanes_per_pos + j;
    const int C = g.c_in;
    const int kh_n = KS ? KS : g.kh, kw_n = KS ? KS : g.kw;
    const int taps = kh_n * kw_n;
    // WLDS only: [WROWS + 1][CT]: the filters (fp32 per tap, or packed pairs of taps), then the bias
    extern __shared__ __align__(16) float dw_w[];
    const int CT = a.lanes_per_pos * VEC; // channels of this workgroup
    if constexpr (WLDS) {
        const int ch_first = blockIdx.z * CT;
        for (int i = threadIdx.x; i < (WROWS + 1) * CT; i += kDwThreads) {
            const int t = i / CT, ch = ch_first + (i - t * CT);
            float v = 0.f;
            if (ch < C) {
                if (t == WROWS) {
                    v = bias ? bias[ch] : 0.f;
                } else if constexpr (PAIR) {
                    const uint32_t lo = w[(int64_t)ch * TAPS_C + 2 * t].bits;
                    const uint32_t hi = 2 * t + 1 < TAPS_C ? (uint32_t)w[(int64_t)ch * TAPS_C + 2 * t + 1].bits : 0u;
                    v = __uint_as_float(lo | (hi << 16));
                } else {
                    v = to_float(w[(int64_t)ch * TAPS_C + t]);
                }
            }
            dw_w[i] = v;
        }
        __syncthreads();
    }
    if (chunk >= a.chunks || pp >= a.pos_per_block) return; // no barrier below
    const int c0 = chunk * VEC;

    // one image and its mask per descriptor; offsets are bytes inside the image
    const uint32_t img_bytes = (uint32_t)g.h * g.w * C * (uint32_t)sizeof(TI);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<TI *>(x + (int64_t)b * g.h * g.w * C), 0, img_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(mask_in ? mask_in + (int64_t)b * g.h * g.w : nullptr), 0,
        mask_in ? (uint32_t)g.h * g.w : 0u, 0x00020000);

    // this lane's filters [channel][tap]: unpacked to fp32 for 3 x 3, left in their storage
    // form for larger kernels of 16-bit types (fewer registers; one more operation per use)
    constexpr bool WPACK = KS > 3 && sizeof(TI) == 2;
    constexpr int WBYTES = KS ? VEC * TAPS_C * (int)sizeof(TI) : 4;
    constexpr int WWORDS = (WBYTES + 3) / 4;
    uint32_t wraw[WWORDS];
    float wr[(KS && !WPACK && !WLDS && !PAIR) ? VEC * TAPS_C : 1];
    uint32_t wpr[(PAIR && !WLDS) ? VEC * kDwPairRows : 1]; // [row][channel] packed pairs of taps
    if constexpr (KS != 0 && !WLDS) {
        const TI *wp = w + (int64_t)c0 * TAPS_C;
        if constexpr (WBYTES % 16 == 0) {
#pragma unroll
            for (int k = 0; k < WBYTES / 16; ++k) {
                const u32x4 t = reinterpret_cast<const u32x4 *>(wp)[k];
                wraw[4 * k] = t.x; wraw[4 * k + 1] = t.y; wraw[4 * k + 2] = t.z; wraw[4 * k + 3] = t.w;
            }
            if constexpr (PAIR) {
#pragma unroll
                for (int v = 0; v < VEC; ++v)
#pragma unroll
                    for (int r = 0; r < kDwPairRows; ++r) {
                        const int e0 = v * TAPS_C + 2 * r, e1 = e0 + 1;
                        const uint32_t lo = (wraw[e0 >> 1] >> (16 * (e0 & 1))) & 0xffffu;
                        const uint32_t hi = 2 * r + 1 < TAPS_C ? (wraw[e1 >> 1] >> (16 * (e1 & 1))) & 0xffffu : 0u;
                        wpr[r * VEC + v] = lo | (hi << 16);
                    }
            } else if constexpr (!WPACK) {
#pragma unroll
                for (int e = 0; e < VEC * TAPS_C; ++e) wr[e] = piece_elem<TI>(wraw, e);
            }
        } else {
            static_assert(!WPACK || VEC * sizeof(TI) == 16, "packed filters come in 16-byte pieces");
#pragma unroll
            for (int e = 0; e < VEC * TAPS_C; ++e) wr[e] = to_float(wp[e]);
        }
    }
    const float *wl = dw_w + j * VEC; // WLDS: this lane's channels of tap 0
    auto filter_pair = [&](int v, int r) -> uint32_t { // taps 2r and 2r + 1 of channel v
        if constexpr (WLDS) return __float_as_uint(wl[r * CT + v]);
        else return wpr[r * VEC + v];
    };
    auto filter = [&](int v, int t) -> float {
        if constexpr (WLDS) return wl[t * CT + v];
        else if constexpr (WPACK) return piece_elem<TI>(wraw, v * TAPS_C + t);
        else return wr[v * TAPS_C + t];
    };
    float bv[WLDS ? 1 : VEC];
    if constexpr (!WLDS) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) bv[v] = bias ? bias[c0 + v] : 0.f;
    }

    const int hw_out = g.ho * g.wo;
    const int ch0 = -g.ph + g.dh * ((kh_n - 1) / 2), cw0 = -g.pw + g.dw * ((kw_n - 1) / 2);
    TO *out_img = out + (int64_t)b * hw_out * C;
    const bool relu = (g.flags & FC_RELU) != 0;
    const bool fill = (g.flags & FC_SKIP_ZERO_FILL) == 0;

    for (int p = blockIdx.x * a.pos_per_block + pp; p < hw_out; p += gridDim.x * a.pos_per_block) {
        const int oh = (int)fast_div((uint32_t)p, a.div_wo);
        const int ow = p - oh * g.wo;
        TO *orow = out_img + (int64_t)p * C + c0;
        if (mask_in) {
            // the position's label: the input mask under the centre tap, clamped into the image
            int ihc = oh * g.sh + ch0, iwc = ow * g.sw + cw0;
            ihc = ihc < 0 ? 0 : (ihc > g.h - 1 ? g.h - 1 : ihc);
            iwc = iwc < 0 ? 0 : (iwc > g.w - 1 ? g.w - 1 : iwc);
            if (__builtin_amdgcn_raw_buffer_load_b8(rm, (uint32_t)(ihc * g.w + iwc), 0, 0) == 0) {
                if (fill) {
                    float z[VEC];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) z[v] = 0.f;
                    store_piece<TO, VEC>(orow, z);
                }
                continue;
            }
        }
        const int ih0 = oh * g.sh - g.ph, iw0 = ow * g.sw - g.pw;
        if constexpr (WPACK) {
            // keep the filters packed across iterations (otherwise their unpacked form is
            // hoisted out of the loop and the register count triples)
#pragma unroll
            for (int k = 0; k < WWORDS; ++k) __asm__ volatile("" : "+v"(wraw[k]));
        }
        float acc[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = WLDS ? wl[WROWS * CT + v] : bv[WLDS ? 0 : v];

        if constexpr (KS != 0) {
            // 3 x 3: all nine taps in flight at once; larger kernels one kernel row at a time
            constexpr int ROWS = KS == 3 ? KS : 1; // kernel rows per group
            constexpr int GT = ROWS * KS;          // taps per group
#pragma unroll
            for (int kh0 = 0; kh0 < KS; kh0 += ROWS) {
                // pixel index of every tap of the group inside the image, or out of range
                uint32_t pix[GT];
#pragma unroll
                for (int r = 0; r < ROWS; ++r) {
                    const int ih = ih0 + (kh0 + r) * g.dh;
                    const bool row_ok = (uint32_t)ih < (uint32_t)g.h;
#pragma unroll
                    for (int kw = 0; kw < KS; ++kw) {
                        const int iw = iw0 + kw * g.dw;
                        const bool ok = row_ok && (uint32_t)iw < (uint32_t)g.w;
                        pix[r * KS + kw] = ok ? (uint32_t)(ih * g.w + iw) : kDwOutOfRange;
                    }
                }
                if (mask_in) {
                    uint32_t mb[GT];
#pragma unroll
                    for (int t = 0; t < GT; ++t) mb[t] = __builtin_amdgcn_raw_buffer_load_b8(rm, pix[t], 0, 0);
#pragma unroll
                    for (int t = 0; t < GT; ++t) pix[t] = mb[t] ? pix[t] : kDwOutOfRange;
                }
                RawWords<PIECE> xv[GT];
#pragma unroll
                for (int t = 0; t < GT; ++t) {
                    const uint32_t off = pix[t] == kDwOutOfRange
                                             ? kDwOutOfRange
                                             : pix[t] * (uint32_t)(C * (int)sizeof(TI)) + (uint32_t)(c0 * (int)sizeof(TI));
                    xv[t] = buffer_load<PIECE>(rx, off);
                }
                if constexpr (PAIR) {
#pragma unroll
                    for (int r = 0; r < kDwPairRows; ++r)
#pragma unroll
                        for (int q = 0; q < VEC / 2; ++q) {
                            const uint32_t x0 = xv[2 * r].v[q];
                            const uint32_t x1 = 2 * r + 1 < GT ? xv[2 * r + 1 < GT ? 2 * r + 1 : 0].v[q] : 0u;
                            // channel 2q of both taps, channel 2q + 1 of both taps
                            const uint32_t even = __builtin_amdgcn_perm(x1, x0, 0x05040100u);
                            const uint32_t odd = __builtin_amdgcn_perm(x1, x0, 0x07060302u);
                            acc[2 * q] = dot2_acc<TI>(even, filter_pair(2 * q, r), acc[2 * q]);
                            acc[2 * q + 1] = dot2_acc<TI>(odd, filter_pair(2 * q + 1, r), acc[2 * q + 1]);
                        }
                } else {
#pragma unroll
                    for (int t = 0; t < GT; ++t)
#pragma unroll
                        for (int v = 0; v < VEC; ++v)
                            acc[v] = fmaf(piece_elem<TI>(xv[t].v, v), filter(v, kh0 * KS + t), acc[v]);
                }
            }
        } else {
            for (int kh = 0; kh < kh_n; ++kh) {
                const int ih = ih0 + kh * g.dh;
                if ((uint32_t)ih >= (uint32_t)g.h) continue;
                for (int kw = 0; kw < kw_n; ++kw) {
                    const int iw = iw0 + kw * g.dw;
                    if ((uint32_t)iw >= (uint32_t)g.w) continue;
                    const uint32_t px = (uint32_t)(ih * g.w + iw);
                    if (mask_in && __builtin_amdgcn_raw_buffer_load_b8(rm, px, 0, 0) == 0) continue;
                    const RawWords<PIECE> xv =
                        buffer_load<PIECE>(rx, px * (uint32_t)(C * (int)sizeof(TI)) + (uint32_t)(c0 * (int)sizeof(TI)));
                    const int t = kh * kw_n + kw;
#pragma unroll
                    for (int v = 0; v < VEC; ++v)
                        acc[v] = fmaf(piece_elem<TI>(xv.v, v), to_float(w[(int64_t)(c0 + v) * taps + t]), acc[v]);
                }
            }
        }
        if (relu) {
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                if (!(acc[v] > 0.f)) acc[v] = (acc[v] != acc[v]) ? acc[v] : 0.f;
        }
        store_piece<TO, VEC>(orow, acc);
    }
}

constexpr size_t kDwWldsBytes = 20 * 1024; // filters in LDS only while eight workgroups still fit a CU

template <typename TI, typename TO, int VEC, int KS>
hipError_t launch_k(const Geom &g, const void *x, const uint8_t *mask_in, const void *w, const float *bias,
                    void *out, hipStream_t s)
{
    DwArgs a;
    a.g = g;
    a.chunks = g.c_in / VEC;
    const int ctiles = (a.chunks + kDwThreads - 1) / kDwThreads;
    a.lanes_per_pos = (a.chunks + ctiles - 1) / ctiles;
    a.pos_per_block = kDwThreads / a.lanes_per_pos;
    a.div_wo = make_fastdiv((uint32_t)g.wo);
    const int64_t hw_out = (int64_t)g.ho * g.wo;
    const int64_t need = (hw_out + a.pos_per_block - 1) / a.pos_per_block;
    constexpr bool pair = KS == 3 && sizeof(TI) == 2 && VEC == 8; // as in the kernel
    const size_t wlds = (size_t)((pair ? kDwPairRows : KS * KS) + 1) * a.lanes_per_pos * VEC * sizeof(float);
    const bool use_wlds = KS == 3 && VEC > 1 && wlds <= kDwWldsBytes;
    // eight workgroups per CU with the filters in LDS when every workgroup still has a few steps
    // to do (its start-up is not free), else four
    const bool wide_grid = use_wlds && need * g.n * ctiles >= 4 * kDwTargetBlocks;
    int64_t cap = (wide_grid ? 2 : 1) * kDwTargetBlocks / ((int64_t)g.n * ctiles);
    if (cap < 1) cap = 1;
    const int gx = (int)(need < cap ? need : cap);
    if constexpr (KS == 3 && VEC > 1) {
        if (use_wlds) {
            hipLaunchKernelGGL((k_dwconv<TI, TO, VEC, KS, true>), dim3(gx, g.n, ctiles), dim3(kDwThreads), wlds, s, a,
                               (const TI *)x, mask_in, (const TI *)w, bias, (TO *)out);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((k_dwconv<TI, TO, VEC, KS, false>), dim3(gx, g.n, ctiles), dim3(kDwThreads), 0, s, a,
                       (const TI *)x, mask_in, (const TI *)w, bias, (TO *)out);
    return hipGetLastError();
}

template <typename TI, typename TO>
hipError_t launch_t(const Geom &g, const void *x, const uint8_t *mask_in, const void *w, const float *bias,
                    void *out, hipStream_t s)
{
    constexpr int VEC = 16 / (int)sizeof(TI);
    const bool square = g.kh == g.kw;
    if (g.c_in % VEC == 0) {
        if (square && g.kh == 3) return launch_k<TI, TO, VEC, 3>(g, x, mask_in, w, bias, out, s);
        if (square && g.kh == 5) return launch_k<TI, TO, VEC, 5>(g, x, mask_in, w, bias, out, s);
        return launch_k<TI, TO, VEC, 0>(g, x, mask_in, w, bias, out, s);
    }
    if (square && g.kh == 3) return launch_k<TI, TO, 1, 3>(g, x, mask_in, w, bias, out, s);
    return launch_k<TI, TO, 1, 0>(g, x, mask_in, w, bias, out, s);
}

} // namespace

bool conv_depthwise_supported(const Geom &g, int in_dtype)
{
    const uint64_t e = in_dtype == FC_F32 ? 4u : 2u;
    // one image per buffer descriptor; images of a batch are separate grid rows
    if ((uint64_t)g.h * g.w * g.c_in * e >= kDwBufferLimit) return false;
    if (g.n > 65535) return false;
    return true;
}

hipError_t launch_conv_depthwise(const Geom &g, int in_dtype, int out_dtype, const void *x, const uint8_t *mask_in,
                                 const void *w, const float *bias, void *out, hipStream_t s)
{
    if (in_dtype == FC_F32) return launch_t<float, float>(g, x, mask_in, w, bias, out, s);
    if (in_dtype == FC_BF16) {
        if (out_dtype == FC_F32) return launch_t<bf16_t, float>(g, x, mask_in, w, bias, out, s);
        return launch_t<bf16_t, bf16_t>(g, x, mask_in, w, bias, out, s);
    }
    if (out_dtype == FC_F32) return launch_t<f16_t, float>(g, x, mask_in, w, bias, out, s);
    return launch_t<f16_t, f16_t>(g, x, mask_in, w, bias, out, s);
}

} // namespace fc
