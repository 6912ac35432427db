// Focused convolution on the gfx950 matrix cores (Sec. III-A: a GEMM over the
// kept patches only, with the dense layer's weights).
//
// GEMM view: rows = kept output positions (from the index list), reduction
// K = (tap, input channel), columns = output channels.  The patch matrix is never
// stored: for every (tap, 64-channel chunk) the workgroup gathers, for each of
// its TM positions, the 128 contiguous bytes of that tap's NHWC pixel into LDS
// (zeros where the tap falls outside the image or on an irrelevant input pixel),
// next to the TN x 64 slab of weights for the same tap, and feeds both to
// v_mfma_f32_32x32x16 with fp32 accumulators.
//
// The weights are the MFMA's A operand (rows = output channel) and the gathered
// activations its B operand (columns = position), so a lane's accumulators hold
// 4 consecutive output channels of one position: the epilogue (bias, ReLU, one
// round-to-nearest-even) stores 8 or 16 contiguous bytes per lane straight into
// the position's NHWC row.
//
// The launch grid never depends on the kept count: workgroups stride over the
// tiles and read the count on the device.
#include "fc_internal.hpp"

namespace fc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

template <int DT>
__device__ __forceinline__ f32x16_t mfma32(const uint4 &a, const uint4 &b, const f32x16_t &c)
{
    if constexpr (DT == FC_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

constexpr int kTK = 64;         // reduction elements per stage (one 128-byte pixel chunk)
constexpr int kTKP = kTK + 8;   // LDS row pitch in elements: 144 B keeps 128-bit reads conflict-free
constexpr int kMaxTaps = 32;    // tap-valid bits per row live in one 32-bit word

template <int TM, int TN>
constexpr size_t mfma_lds_bytes()
{
    return (size_t)2 * (TM + TN) * kTKP * sizeof(uint16_t) + (size_t)TM * 3 * sizeof(int32_t);
}

template <int DT, typename TO>
__device__ __forceinline__ void store4(TO *dst, float a, float b, float c, float d)
{
    if constexpr (sizeof(TO) == 4) {
        *reinterpret_cast<float4 *>(dst) = make_float4(a, b, c, d);
    } else if constexpr (DT == FC_BF16) {
        uint2 v;
        v.x = (uint32_t)bf16_bits_rne(a) | ((uint32_t)bf16_bits_rne(b) << 16);
        v.y = (uint32_t)bf16_bits_rne(c) | ((uint32_t)bf16_bits_rne(d) << 16);
        *reinterpret_cast<uint2 *>(dst) = v;
    } else {
        uint2 v;
        v.x = (uint32_t)f16_bits_rne(a) | ((uint32_t)f16_bits_rne(b) << 16);
        v.y = (uint32_t)f16_bits_rne(c) | ((uint32_t)f16_bits_rne(d) << 16);
        *reinterpret_cast<uint2 *>(dst) = v;
    }
}

__device__ __forceinline__ float relu_keep_nan(float v) { return (v > 0.f || v != v) ? v : 0.f; }

// DT: storage type of x and w; TO: float or a 16-bit carrier; TM x TN: workgroup
// tile (positions x output channels); WM x WN: wave grid inside it.
template <int DT, typename TO, int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64) void k_conv_mfma(Geom g, const uint16_t *__restrict__ x,
                                                            const uint8_t *__restrict__ mask_in,
                                                            const uint16_t *__restrict__ w,
                                                            const float *__restrict__ bias,
                                                            const int32_t *__restrict__ idx,
                                                            const int32_t *__restrict__ count,
                                                            TO *__restrict__ out)
{
    constexpr int NT = WM * WN * 64;
    constexpr int RPP = NT / 8;        // rows covered by one pass of 16-byte loads
    constexpr int XR = TM / RPP;       // 16-byte pieces of the activation tile per thread
    constexpr int WR = TN / RPP;       // ... of the weight tile
    constexpr int WTM = TM / WM, WTN = TN / WN;
    constexpr int PB = WTM / 32, CB = WTN / 32;
    static_assert(TM % RPP == 0 && TN % RPP == 0 && WTM % 32 == 0 && WTN % 32 == 0, "tile shape");

    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint16_t *Xs = reinterpret_cast<uint16_t *>(smem_raw);             // [2][TM][kTKP]
    uint16_t *Ws = Xs + 2 * TM * kTKP;                                 // [2][TN][kTKP]
    int32_t *row_p = reinterpret_cast<int32_t *>(Ws + 2 * TN * kTKP);  // flat output position or -1
    int32_t *row_base = row_p + TM;                                    // pixel index of tap (0,0)
    uint32_t *row_bits = reinterpret_cast<uint32_t *>(row_base + TM);  // bit t: tap t is inside and relevant

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave % WM, wave_n = wave / WM;
    const int piece = tid & 7, prow = tid >> 3;

    const int rows = idx ? *count : g.m;
    const int n_nt = (g.c_out + TN - 1) / TN;
    const int ntiles = ((rows + TM - 1) / TM) * n_nt;
    const int taps = g.kh * g.kw;
    const int cchunks = (g.c_in + kTK - 1) / kTK;
    const int stages = taps * cchunks;

    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int mt = tile / n_nt, nt = tile - mt * n_nt;
        const int co0 = nt * TN;

        __syncthreads(); // the previous tile's epilogue and last stage are done with LDS
        for (int r = tid; r < TM; r += NT) {
            const int m = mt * TM + r;
            int p = -1, base = 0;
            uint32_t bits = 0;
            if (m < rows) {
                p = idx ? idx[m] : m;
                const int ow = p % g.wo;
                const int q = p / g.wo;
                const int oh = q % g.ho;
                const int b = q / g.ho;
                const int ih0 = oh * g.sh - g.ph, iw0 = ow * g.sw - g.pw;
                base = (b * g.h + ih0) * g.w + iw0;
                for (int kh = 0; kh < g.kh; ++kh) {
                    const int ih = ih0 + kh * g.dh;
                    for (int kw = 0; kw < g.kw; ++kw) {
                        const int iw = iw0 + kw * g.dw;
                        bool ok = ih >= 0 && ih < g.h && iw >= 0 && iw < g.w;
                        if (ok && mask_in) ok = mask_in[(int64_t)(b * g.h + ih) * g.w + iw] != 0;
                        bits |= ok ? (1u << (kh * g.kw + kw)) : 0u;
                    }
                }
            }
            row_p[r] = p;
            row_base[r] = base;
            row_bits[r] = bits;
        }
        __syncthreads();

        int xbase[XR];
        uint32_t xbits[XR];
#pragma unroll
        for (int j = 0; j < XR; ++j) {
            xbase[j] = row_base[prow + j * RPP];
            xbits[j] = row_bits[prow + j * RPP];
        }

        f32x16_t acc[PB][CB];
#pragma unroll
        for (int a = 0; a < PB; ++a)
#pragma unroll
            for (int b = 0; b < CB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

        uint4 xr[XR], wr[WR];
        int tap = 0, cc = 0, kh = 0, kw = 0; // of the stage being loaded

        auto load_stage = [&]() {
            const int ci = cc * kTK + piece * 8;
            const bool ci_ok = ci < g.c_in;
            const int tapoff = (kh * g.dh) * g.w + kw * g.dw;
#pragma unroll
            for (int j = 0; j < XR; ++j) {
                const bool ok = ci_ok && ((xbits[j] >> tap) & 1u);
                xr[j] = ok ? *reinterpret_cast<const uint4 *>(x + (int64_t)(xbase[j] + tapoff) * g.c_in + ci)
                           : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < WR; ++j) {
                const int co = co0 + prow + j * RPP;
                const bool ok = ci_ok && co < g.c_out;
                wr[j] = ok ? *reinterpret_cast<const uint4 *>(w + ((int64_t)co * taps + tap) * g.c_in + ci)
                           : make_uint4(0, 0, 0, 0);
            }
            if (++cc == cchunks) {
                cc = 0;
                ++tap;
                if (++kw == g.kw) {
                    kw = 0;
                    ++kh;
                }
            }
        };
        auto store_stage = [&](int buf) {
            uint16_t *xs = Xs + buf * TM * kTKP, *ws = Ws + buf * TN * kTKP;
#pragma unroll
            for (int j = 0; j < XR; ++j)
                *reinterpret_cast<uint4 *>(xs + (prow + j * RPP) * kTKP + piece * 8) = xr[j];
#pragma unroll
            for (int j = 0; j < WR; ++j)
                *reinterpret_cast<uint4 *>(ws + (prow + j * RPP) * kTKP + piece * 8) = wr[j];
        };

        load_stage();
        store_stage(0);
        __syncthreads();

        for (int s = 0; s < stages; ++s) {
            const int cur = s & 1;
            if (s + 1 < stages) load_stage();
            const uint16_t *xs = Xs + cur * TM * kTKP + (wave_m * WTM + (lane & 31)) * kTKP + (lane >> 5) * 8;
            const uint16_t *ws = Ws + cur * TN * kTKP + (wave_n * WTN + (lane & 31)) * kTKP + (lane >> 5) * 8;
#pragma unroll
            for (int kk = 0; kk < kTK / 16; ++kk) {
                uint4 wf[CB], xf[PB];
#pragma unroll
                for (int b = 0; b < CB; ++b) wf[b] = *reinterpret_cast<const uint4 *>(ws + b * 32 * kTKP + kk * 16);
#pragma unroll
                for (int a = 0; a < PB; ++a) xf[a] = *reinterpret_cast<const uint4 *>(xs + a * 32 * kTKP + kk * 16);
#pragma unroll
                for (int a = 0; a < PB; ++a)
#pragma unroll
                    for (int b = 0; b < CB; ++b) acc[a][b] = mfma32<DT>(wf[b], xf[a], acc[a][b]);
            }
            if (s + 1 < stages) store_stage(cur ^ 1);
            __syncthreads();
        }

        // epilogue: lane holds position (lane & 31) of each 32-block and channels
        // 8*q + 4*(lane >> 5) + {0..3} of each 32-channel block
#pragma unroll
        for (int a = 0; a < PB; ++a) {
            const int p = row_p[wave_m * WTM + a * 32 + (lane & 31)];
            if (p < 0) continue;
            TO *orow = out + (int64_t)p * g.c_out;
#pragma unroll
            for (int b = 0; b < CB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int co = co0 + wave_n * WTN + b * 32 + q * 8 + (lane >> 5) * 4;
                    if (co >= g.c_out) continue;
                    float v0 = acc[a][b][q * 4 + 0], v1 = acc[a][b][q * 4 + 1];
                    float v2 = acc[a][b][q * 4 + 2], v3 = acc[a][b][q * 4 + 3];
                    if (bias) {
                        const float4 bv = *reinterpret_cast<const float4 *>(bias + co);
                        v0 += bv.x; v1 += bv.y; v2 += bv.z; v3 += bv.w;
                    }
                    if (g.flags & FC_RELU) {
                        v0 = relu_keep_nan(v0); v1 = relu_keep_nan(v1);
                        v2 = relu_keep_nan(v2); v3 = relu_keep_nan(v3);
                    }
                    store4<DT, TO>(orow + co, v0, v1, v2, v3);
                }
        }
    }
}

// ---------------------------------------------------------------------------

bool conv_mfma_supported(const Geom &g, int in_dtype, int out_dtype)
{
    if (in_dtype != FC_BF16 && in_dtype != FC_F16) return false;
    if (out_dtype != in_dtype && out_dtype != FC_F32) return false;
    if (g.c_in % 8 != 0 || g.c_out % 8 != 0) return false; // 16-byte gathers, 4-channel stores
    if (g.kh * g.kw > kMaxTaps) return false;
    return true;
}

template <int DT, typename TO, int TM, int TN, int WM, int WN>
static hipError_t launch_cfg(const Geom &g, const void *x, const uint8_t *mask_in, const void *w,
                             const float *bias, const int32_t *idx, const int32_t *count, void *out,
                             hipStream_t s)
{
    auto kern = k_conv_mfma<DT, TO, TM, TN, WM, WN>;
    constexpr size_t lds = mfma_lds_bytes<TM, TN>();
    static bool attr_set = false; // per instantiation; the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // grid for the dense row count; workgroups beyond the kept tiles exit at once
    const int64_t max_tiles = (int64_t)((g.m + TM - 1) / TM) * ((g.c_out + TN - 1) / TN);
    const int64_t cap = 256 * 8;
    const int blocks = (int)(max_tiles < cap ? max_tiles : cap);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(WM * WN * 64), lds, s, g, (const uint16_t *)x, mask_in,
                       (const uint16_t *)w, bias, idx, count, (TO *)out);
    return hipGetLastError();
}

template <int DT, typename TO>
static hipError_t launch_dt(const Geom &g, const void *x, const uint8_t *mask_in, const void *w,
                            const float *bias, const int32_t *idx, const int32_t *count, void *out,
                            hipStream_t s)
{
    if (g.c_out > 64) return launch_cfg<DT, TO, 128, 128, 2, 2>(g, x, mask_in, w, bias, idx, count, out, s);
    return launch_cfg<DT, TO, 128, 64, 2, 2>(g, x, mask_in, w, bias, idx, count, out, s);
}

hipError_t launch_conv_mfma(const Geom &g, int in_dtype, int out_dtype, const void *x, const uint8_t *mask_in,
                            const void *w, const float *bias, const int32_t *idx, const int32_t *count,
                            void *out, hipStream_t s)
{
    if (in_dtype == FC_BF16) {
        if (out_dtype == FC_F32) return launch_dt<FC_BF16, float>(g, x, mask_in, w, bias, idx, count, out, s);
        return launch_dt<FC_BF16, uint16_t>(g, x, mask_in, w, bias, idx, count, out, s);
    }
    if (out_dtype == FC_F32) return launch_dt<FC_F16, float>(g, x, mask_in, w, bias, idx, count, out, s);
    return launch_dt<FC_F16, uint16_t>(g, x, mask_in, w, bias, idx, count, out, s);
}

} // namespace fc
