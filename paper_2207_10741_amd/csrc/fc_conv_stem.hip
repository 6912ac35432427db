// Focused convolution on the matrix cores for layers with very few input channels
// (RGB stems: C_in <= 4, K = KH*KW*C_in small).  Sec. III-A: only the kept patches
// become columns of the product.
//
// Such a layer is far too thin for the gather of the wide-layer kernel (a pixel is 6 bytes,
// not a 128-byte chunk), but its whole reduction fits a handful of 16-wide MFMA steps.  So
// the patch of a kept position is gathered element by element straight into the MFMA's
// B-operand registers: lane l of a wave owns position l % 32 of its 32-row block and the
// reduction elements (l / 32) * 8 .. + 8 of every 16-wide step; a small table in LDS gives,
// for each reduction index k = (kh, kw, ci), the tap number and the element offset from the
// position's first tap.  A tap that falls outside the image or on an irrelevant input pixel
// contributes zeros and is never loaded.  The weights of 64 output channels sit in LDS as
// the A operand for the whole kernel; accumulators start from the bias; the epilogue applies
// ReLU, rounds once, transposes the tile through LDS and stores whole 16-byte row pieces.
#include "fc_mfma_util.hpp"

namespace fc {

constexpr int kStemThreads = 256;   // 4 waves, 32 positions each
constexpr int kStemRows = 128;      // positions per tile
constexpr int kStemCo = 64;         // output channels per workgroup
constexpr int kStemMaxK = 160;      // padded reduction length the tables are sized for (7x7x3 = 147)
constexpr int kStemMaxTaps = 64;    // tap-valid bits live in one 64-bit word per position

bool conv_stem_supported(const Geom &g, int in_dtype, int out_dtype)
{
    if (in_dtype != FC_BF16 && in_dtype != FC_F16) return false;
    if (out_dtype != in_dtype && out_dtype != FC_F32) return false;
    if (g.c_in > 4 || g.c_out % 8 != 0) return false;
    if (g.kh * g.kw > kStemMaxTaps || (g.kh * g.kw * g.c_in + 15) / 16 * 16 > kStemMaxK) return false;
    // element offset of the last tap from the first one, packed into 24 bits of a table entry
    const int64_t far = ((int64_t)(g.kh - 1) * g.dh * g.w + (int64_t)(g.kw - 1) * g.dw) * g.c_in + g.c_in;
    if (far >= (1 << 24)) return false;
    if ((int64_t)g.n * g.h * g.w * g.c_in >= INT32_MAX) return false; // 32-bit element indices
    return true;
}

template <int DT, typename TO>
__global__ __launch_bounds__(kStemThreads) void k_conv_stem(Geom g, const uint16_t *__restrict__ x,
                                                            const uint8_t *__restrict__ mask_in,
                                                            const uint16_t *__restrict__ w,
                                                            const float *__restrict__ bias,
                                                            const int32_t *__restrict__ idx,
                                                            const int32_t *__restrict__ count,
                                                            TO *__restrict__ out)
{
    constexpr int WPITCH = kStemMaxK * 2 + 16;                 // bytes per weight row in LDS
    constexpr int OP = kStemCo * (int)sizeof(TO) + 16;         // bytes per output row in LDS
    __shared__ __align__(16) unsigned char w_s[kStemCo * WPITCH];   // [channel][k] as stored
    __shared__ __align__(16) unsigned char o_s[kStemRows * OP];
    __shared__ __align__(16) uint32_t lut[kStemMaxK];               // tap << 24 | element offset
    __shared__ int32_t row_p[kStemRows];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    const int rows = idx ? *count : g.m;
    const int taps = g.kh * g.kw;
    const int K = taps * g.c_in;
    const int ksteps = (K + 15) / 16;
    const int co0 = blockIdx.y * kStemCo;

    // ---- once per workgroup: weights and the reduction-index table ----
    for (int i = tid; i < kStemCo * ksteps * 16; i += kStemThreads) {
        const int j = i / (ksteps * 16), k = i - j * (ksteps * 16);
        const int co = co0 + j;
        const uint16_t v = (co < g.c_out && k < K) ? w[(int64_t)co * K + k] : (uint16_t)0;
        *reinterpret_cast<uint16_t *>(w_s + j * WPITCH + k * 2) = v;
    }
    for (int k = tid; k < ksteps * 16; k += kStemThreads) {
        uint32_t e = 0xff000000u; // padding of the reduction: a tap number no position has
        if (k < K) {
            const int tap = k / g.c_in, ci = k - tap * g.c_in;
            const int kh = tap / g.kw, kw = tap - kh * g.kw;
            e = ((uint32_t)tap << 24) | (uint32_t)((kh * g.dh * g.w + kw * g.dw) * g.c_in + ci);
        }
        lut[k] = e;
    }
    __syncthreads();

    // bias of this lane's channels (channel = cb*32 + (i/4)*8 + half*4 + i%4 of accumulator i)
    float4 bias_q[2][4];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int co = co0 + cb * 32 + q * 8 + half * 4;
            bias_q[cb][q] = (bias && co < g.c_out) ? *reinterpret_cast<const float4 *>(bias + co)
                                                    : make_float4(0.f, 0.f, 0.f, 0.f);
        }

    const int ntiles = (rows + kStemRows - 1) / kStemRows;
    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        // ---- this lane's position and its tap-valid bits ----
        const int r = tile * kStemRows + wave * 32 + (lane & 31);
        int p = -1, base = 0;
        uint64_t bits = 0;
        if (r < rows) {
            p = idx ? idx[r] : r;
            const int ow = p % g.wo;
            const int q = p / g.wo;
            const int oh = q % g.ho;
            const int b = q / g.ho;
            const int ih0 = oh * g.sh - g.ph, iw0 = ow * g.sw - g.pw;
            base = ((b * g.h + ih0) * g.w + iw0) * g.c_in; // may point before the image: only used with a valid tap
            // the two halves of the wave own the same positions: each looks at half of the taps
            for (int t = half; t < taps; t += 2) {
                const int kh = t / g.kw, kw = t - kh * g.kw;
                const int ih = ih0 + kh * g.dh, iw = iw0 + kw * g.dw;
                bool ok = ih >= 0 && ih < g.h && iw >= 0 && iw < g.w;
                if (ok && mask_in) ok = mask_in[((int64_t)b * g.h + ih) * g.w + iw] != 0;
                bits |= (uint64_t)ok << t;
            }
        }
        {
            // merge the halves' bits
            const uint32_t lo = (uint32_t)bits, hi = (uint32_t)(bits >> 32);
            const uint32_t lo2 = lo | (uint32_t)__shfl_xor((int)lo, 32, 64);
            const uint32_t hi2 = hi | (uint32_t)__shfl_xor((int)hi, 32, 64);
            bits = (uint64_t)lo2 | ((uint64_t)hi2 << 32);
        }
        if (half == 0) row_p[wave * 32 + (lane & 31)] = p;

        f32x16_t acc[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc[cb][q * 4 + 0] = bias_q[cb][q].x;
                acc[cb][q * 4 + 1] = bias_q[cb][q].y;
                acc[cb][q * 4 + 2] = bias_q[cb][q].z;
                acc[cb][q * 4 + 3] = bias_q[cb][q].w;
            }

        for (int j = 0; j < ksteps; ++j) {
            // this lane's 8 reduction elements of step j
            const uint4 e0 = *reinterpret_cast<const uint4 *>(&lut[j * 16 + half * 8]);
            const uint4 e1 = *reinterpret_cast<const uint4 *>(&lut[j * 16 + half * 8 + 4]);
            const uint32_t ent[8] = {e0.x, e0.y, e0.z, e0.w, e1.x, e1.y, e1.z, e1.w};
            uint32_t val[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t tap = ent[e] >> 24;
                const bool ok = tap < (uint32_t)kStemMaxTaps && ((bits >> tap) & 1ull);
                val[e] = ok ? (uint32_t)x[base + (int)(ent[e] & 0xffffffu)] : 0u;
            }
            uint4 xf;
            xf.x = val[0] | (val[1] << 16);
            xf.y = val[2] | (val[3] << 16);
            xf.z = val[4] | (val[5] << 16);
            xf.w = val[6] | (val[7] << 16);
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const uint4 wf = *reinterpret_cast<const uint4 *>(w_s + (cb * 32 + (lane & 31)) * WPITCH +
                                                                   (j * 16 + half * 8) * 2);
                acc[cb] = mfma32<DT>(wf, xf, acc[cb]);
            }
        }

        // ---- epilogue: ReLU, one rounding, transposed through LDS, 16-byte row pieces ----
        __syncthreads(); // the previous tile's stores have read o_s; row_p is complete
        const int rl = wave * 32 + (lane & 31);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cl = cb * 32 + q * 8 + half * 4;
                float v0 = acc[cb][q * 4 + 0], v1 = acc[cb][q * 4 + 1];
                float v2 = acc[cb][q * 4 + 2], v3 = acc[cb][q * 4 + 3];
                if constexpr (sizeof(TO) == 4) {
                    if (g.flags & FC_RELU) {
                        v0 = relu_keep_nan(v0); v1 = relu_keep_nan(v1);
                        v2 = relu_keep_nan(v2); v3 = relu_keep_nan(v3);
                    }
                    store4<DT, TO>(reinterpret_cast<TO *>(o_s + rl * OP) + cl, v0, v1, v2, v3);
                } else {
                    uint2 pk;
                    store4<DT, TO>(reinterpret_cast<TO *>(&pk), v0, v1, v2, v3);
                    if (g.flags & FC_RELU) {
                        pk.x = relu_packed16(pk.x);
                        pk.y = relu_packed16(pk.y);
                    }
                    *reinterpret_cast<uint2 *>(o_s + rl * OP + cl * 2) = pk;
                }
            }
        __syncthreads();
        constexpr int PPR = kStemCo * (int)sizeof(TO) / 16; // 16-byte pieces per row
        constexpr int EPT = 16 / (int)sizeof(TO);
        for (int i = tid; i < kStemRows * PPR; i += kStemThreads) {
            const int rr = i / PPR, pc = i - rr * PPR;
            const int pp = row_p[rr];
            const int co = co0 + pc * EPT;
            if (pp >= 0 && co < g.c_out)
                __builtin_nontemporal_store(*reinterpret_cast<const u32x4_t *>(o_s + rr * OP + pc * 16),
                                            reinterpret_cast<u32x4_t *>(out + (int64_t)pp * g.c_out + co));
        }
        __syncthreads(); // everyone is done with row_p and o_s before the next tile rewrites them
    }
}

template <int DT, typename TO>
static hipError_t launch_stem_t(const Geom &g, const void *x, const uint8_t *mask_in, const void *w,
                                const float *bias, const int32_t *idx, const int32_t *count, void *out,
                                hipStream_t s)
{
    // grid sized for the dense row count (the kept count is only known on the device),
    // capped at a few workgroups per CU: they stride over the tiles
    const int64_t tiles = ((int64_t)g.m + kStemRows - 1) / kStemRows;
    const int gx = (int)(tiles > 2048 ? 2048 : tiles);
    const int gy = (g.c_out + kStemCo - 1) / kStemCo;
    hipLaunchKernelGGL((k_conv_stem<DT, TO>), dim3(gx, gy), dim3(kStemThreads), 0, s, g, (const uint16_t *)x,
                       mask_in, (const uint16_t *)w, bias, idx, count, (TO *)out);
    return hipGetLastError();
}

hipError_t launch_conv_stem(const Geom &g, int in_dtype, int out_dtype, const void *x, const uint8_t *mask_in,
                            const void *w, const float *bias, const int32_t *idx, const int32_t *count,
                            void *out, hipStream_t s)
{
    if (in_dtype == FC_BF16) {
        if (out_dtype == FC_F32) return launch_stem_t<FC_BF16, float>(g, x, mask_in, w, bias, idx, count, out, s);
        return launch_stem_t<FC_BF16, uint16_t>(g, x, mask_in, w, bias, idx, count, out, s);
    }
    if (out_dtype == FC_F32) return launch_stem_t<FC_F16, float>(g, x, mask_in, w, bias, idx, count, out, s);
    return launch_stem_t<FC_F16, uint16_t>(g, x, mask_in, w, bias, idx, count, out, s);
}

} // namespace fc
