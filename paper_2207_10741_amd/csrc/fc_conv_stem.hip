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

// bytes per weight row in LDS: the padded reduction plus one 16-byte piece, so that the 32
// rows a wave reads together start in different banks
__host__ __device__ static inline int stem_weight_pitch(int ksteps) { return ksteps * 32 + 16; }

bool conv_stem_supported(const Geom &g, int in_dtype, int out_dtype)
{
    if (in_dtype != FC_BF16 && in_dtype != FC_F16) return false;
    if (out_dtype != in_dtype && out_dtype != FC_F32 && out_dtype != FC_FP8) return false;
    if (g.c_in > 4 || g.c_out % 8 != 0) return false;
    if (out_dtype == FC_FP8 && g.c_out % 16 != 0) return false; // rows are stored in 16-byte pieces
    if (g.kh * g.kw > kStemMaxTaps || (g.kh * g.kw * g.c_in + 15) / 16 * 16 > kStemMaxK) return false;
    // element offset of the last tap from the first one, packed into 24 bits of a table entry
    const int64_t far = ((int64_t)(g.kh - 1) * g.dh * g.w + (int64_t)(g.kw - 1) * g.dw) * g.c_in + g.c_in;
    if (far >= (1 << 24)) return false;
    if ((int64_t)(g.kh - 1) * g.dh >= 65536 || (int64_t)(g.kw - 1) * g.dw >= 65536) return false; // 16-bit tap offsets
    if ((int64_t)g.n * g.h * g.w * g.c_in >= INT32_MAX) return false; // 32-bit element indices
    return true;
}

// divisors of the position decode, prepared on the host
struct StemDivs {
    FastDiv wo, ho;
};

template <int DT, typename TO>
__global__ __launch_bounds__(kStemThreads, 5) void k_conv_stem(Geom g, StemDivs dv, const uint16_t *__restrict__ x,
                                                            const uint8_t *__restrict__ mask_in,
                                                            const uint16_t *__restrict__ w,
                                                            const float *__restrict__ bias,
                                                            const int32_t *__restrict__ idx,
                                                            const int32_t *__restrict__ count,
                                                            TO *__restrict__ out)
{
    constexpr int OP = kStemCo * (int)sizeof(TO) + 16;         // bytes per output row in LDS
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    const int rows = idx ? *count : g.m;
    const int taps = g.kh * g.kw;
    const int K = taps * g.c_in;
    const int ksteps = (K + 15) / 16;
    // LDS, sized by the launcher for this layer's reduction length (a 3x3x3 stem needs 24 KB,
    // so six workgroups share a CU and hide each other's gather latency)
    const int WPITCH = stem_weight_pitch(ksteps);                   // bytes per weight row
    extern __shared__ __align__(16) unsigned char stem_lds[];
    unsigned char *o_s = stem_lds;                                  // [rows][OP]
    unsigned char *w_s = o_s + kStemRows * OP;                      // [channel][k] as stored
    uint32_t *lut = reinterpret_cast<uint32_t *>(w_s + kStemCo * WPITCH); // tap << 24 | element offset
    int32_t *row_p = reinterpret_cast<int32_t *>(lut + ksteps * 16);
    float *bias_s = reinterpret_cast<float *>(row_p + kStemRows);   // [channel]
    uint32_t *tap_s = reinterpret_cast<uint32_t *>(bias_s + kStemCo); // [tap] kh*dh | kw*dw << 16
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
    if (tid < kStemCo) bias_s[tid] = (bias && co0 + tid < g.c_out) ? bias[co0 + tid] : 0.f;
    if (tid < kStemMaxTaps) {
        const int kh = tid / g.kw, kw = tid - kh * g.kw;
        tap_s[tid] = tid < taps ? (uint32_t)(kh * g.dh) | ((uint32_t)(kw * g.dw) << 16) : 0u;
    }
    __syncthreads();
    const uint64_t all_taps = taps >= 64 ? ~0ull : ((1ull << taps) - 1ull);
    const int reach_h = (g.kh - 1) * g.dh, reach_w = (g.kw - 1) * g.dw;

    const int ntiles = (rows + kStemRows - 1) / kStemRows;
    // ---- locating a tile's rows, in pieces so that the memory round trips of the NEXT tile
    // (position list, then mask bytes) run under the gathers, MFMAs and stores of the current
    // one.  Piece 1: the list entry.  Piece 2: decode it and request the first sixteen taps'
    // mask bytes (eight per half-wave).  Piece 3: tap-valid bits from those bytes, the remaining
    // taps (kernels with more than sixteen) fetched on the spot, halves merged. ----
    struct Located {
        int p, base, ih0, iw0;
        const uint8_t *mimg;
        bool lookup;       // bits have to be built tap by tap
        bool inside[8];
        uint8_t mb[8];
    };
    auto fetch_entry = [&](int tile) -> int {
        const int r = tile * kStemRows + wave * 32 + (lane & 31);
        return r < rows ? (idx ? idx[r] : r) : -1;
    };
    auto request_taps = [&](const Located &L, int t0, bool (&inside)[8], uint8_t (&mb)[8]) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int t = t0 + 2 * u;
            const uint32_t e = tap_s[t & (kStemMaxTaps - 1)];
            const int ih = L.ih0 + (int)(e & 0xffffu), iw = L.iw0 + (int)(e >> 16);
            inside[u] = t < taps && ih >= 0 && ih < g.h && iw >= 0 && iw < g.w;
            mb[u] = 1;
            // a tap outside the image reads the image's first pixel instead and is dropped afterwards
            if (L.mimg) mb[u] = L.mimg[inside[u] ? ih * g.w + iw : 0];
        }
    };
    auto decode = [&](int p, Located &L) {
        L.p = p;
        L.base = 0;
        L.ih0 = L.iw0 = 0;
        L.mimg = nullptr;
        L.lookup = false;
        if (p >= 0) {
            const int q = (int)fast_div((uint32_t)p, dv.wo);
            const int ow = p - q * g.wo;
            const int b = (int)fast_div((uint32_t)q, dv.ho);
            const int oh = q - b * g.ho;
            L.ih0 = oh * g.sh - g.ph;
            L.iw0 = ow * g.sw - g.pw;
            L.base = ((b * g.h + L.ih0) * g.w + L.iw0) * g.c_in; // may point before the image: only used with a valid tap
            L.mimg = mask_in ? mask_in + (int64_t)b * g.h * g.w : nullptr;
            const bool interior = L.ih0 >= 0 && L.ih0 + reach_h < g.h && L.iw0 >= 0 && L.iw0 + reach_w < g.w;
            L.lookup = mask_in || !interior; // else every tap is inside the image and nothing gates it
            // the two halves of the wave own the same positions: each looks at half of the taps
            if (L.lookup) request_taps(L, half, L.inside, L.mb);
        }
    };
    auto finish = [&](const Located &L) -> uint64_t {
        uint64_t bits = 0;
        if (L.p >= 0) {
            if (!L.lookup) {
                bits = all_taps;
            } else {
#pragma unroll
                for (int u = 0; u < 8; ++u) bits |= (uint64_t)(L.inside[u] && L.mb[u] != 0) << ((half + 2 * u) & 63);
                for (int t0 = half + 16; t0 < taps; t0 += 16) {
                    bool inside[8];
                    uint8_t mb[8];
                    request_taps(L, t0, inside, mb);
#pragma unroll
                    for (int u = 0; u < 8; ++u) bits |= (uint64_t)(inside[u] && mb[u] != 0) << ((t0 + 2 * u) & 63);
                }
            }
        }
        // merge the halves' bits
        const uint32_t lo = (uint32_t)bits, hi = (uint32_t)(bits >> 32);
        const uint32_t lo2 = lo | (uint32_t)__shfl_xor((int)lo, 32, 64);
        const uint32_t hi2 = hi | (uint32_t)__shfl_xor((int)hi, 32, 64);
        return (uint64_t)lo2 | ((uint64_t)hi2 << 32);
    };

    Located nxt;
    uint64_t bits_n = 0;
    if ((int)blockIdx.x < ntiles) {
        decode(fetch_entry(blockIdx.x), nxt);
        bits_n = finish(nxt);
    }
    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int p = nxt.p, base = nxt.base;
        const uint64_t bits = bits_n;
        const bool more = tile + (int)gridDim.x < ntiles;
        const int entry_n = more ? fetch_entry(tile + gridDim.x) : -1; // piece 1 of the next tile
        if (half == 0) row_p[wave * 32 + (lane & 31)] = p;

        f32x16_t acc[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // channel = cb*32 + (i/4)*8 + half*4 + i%4 of accumulator i
                const float4 bq = *reinterpret_cast<const float4 *>(bias_s + cb * 32 + q * 8 + half * 4);
                acc[cb][q * 4 + 0] = bq.x;
                acc[cb][q * 4 + 1] = bq.y;
                acc[cb][q * 4 + 2] = bq.z;
                acc[cb][q * 4 + 3] = bq.w;
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

        if (more) decode(entry_n, nxt); // piece 2 of the next tile: its mask bytes travel during the epilogue

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
                } else if constexpr (sizeof(TO) == 1) {
                    uint32_t pk;
                    store4<DT, TO>(reinterpret_cast<TO *>(&pk), v0, v1, v2, v3);
                    if (g.flags & FC_RELU) pk = relu_packed8(pk);
                    *reinterpret_cast<uint32_t *>(o_s + rl * OP + cl) = pk;
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
        if (more) bits_n = finish(nxt); // piece 3
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
    const int ksteps = (g.kh * g.kw * g.c_in + 15) / 16;
    const size_t lds = (size_t)kStemRows * (kStemCo * sizeof(TO) + 16) + (size_t)kStemCo * stem_weight_pitch(ksteps) +
                       (size_t)ksteps * 16 * sizeof(uint32_t) + (size_t)kStemRows * sizeof(int32_t) + (size_t)kStemCo * sizeof(float) + (size_t)kStemMaxTaps * sizeof(uint32_t);
    StemDivs dv;
    dv.wo = make_fastdiv((uint32_t)g.wo);
    dv.ho = make_fastdiv((uint32_t)g.ho);
    hipLaunchKernelGGL((k_conv_stem<DT, TO>), dim3(gx, gy), dim3(kStemThreads), lds, s, g, dv, (const uint16_t *)x,
                       mask_in, (const uint16_t *)w, bias, idx, count, (TO *)out);
    return hipGetLastError();
}

hipError_t launch_conv_stem(const Geom &g, int in_dtype, int out_dtype, const void *x, const uint8_t *mask_in,
                            const void *w, const float *bias, const int32_t *idx, const int32_t *count,
                            void *out, hipStream_t s)
{
    if (in_dtype == FC_BF16) {
        if (out_dtype == FC_F32) return launch_stem_t<FC_BF16, float>(g, x, mask_in, w, bias, idx, count, out, s);
        if (out_dtype == FC_FP8) return launch_stem_t<FC_BF16, uint8_t>(g, x, mask_in, w, bias, idx, count, out, s);
        return launch_stem_t<FC_BF16, uint16_t>(g, x, mask_in, w, bias, idx, count, out, s);
    }
    if (out_dtype == FC_F32) return launch_stem_t<FC_F16, float>(g, x, mask_in, w, bias, idx, count, out, s);
    if (out_dtype == FC_FP8) return launch_stem_t<FC_F16, uint8_t>(g, x, mask_in, w, bias, idx, count, out, s);
    return launch_stem_t<FC_F16, uint16_t>(g, x, mask_in, w, bias, idx, count, out, s);
}

} // namespace fc
