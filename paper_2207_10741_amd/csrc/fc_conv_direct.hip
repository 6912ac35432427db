// Direct focused convolution for shapes the matrix-core path does not take
// (odd channel counts such as RGB stems, fp32 storage).  One lane owns one
// (active row, output channel) pair and walks the taps in the order kh, kw, ci
// with an fp32 accumulator (Sec. III-A: only the kept patches are evaluated).
#include "fc_internal.hpp"

namespace fc {

template <typename TI, typename TO>
__global__ __launch_bounds__(256) void k_conv_direct(Geom g, const TI *__restrict__ x,
                                                     const uint8_t *__restrict__ mask_in,
                                                     const TI *__restrict__ w, const float *__restrict__ bias,
                                                     const int32_t *__restrict__ idx,
                                                     const int32_t *__restrict__ count, TO *__restrict__ out)
{
    const int rows = idx ? *count : g.m;
    const int64_t total = (int64_t)rows * g.c_out;
    const int taps_k = g.kh * g.kw * g.c_in;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (int64_t)gridDim.x * blockDim.x) {
        const int co = (int)(t % g.c_out);
        const int r = (int)(t / g.c_out);
        const int p = idx ? idx[r] : r;
        const int ow = p % g.wo;
        const int q = p / g.wo;
        const int oh = q % g.ho;
        const int b = q / g.ho;
        float acc = 0.f;
        const TI *wrow = w + (int64_t)co * taps_k;
        for (int kh = 0; kh < g.kh; ++kh) {
            const int ih = oh * g.sh - g.ph + kh * g.dh;
            if (ih < 0 || ih >= g.h) continue;
            for (int kw = 0; kw < g.kw; ++kw) {
                const int iw = ow * g.sw - g.pw + kw * g.dw;
                if (iw < 0 || iw >= g.w) continue;
                const int64_t pix = ((int64_t)b * g.h + ih) * g.w + iw;
                if (mask_in && !mask_in[pix]) continue;
                const TI *xp = x + pix * g.c_in;
                const TI *wp = wrow + (kh * g.kw + kw) * g.c_in;
                for (int ci = 0; ci < g.c_in; ++ci) acc = fmaf(to_float(xp[ci]), to_float(wp[ci]), acc);
            }
        }
        if (bias) acc += bias[co];
        if ((g.flags & FC_RELU) && !(acc > 0.f)) acc = (acc != acc) ? acc : 0.f;
        from_float(acc, &out[(int64_t)p * g.c_out + co]);
    }
}

template <typename TI, typename TO>
static hipError_t launch_t(const Geom &g, const void *x, const uint8_t *mask_in, const void *w,
                           const float *bias, const int32_t *idx, const int32_t *count, void *out,
                           hipStream_t s)
{
    // grid sized for the dense row count: the kept count is only known on the device
    const int64_t total = (int64_t)g.m * g.c_out;
    int blocks = (int)((total + 255) / 256 > 32768 ? 32768 : (total + 255) / 256);
    hipLaunchKernelGGL((k_conv_direct<TI, TO>), dim3(blocks), dim3(256), 0, s, g, (const TI *)x, mask_in,
                       (const TI *)w, bias, idx, count, (TO *)out);
    return hipGetLastError();
}

hipError_t launch_conv_direct(const Geom &g, int in_dtype, int out_dtype, const void *x,
                              const uint8_t *mask_in, const void *w, const float *bias, const int32_t *idx,
                              const int32_t *count, void *out, hipStream_t s)
{
    if (in_dtype == FC_F32) return launch_t<float, float>(g, x, mask_in, w, bias, idx, count, out, s);
    if (in_dtype == FC_BF16) {
        if (out_dtype == FC_F32) return launch_t<bf16_t, float>(g, x, mask_in, w, bias, idx, count, out, s);
        return launch_t<bf16_t, bf16_t>(g, x, mask_in, w, bias, idx, count, out, s);
    }
    if (out_dtype == FC_F32) return launch_t<f16_t, float>(g, x, mask_in, w, bias, idx, count, out, s);
    return launch_t<f16_t, f16_t>(g, x, mask_in, w, bias, idx, count, out, s);
}

} // namespace fc
