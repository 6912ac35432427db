/*
 * CPU oracle for the focused convolution (Tung et al., "Irrelevant Pixels are
 * Everywhere", Sec. III-A and III-B).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU
 * library can be checked against something that is slow, plain and easy to
 * compare with the paper by eye.  Nothing under the product package may call
 * it; only the tests, the smoke check and the benchmark's cpu_baseline leg do.
 * It shares no code, header, table or helper with the HIP path.
 *
 * What the method computes has a plain definition, so the oracle is that
 * definition written out, not a re-enactment of im2col:
 *
 *   - Sec. III-A: a patch labelled irrelevant is never turned into a column of
 *     the GEMM matrix, so no output feature is produced for it; every other
 *     patch is multiplied by the unchanged weights and gets the unchanged bias.
 *     With no mask the layer is the standard convolution.
 *   - Sec. III-B: the pixel mask is carried through the network by rescaling it
 *     to each layer's spatial size.
 *
 * Readings fixed where the paper is silent (listed with reasons in the design
 * document of this repository):
 *   - a patch's label is the mask value under the centre tap of its receptive
 *     field (nearest-neighbour rescaling of the mask, Sec. III-B; it is the
 *     only rule that keeps the kept fraction constant through the layers, as
 *     Table I's multiply-add ratios require);
 *   - a kept patch sees zero at input pixels the input mask marks irrelevant;
 *   - irrelevant output positions hold +0.0 in every channel, no bias;
 *   - output size is floor((H + 2p - d(K-1) - 1)/s) + 1 (the Fig. 5 caption's
 *     4x6 input / 3x3 kernel / stride 1 -> 8 columns fixes the "+1");
 *   - masks are one byte per pixel, per image, nonzero = relevant.
 *
 * Layouts: x[N][H][W][C_in], w[C_out][KH][KW][C_in], bias[C_out] (float),
 * masks uint8 [N][H][W], out double [N][Ho][Wo][C_out].  Inputs arrive already
 * rounded to their storage type (float32, bfloat16, IEEE half, or the 8-bit
 * E4M3 format, one byte per value); they are widened exactly and accumulated in double in the loop order
 * n, oh, ow, co, kh, kw, ci.  The result is left unrounded.
 *
 * The depthwise layer at the end of this file (one filter per channel, the
 * building block of the networks the paper evaluates in Sec. IV) follows the
 * same definition with the sum over input channels removed.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (figure counts, closed forms, hand-computed cases, an independently written
 * im2col+matmul, a library convolution, invariants).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { FCO_F32 = 0, FCO_BF16 = 1, FCO_F16 = 2, FCO_FP8 = 3 };

typedef struct {
    int32_t n, h, w, c_in, c_out, kh, kw;
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
    int32_t dtype; /* storage type of x and w */
    int32_t relu;  /* apply max(.,0) at kept positions */
} fco_conv;

/* ---- exact widening of the storage types ------------------------------- */

static double widen_f32(const void *p, size_t i) { return (double)((const float *)p)[i]; }

static double widen_bf16(const void *p, size_t i)
{
    /* bfloat16 is the upper half of a float32 */
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double widen_f16(const void *p, size_t i)
{
    uint16_t hbits = ((const uint16_t *)p)[i];
    int sign = hbits >> 15, e = (hbits >> 10) & 31, frac = hbits & 1023;
    double v;
    if (e == 0)
        v = (double)frac * (1.0 / 16777216.0); /* subnormal: frac * 2^-24 */
    else if (e == 31)
        v = frac ? (0.0 / 0.0) : (1.0 / 0.0);
    else {
        v = 1.0 + (double)frac / 1024.0;
        int k = e - 15;
        while (k > 0) { v *= 2.0; --k; }
        while (k < 0) { v *= 0.5; ++k; }
    }
    return sign ? -v : v;
}

/* 8-bit floating point, format E4M3 of the OCP 8-bit floating point specification
 * (the variant without infinities): 1 sign bit, 4 exponent bits with bias 7, 3
 * fraction bits.  Exponent field 0 holds the subnormals frac * 2^-9; exponent
 * field 15 holds ordinary numbers (up to 1.75 * 2^8 = 448) except fraction 7,
 * which is NaN. */
static double widen_fp8(const void *p, size_t i)
{
    uint8_t bits = ((const uint8_t *)p)[i];
    int sign = bits >> 7, e = (bits >> 3) & 15, frac = bits & 7;
    double v;
    if (e == 15 && frac == 7) return 0.0 / 0.0;
    if (e == 0)
        v = (double)frac / 512.0;
    else {
        v = 1.0 + (double)frac / 8.0;
        int k = e - 7;
        while (k > 0) { v *= 2.0; --k; }
        while (k < 0) { v *= 0.5; ++k; }
    }
    return sign ? -v : v;
}

/* one stored value, widened (lets the tests pin the decoders one by one) */
typedef double (*widen_fn)(const void *, size_t);

static widen_fn pick_widen(int dtype)
{
    return dtype == FCO_BF16 ? widen_bf16 : dtype == FCO_F16 ? widen_f16 : dtype == FCO_FP8 ? widen_fp8 : widen_f32;
}

/* out[i] = value of the i-th stored element */
int32_t fco_widen(int32_t dtype, const void *stored, int64_t count, double *out)
{
    if (dtype < FCO_F32 || dtype > FCO_FP8) return -1;
    widen_fn wd = pick_widen(dtype);
    for (int64_t i = 0; i < count; ++i) out[i] = wd(stored, (size_t)i);
    return 0;
}

/* The 8-bit code an output value is stored as when a layer writes FCO_FP8 (an extension
 * beyond the paper, which stores fp32): the nearest of the format's values, a tie going to
 * the code with the even fraction; magnitudes beyond the largest value (448) store that
 * value; NaN stores code 0x7F with the sign.  Written as the definition: the value's
 * binade fixes the spacing of the candidates, nearbyint (round-half-even in the default
 * rounding mode) picks among them. */
static uint8_t narrow_fp8(double v)
{
    uint8_t sign = signbit(v) ? 0x80 : 0x00;
    double a = fabs(v);
    if (isnan(v)) return (uint8_t)(sign | 0x7F);
    if (a >= 448.0) return (uint8_t)(sign | 0x7E);
    if (a < 1.0 / 64.0) /* subnormals and the first ordinary value: multiples of 2^-9, codes 0..8 */
        return (uint8_t)(sign | (uint8_t)nearbyint(a * 512.0));
    int e;
    double m = frexp(a, &e); /* a = m * 2^e, m in [0.5, 1) */
    int q = (int)nearbyint((2.0 * m - 1.0) * 8.0); /* eighths above 2^(e-1): 0..8 */
    int ex = e - 1;
    if (q == 8) { q = 0; ++ex; }
    return (uint8_t)(sign | ((ex + 7) << 3) | q);
}

/* codes[i] = the 8-bit code of values[i] */
int32_t fco_narrow_fp8(const double *values, int64_t count, uint8_t *codes)
{
    if (!values || !codes) return -1;
    for (int64_t i = 0; i < count; ++i) codes[i] = narrow_fp8(values[i]);
    return 0;
}

/* ---- output size (Sec. III-A operation count; Fig. 5 caption) ---------- */

int32_t fco_out_dim(int32_t in, int32_t k, int32_t stride, int32_t pad, int32_t dil)
{
    int32_t span = in + 2 * pad - dil * (k - 1) - 1;
    if (span < 0) return 0;
    return span / stride + 1;
}

/* threads the convolution loops will use (for the benchmark's report) */
int32_t fco_num_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

static int32_t clampi(int32_t v, int32_t lo, int32_t hi) { return v < lo ? lo : (v > hi ? hi : v); }

/* ---- mask propagation (Sec. III-B) -------------------------------------
 * The output-resolution mask takes, for each output position, the input mask
 * under the centre tap of that position's receptive field, clamped into the
 * image.  Output bytes are exactly 0 or 1.  Returns 0, or -1 on bad sizes. */
int32_t fco_mask_downsample(const uint8_t *mask_in, int32_t n, int32_t h, int32_t w,
                            int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                            int32_t ph, int32_t pw, int32_t dh, int32_t dw,
                            uint8_t *mask_out)
{
    int32_t ho = fco_out_dim(h, kh, sh, ph, dh), wo = fco_out_dim(w, kw, sw, pw, dw);
    if (n <= 0 || ho <= 0 || wo <= 0) return -1;
    for (int32_t b = 0; b < n; ++b)
        for (int32_t oh = 0; oh < ho; ++oh)
            for (int32_t ow = 0; ow < wo; ++ow) {
                int32_t ih = clampi(oh * sh - ph + dh * ((kh - 1) / 2), 0, h - 1);
                int32_t iw = clampi(ow * sw - pw + dw * ((kw - 1) / 2), 0, w - 1);
                uint8_t v = mask_in ? mask_in[((size_t)b * h + ih) * w + iw] : 1;
                mask_out[((size_t)b * ho + oh) * wo + ow] = v ? 1 : 0;
            }
    return 0;
}

/* ---- other ways to label a patch ---------------------------------------
 * Sec. III-A only says "a patch labelled irrelevant"; the reading used everywhere
 * else in this file is the centre tap (rule 0).  The two window rules are the other
 * readings of that sentence: rule 1 keeps a patch if ANY pixel of its window is
 * relevant, rule 2 only if ALL are.  Pixels outside the image are not part of the
 * window; a window with no pixel inside the image is irrelevant under both. */
int32_t fco_mask_downsample_rule(const uint8_t *mask_in, int32_t n, int32_t h, int32_t w,
                                 int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                                 int32_t ph, int32_t pw, int32_t dh, int32_t dw,
                                 int32_t rule, uint8_t *mask_out)
{
    if (rule == 0)
        return fco_mask_downsample(mask_in, n, h, w, kh, kw, sh, sw, ph, pw, dh, dw, mask_out);
    if (rule != 1 && rule != 2) return -3;
    int32_t ho = fco_out_dim(h, kh, sh, ph, dh), wo = fco_out_dim(w, kw, sw, pw, dw);
    if (n <= 0 || ho <= 0 || wo <= 0 || !mask_in) return -1;
    for (int32_t b = 0; b < n; ++b)
        for (int32_t oh = 0; oh < ho; ++oh)
            for (int32_t ow = 0; ow < wo; ++ow) {
                int32_t inside = 0, relevant = 0;
                for (int32_t i = 0; i < kh; ++i)
                    for (int32_t j = 0; j < kw; ++j) {
                        int32_t ih = oh * sh - ph + i * dh, iw = ow * sw - pw + j * dw;
                        if (ih < 0 || ih >= h || iw < 0 || iw >= w) continue;
                        ++inside;
                        if (mask_in[((size_t)b * h + ih) * w + iw]) ++relevant;
                    }
                uint8_t v = rule == 1 ? (relevant > 0) : (inside > 0 && relevant == inside);
                mask_out[((size_t)b * ho + oh) * wo + ow] = v;
            }
    return 0;
}

/* ---- which columns survive (Sec. III-A) --------------------------------
 * Ascending list of the flat positions whose mask byte is nonzero. */
int64_t fco_active_index_compact(const uint8_t *mask, int64_t m, int32_t *idx)
{
    int64_t j = 0;
    for (int64_t p = 0; p < m; ++p)
        if (mask[p]) idx[j++] = (int32_t)p;
    return j;
}

/* ---- one output position, all channels --------------------------------- */
static void conv_position(const fco_conv *c, widen_fn wd, const void *x, const uint8_t *mask_in,
                          const void *w, const float *bias, int32_t b, int32_t oh, int32_t ow,
                          double *out_row)
{
    int32_t ch = oh * c->stride_h - c->pad_h + c->dil_h * ((c->kh - 1) / 2);
    int32_t cw = ow * c->stride_w - c->pad_w + c->dil_w * ((c->kw - 1) / 2);
    ch = clampi(ch, 0, c->h - 1);
    cw = clampi(cw, 0, c->w - 1);
    if (mask_in && !mask_in[((size_t)b * c->h + ch) * c->w + cw]) {
        for (int32_t co = 0; co < c->c_out; ++co) out_row[co] = 0.0;
        return;
    }
    for (int32_t co = 0; co < c->c_out; ++co) {
        double acc = bias ? (double)bias[co] : 0.0;
        for (int32_t kh = 0; kh < c->kh; ++kh)
            for (int32_t kw = 0; kw < c->kw; ++kw) {
                int32_t ih = oh * c->stride_h - c->pad_h + kh * c->dil_h;
                int32_t iw = ow * c->stride_w - c->pad_w + kw * c->dil_w;
                if (ih < 0 || ih >= c->h || iw < 0 || iw >= c->w) continue; /* zero padding */
                size_t pix = ((size_t)b * c->h + ih) * c->w + iw;
                if (mask_in && !mask_in[pix]) continue; /* irrelevant input pixel counts as zero */
                size_t xo = pix * c->c_in;
                size_t wo = (((size_t)co * c->kh + kh) * c->kw + kw) * c->c_in;
                for (int32_t ci = 0; ci < c->c_in; ++ci)
                    acc += wd(x, xo + ci) * wd(w, wo + ci);
            }
        if (c->relu && acc < 0.0) acc = 0.0;
        out_row[co] = acc;
    }
}

/* ---- kept-position list in tile order -----------------------------------
 * Sec. III-A only says which patches become columns, not in which order; any
 * order gives the same features.  This order walks an image tile by tile
 * (tiles of tile_h x tile_w positions, row-major over the tiles, row-major
 * inside a tile), so that consecutive entries are neighbours in both
 * directions.  mask: [n][ho][wo] bytes.  Returns the count, or -1. */
int64_t fco_active_index_compact_tiled(const uint8_t *mask, int32_t n, int32_t ho, int32_t wo,
                                       int32_t tile_h, int32_t tile_w, int32_t *idx)
{
    if (n <= 0 || ho <= 0 || wo <= 0 || tile_h <= 0 || tile_w <= 0) return -1;
    int64_t count = 0;
    for (int32_t b = 0; b < n; ++b)
        for (int32_t y0 = 0; y0 < ho; y0 += tile_h)
            for (int32_t x0 = 0; x0 < wo; x0 += tile_w)
                for (int32_t y = y0; y < y0 + tile_h && y < ho; ++y)
                    for (int32_t x = x0; x < x0 + tile_w && x < wo; ++x) {
                        int64_t p = ((int64_t)b * ho + y) * wo + x;
                        if (mask[p]) idx[count++] = (int32_t)p;
                    }
    return count;
}

/* ---- the whole layer ----------------------------------------------------
 * out[N][Ho][Wo][C_out] in double.  mask_in NULL = every pixel relevant (the
 * standard convolution, Sec. III-A last paragraph).  bias NULL = no bias. */
int32_t fco_focused_conv2d(const fco_conv *c, const void *x, const uint8_t *mask_in,
                           const void *w, const float *bias, double *out)
{
    int32_t ho = fco_out_dim(c->h, c->kh, c->stride_h, c->pad_h, c->dil_h);
    int32_t wo = fco_out_dim(c->w, c->kw, c->stride_w, c->pad_w, c->dil_w);
    if (c->n <= 0 || ho <= 0 || wo <= 0 || c->c_in <= 0 || c->c_out <= 0) return -1;
    widen_fn wd = pick_widen(c->dtype);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int32_t b = 0; b < c->n; ++b)
        for (int32_t oh = 0; oh < ho; ++oh)
            for (int32_t ow = 0; ow < wo; ++ow)
                conv_position(c, wd, x, mask_in, w, bias, b, oh, ow,
                              out + (((size_t)b * ho + oh) * wo + ow) * c->c_out);
    return 0;
}

/* ---- the same definition at a list of flat output positions -------------
 * positions[j] = (b*Ho + oh)*Wo + ow; out[npos][C_out].  Lets large layers be
 * checked on a sample. */
int32_t fco_focused_conv2d_at(const fco_conv *c, const void *x, const uint8_t *mask_in,
                              const void *w, const float *bias, const int64_t *positions,
                              int64_t npos, double *out)
{
    int32_t ho = fco_out_dim(c->h, c->kh, c->stride_h, c->pad_h, c->dil_h);
    int32_t wo = fco_out_dim(c->w, c->kw, c->stride_w, c->pad_w, c->dil_w);
    if (c->n <= 0 || ho <= 0 || wo <= 0 || c->c_in <= 0 || c->c_out <= 0) return -1;
    int64_t m = (int64_t)c->n * ho * wo;
    for (int64_t j = 0; j < npos; ++j)
        if (positions[j] < 0 || positions[j] >= m) return -2;
    widen_fn wd = pick_widen(c->dtype);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t j = 0; j < npos; ++j) {
        int64_t p = positions[j];
        int32_t ow = (int32_t)(p % wo);
        int32_t oh = (int32_t)((p / wo) % ho);
        int32_t b = (int32_t)(p / ((int64_t)wo * ho));
        conv_position(c, wd, x, mask_in, w, bias, b, oh, ow, out + (size_t)j * c->c_out);
    }
    return 0;
}

/* ---- grouped layer --------------------------------------------------------
 * The layer type between the full layer and the depthwise one: the channels are
 * cut into `groups` equal slices, output slice g sees input slice g only.
 * Everything else is Sec. III-A unchanged (labels, zero at irrelevant inputs,
 * +0.0 at irrelevant positions).  Layouts: x[N][H][W][C_in],
 * w[C_out][KH][KW][C_in/groups], bias[C_out].  Returns -3 when the channel
 * counts are not multiples of groups. */
int32_t fco_focused_gconv2d(const fco_conv *c, int32_t groups, const void *x, const uint8_t *mask_in,
                            const void *w, const float *bias, double *out)
{
    int32_t ho = fco_out_dim(c->h, c->kh, c->stride_h, c->pad_h, c->dil_h);
    int32_t wo = fco_out_dim(c->w, c->kw, c->stride_w, c->pad_w, c->dil_w);
    if (c->n <= 0 || ho <= 0 || wo <= 0 || c->c_in <= 0 || c->c_out <= 0) return -1;
    if (groups <= 0 || c->c_in % groups || c->c_out % groups) return -3;
    int32_t cig = c->c_in / groups, cog = c->c_out / groups;
    widen_fn wd = pick_widen(c->dtype);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int32_t b = 0; b < c->n; ++b)
        for (int32_t oh = 0; oh < ho; ++oh)
            for (int32_t ow = 0; ow < wo; ++ow) {
                double *out_row = out + (((size_t)b * ho + oh) * wo + ow) * c->c_out;
                int32_t ch = clampi(oh * c->stride_h - c->pad_h + c->dil_h * ((c->kh - 1) / 2), 0, c->h - 1);
                int32_t cw = clampi(ow * c->stride_w - c->pad_w + c->dil_w * ((c->kw - 1) / 2), 0, c->w - 1);
                if (mask_in && !mask_in[((size_t)b * c->h + ch) * c->w + cw]) {
                    for (int32_t co = 0; co < c->c_out; ++co) out_row[co] = 0.0;
                    continue;
                }
                for (int32_t co = 0; co < c->c_out; ++co) {
                    int32_t g = co / cog; /* the slice this output channel belongs to */
                    double acc = bias ? (double)bias[co] : 0.0;
                    for (int32_t kh = 0; kh < c->kh; ++kh)
                        for (int32_t kw = 0; kw < c->kw; ++kw) {
                            int32_t ih = oh * c->stride_h - c->pad_h + kh * c->dil_h;
                            int32_t iw = ow * c->stride_w - c->pad_w + kw * c->dil_w;
                            if (ih < 0 || ih >= c->h || iw < 0 || iw >= c->w) continue;
                            size_t pix = ((size_t)b * c->h + ih) * c->w + iw;
                            if (mask_in && !mask_in[pix]) continue;
                            size_t xo = pix * c->c_in + (size_t)g * cig;
                            size_t wo_ = (((size_t)co * c->kh + kh) * c->kw + kw) * cig;
                            for (int32_t ci = 0; ci < cig; ++ci) acc += wd(x, xo + ci) * wd(w, wo_ + ci);
                        }
                    if (c->relu && acc < 0.0) acc = 0.0;
                    out_row[co] = acc;
                }
            }
    return 0;
}

/* ---- depthwise layer -----------------------------------------------------
 * Sec. IV replaces every convolutional layer of EfficientDet and SSD-Lite by
 * its focused form; most of those layers are depthwise: channel c of the
 * output sees channel c of the input only, through its own KH x KW filter.
 * Everything else is Sec. III-A unchanged: a position whose centre-tap mask
 * byte is zero produces no features (+0.0), a kept position sees zero at
 * irrelevant input pixels and outside the image.
 * Layouts: x[N][H][W][C], w[C][KH][KW], bias[C]; c_in must equal c_out.
 * Loop order n, oh, ow, c, kh, kw; double accumulation; result unrounded. */
static void dw_position(const fco_conv *c, widen_fn wd, const void *x, const uint8_t *mask_in,
                        const void *w, const float *bias, int32_t b, int32_t oh, int32_t ow,
                        double *out_row)
{
    int32_t ch = clampi(oh * c->stride_h - c->pad_h + c->dil_h * ((c->kh - 1) / 2), 0, c->h - 1);
    int32_t cw = clampi(ow * c->stride_w - c->pad_w + c->dil_w * ((c->kw - 1) / 2), 0, c->w - 1);
    if (mask_in && !mask_in[((size_t)b * c->h + ch) * c->w + cw]) {
        for (int32_t k = 0; k < c->c_out; ++k) out_row[k] = 0.0;
        return;
    }
    for (int32_t k = 0; k < c->c_out; ++k) {
        double acc = bias ? (double)bias[k] : 0.0;
        for (int32_t kh = 0; kh < c->kh; ++kh)
            for (int32_t kw = 0; kw < c->kw; ++kw) {
                int32_t ih = oh * c->stride_h - c->pad_h + kh * c->dil_h;
                int32_t iw = ow * c->stride_w - c->pad_w + kw * c->dil_w;
                if (ih < 0 || ih >= c->h || iw < 0 || iw >= c->w) continue;
                size_t pix = ((size_t)b * c->h + ih) * c->w + iw;
                if (mask_in && !mask_in[pix]) continue;
                acc += wd(x, pix * c->c_in + k) * wd(w, ((size_t)k * c->kh + kh) * c->kw + kw);
            }
        if (c->relu && acc < 0.0) acc = 0.0;
        out_row[k] = acc;
    }
}

int32_t fco_focused_dwconv2d(const fco_conv *c, const void *x, const uint8_t *mask_in,
                             const void *w, const float *bias, double *out)
{
    int32_t ho = fco_out_dim(c->h, c->kh, c->stride_h, c->pad_h, c->dil_h);
    int32_t wo = fco_out_dim(c->w, c->kw, c->stride_w, c->pad_w, c->dil_w);
    if (c->n <= 0 || ho <= 0 || wo <= 0 || c->c_in <= 0 || c->c_out != c->c_in) return -1;
    widen_fn wd = pick_widen(c->dtype);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int32_t b = 0; b < c->n; ++b)
        for (int32_t oh = 0; oh < ho; ++oh)
            for (int32_t ow = 0; ow < wo; ++ow)
                dw_position(c, wd, x, mask_in, w, bias, b, oh, ow,
                            out + (((size_t)b * ho + oh) * wo + ow) * c->c_out);
    return 0;
}

int32_t fco_focused_dwconv2d_at(const fco_conv *c, const void *x, const uint8_t *mask_in,
                                const void *w, const float *bias, const int64_t *positions,
                                int64_t npos, double *out)
{
    int32_t ho = fco_out_dim(c->h, c->kh, c->stride_h, c->pad_h, c->dil_h);
    int32_t wo = fco_out_dim(c->w, c->kw, c->stride_w, c->pad_w, c->dil_w);
    if (c->n <= 0 || ho <= 0 || wo <= 0 || c->c_in <= 0 || c->c_out != c->c_in) return -1;
    int64_t m = (int64_t)c->n * ho * wo;
    for (int64_t j = 0; j < npos; ++j)
        if (positions[j] < 0 || positions[j] >= m) return -2;
    widen_fn wd = pick_widen(c->dtype);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t j = 0; j < npos; ++j) {
        int64_t p = positions[j];
        int32_t ow = (int32_t)(p % wo);
        int32_t oh = (int32_t)((p / wo) % ho);
        int32_t b = (int32_t)(p / ((int64_t)wo * ho));
        dw_position(c, wd, x, mask_in, w, bias, b, oh, ow, out + (size_t)j * c->c_out);
    }
    return 0;
}

/* ---- the layer with the labels given --------------------------------------
 * labels[N][Ho][Wo] (nonzero = kept) say which patches become columns, however
 * they were obtained (fco_mask_downsample_rule); a kept patch still sees zero at
 * pixels the input mask marks irrelevant and outside the image.  Same loops and
 * arithmetic as fco_focused_conv2d. */
int32_t fco_focused_conv2d_labelled(const fco_conv *c, const void *x, const uint8_t *mask_in,
                                    const uint8_t *labels, const void *w, const float *bias,
                                    double *out)
{
    int32_t ho = fco_out_dim(c->h, c->kh, c->stride_h, c->pad_h, c->dil_h);
    int32_t wo = fco_out_dim(c->w, c->kw, c->stride_w, c->pad_w, c->dil_w);
    if (c->n <= 0 || ho <= 0 || wo <= 0 || c->c_in <= 0 || c->c_out <= 0 || !labels) return -1;
    widen_fn wd = pick_widen(c->dtype);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int32_t b = 0; b < c->n; ++b)
        for (int32_t oh = 0; oh < ho; ++oh)
            for (int32_t ow = 0; ow < wo; ++ow) {
                size_t p = ((size_t)b * ho + oh) * wo + ow;
                double *out_row = out + p * c->c_out;
                for (int32_t co = 0; co < c->c_out; ++co) {
                    if (!labels[p]) { out_row[co] = 0.0; continue; }
                    double acc = bias ? (double)bias[co] : 0.0;
                    for (int32_t kh = 0; kh < c->kh; ++kh)
                        for (int32_t kw = 0; kw < c->kw; ++kw) {
                            int32_t ih = oh * c->stride_h - c->pad_h + kh * c->dil_h;
                            int32_t iw = ow * c->stride_w - c->pad_w + kw * c->dil_w;
                            if (ih < 0 || ih >= c->h || iw < 0 || iw >= c->w) continue;
                            size_t pix = ((size_t)b * c->h + ih) * c->w + iw;
                            if (mask_in && !mask_in[pix]) continue;
                            for (int32_t ci = 0; ci < c->c_in; ++ci)
                                acc += wd(x, pix * c->c_in + ci) *
                                       wd(w, (((size_t)co * c->kh + kh) * c->kw + kw) * c->c_in + ci);
                        }
                    if (c->relu && acc < 0.0) acc = 0.0;
                    out_row[co] = acc;
                }
            }
    return 0;
}
