// C ABI of the library: argument checks on the host, then launches.
#include "fc_internal.hpp"
#include <atomic>

using namespace fc;

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t dtype_bytes(int32_t dt) { return dt == FC_F32 ? 4 : (dt == FC_FP8 ? 1 : 2); }

// [x, x + x_bytes) and [out, out + out_bytes) share a byte?
bool ranges_overlap(const void *x, size_t x_bytes, const void *out, size_t out_bytes)
{
    const uintptr_t a = reinterpret_cast<uintptr_t>(x), b = reinterpret_cast<uintptr_t>(out);
    return a < b + out_bytes && b < a + x_bytes;
}

// input and output tensor of a layer (rows in list order count as full tensors: capacity)
bool conv_tensors_overlap(const Geom &g, const fc_conv_desc *d, const void *x, const void *out)
{
    const size_t xb = (size_t)g.n * g.h * g.w * g.c_in * dtype_bytes(d->in_dtype);
    const size_t ob = (size_t)g.m * g.c_out * dtype_bytes(d->out_dtype);
    return ranges_overlap(x, xb, out, ob);
}

int32_t out_dim(int32_t in, int32_t k, int32_t s, int32_t p, int32_t d)
{
    const int64_t span = (int64_t)in + 2 * (int64_t)p - (int64_t)d * (k - 1) - 1;
    if (span < 0) return 0;
    return (int32_t)(span / s + 1);
}

// Validates the descriptor and fills the kernel geometry.
int32_t make_geom(const fc_conv_desc *d, Geom *g)
{
    if (!d) return FC_ERR_NULL;
    if (d->n <= 0 || d->h <= 0 || d->w <= 0 || d->c_in <= 0 || d->c_out <= 0 || d->kh <= 0 || d->kw <= 0 ||
        d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0 || d->dil_h <= 0 || d->dil_w <= 0)
        return FC_ERR_SHAPE;
    if (d->in_dtype != FC_F32 && d->in_dtype != FC_BF16 && d->in_dtype != FC_F16 && d->in_dtype != FC_FP8)
        return FC_ERR_DTYPE;
    // 8-bit inputs round to bfloat16 (or stay fp32); every other type to itself or fp32; all but
    // fp32 storage can also round to 8 bits
    if (d->out_dtype != (d->in_dtype == FC_FP8 ? FC_BF16 : d->in_dtype) && d->out_dtype != FC_F32 &&
        !(d->in_dtype != FC_F32 && d->out_dtype == FC_FP8))
        return FC_ERR_DTYPE;
    if (d->flags & ~(uint32_t)(FC_RELU | FC_SKIP_ZERO_FILL | FC_WORKSPACE_READY | FC_COMPACT_OUT | FC_COMPACT_IN |
                               FC_PACKED_MASKS | FC_RESIDENT_WEIGHTS))
        return FC_ERR_DTYPE;
    const int32_t ho = out_dim(d->h, d->kh, d->stride_h, d->pad_h, d->dil_h);
    const int32_t wo = out_dim(d->w, d->kw, d->stride_w, d->pad_w, d->dil_w);
    if (ho <= 0 || wo <= 0) return FC_ERR_SHAPE;
    const int64_t m = (int64_t)d->n * ho * wo, pix = (int64_t)d->n * d->h * d->w;
    if (m >= INT32_MAX || pix >= INT32_MAX) return FC_ERR_RANGE;
    if ((int64_t)d->kh * d->kw * d->c_in >= INT32_MAX) return FC_ERR_RANGE;
    g->n = d->n; g->h = d->h; g->w = d->w; g->c_in = d->c_in; g->c_out = d->c_out;
    g->kh = d->kh; g->kw = d->kw; g->sh = d->stride_h; g->sw = d->stride_w;
    g->ph = d->pad_h; g->pw = d->pad_w; g->dh = d->dil_h; g->dw = d->dil_w;
    g->ho = ho; g->wo = wo; g->m = (int32_t)m; g->flags = d->flags;
    return FC_OK;
}

// Does the one-workgroup-per-CU kernel serve this layer?  Focused 3x3 layers of 65 .. 128 output
// channels whose kept rows come to at most one tile per CU (eight 32-row blocks on each of 256
// CUs) and whose irrelevant rows are left unwritten (FC_SKIP_ZERO_FILL: a layer inside a chain).
// There it deals the kept rows out evenly, one round whatever the kept count (12 % faster than the
// tiled kernel at a kept share of one half).  With the zero-fill in the launch the tiled kernel
// stays: its idle workgroups clear rows beside the tiles, while a launch that keeps every CU
// busy can only clear them after its tiles (measured: no gain at one half, slower elsewhere).
// Layers small enough to rank their rows inside the tiled kernel stay there as well, whether
// or not the caller brings a list (one kernel, one summation order per layer).
bool conv_line_wanted(const Geom &g, int in_dtype, int out_dtype, bool focused)
{
    if (!focused || !(g.flags & FC_SKIP_ZERO_FILL) || !conv_line_supported(g, in_dtype, out_dtype)) return false;
    if (g.m <= kInlineRankPositions) return false;
    if (g.c_out <= 64 || g.c_out > 128) return false;
    return (int64_t)(g.m + 31) / 32 <= 8 * 256;
}

// 3x3 layers of 128-byte pixels (64 16-bit channels) into at most 64 channels (the first stage of ResNet-18/34 and the 3x3
// of a ResNet-50's first stage, VGG's conv1_2): the nine taps' weights (72 KB) stay in LDS and
// every wave runs its own pipeline, against 128-row tiles that stage the weights again for every
// tile.  Measured against the tiled kernel at 48 % irrelevant pixels on 50 000 .. 2.5 M
// positions: without a mask 12 .. 25 % faster up to 0.6 M positions (6 % slower at 2.5 M);
// chained (no zero-fill) equal at 50 000, 1 .. 17 % faster from 100 000 on; with zero-fill 4 .. 7 %
// slower up to 0.4 M (the zero-fill comes after a wave's units instead of between tiles), 16 %
// faster at 0.6 M, equal at 2.5 M.  Into 128 channels the tiled kernels win or draw.  128 8-bit
// channels into 64 follow the same pattern (0.6 M positions: 25 .. 28 % faster in all three modes).
static bool conv_pw_wanted_3x3(const Geom &g, bool masked)
{
    if (g.c_out > 64) return false;
    if (!masked) return g.m >= 40000 && g.m < 1500000;
    if (g.flags & (FC_SKIP_ZERO_FILL | FC_COMPACT_OUT)) return g.m >= 80000;
    return g.m >= 500000 && g.m < 2000000;
}

// Does the resident-weights kernel serve this layer?  1x1 layers without padding whose rows are whole
// 16-byte pieces on both sides and whose weights, cut into slices of 64 .. 256 output channels,
// stay in LDS (see fc_conv_pw.hip), with the kept list at hand or no mask at all (3x3 layers:
// the rule above; FC_RESIDENT_WEIGHTS: every layer the kernel supports).  In such a
// layer every labelling rule reduces to the one pixel under the tap, so a kept row never has a
// gated tap and the kernel reads no input mask while it gathers.  Measured against the tiled
// kernel on the 1x1 layers of a ResNet-50 (batch 32, 16-bit and 8-bit storage) and of a
// MobileNetV2 (batch 256): 10 .. 45 % faster, except (a) 16-bit rows of four 128-byte chunks
// into at most 128 output channels on the largest activations (256 -> 64, 256 -> 128: bound by
// reading them, 5 .. 15 % slower) and (b) three or more chunks into a single slice on fewer than
// 100 000 positions (24 .. 88 KB of weights per workgroup for a few rows each: up to 20 %
// slower).  Those stay on the tiled kernel.
bool conv_pw_wanted(const Geom &g, int in_dtype, int out_dtype, bool masked)
{
    if (g.m <= kInlineRankPositions || !conv_pw_supported(g, in_dtype, out_dtype)) return false;
    if (g.flags & FC_RESIDENT_WEIGHTS) return true; // the caller's choice
    if (g.kh == 3) return conv_pw_wanted_3x3(g, masked);
    const int kch = (g.c_in * (in_dtype == FC_FP8 ? 1 : 2) + 127) / 128; // 128-byte chunks of an input row
    if (in_dtype != FC_FP8 && kch == 4 && g.c_out <= 128) return false;
    if (kch >= 3 && g.c_out <= (kch > 4 ? 64 : 128) && g.m < 100000) return false;
    return true;
}

size_t compact_ws(int64_t m) { return align_up((size_t)compact_blocks(m) * sizeof(int32_t), 256); }

static_assert(kSplitGrid * sizeof(int32_t) == FC_WORKSPACE_COUNTER_BYTES, "the header promises this size");
struct ConvWorkspace {
    size_t counters, partials, mask_out, idx, count, scan, total, split_only;
};

// [tile counters | fp32 partial tiles] (split-K; empty for layers with many tiles), then
// [mask_out | idx | count | per-block counts] (only used when the call builds the list).
ConvWorkspace conv_ws_layout(const Geom &g)
{
    const int64_t m = g.m;
    ConvWorkspace l;
    l.counters = 0;
    l.partials = split_k_counter_bytes(g);
    l.split_only = l.partials + split_k_partial_bytes(g);
    l.mask_out = l.split_only;
    l.idx = l.mask_out + align_up((size_t)m, 256);
    l.count = l.idx + align_up((size_t)m * sizeof(int32_t), 256);
    l.scan = l.count + 256;
    l.total = l.scan + compact_ws(m);
    return l;
}

} // namespace

extern "C" {

const char *fc_status_string(int32_t status)
{
    switch (status) {
    case FC_OK: return "FC_OK";
    case FC_ERR_NULL: return "FC_ERR_NULL: a required pointer is NULL";
    case FC_ERR_SHAPE: return "FC_ERR_SHAPE: a size is not positive or the output is empty";
    case FC_ERR_DTYPE: return "FC_ERR_DTYPE: unsupported type or flag combination";
    case FC_ERR_ALIGN: return "FC_ERR_ALIGN: a device pointer is not 16-byte aligned";
    case FC_ERR_WORKSPACE: return "FC_ERR_WORKSPACE: workspace missing or too small";
    case FC_ERR_RANGE: return "FC_ERR_RANGE: position count does not fit 31 bits";
    case FC_ERR_HIP: return "FC_ERR_HIP: the HIP runtime refused a launch";
    default: return "unknown fc_status";
    }
}

int32_t fc_out_dims(const fc_conv_desc *desc, int32_t *ho, int32_t *wo)
{
    if (!desc || !ho || !wo) return FC_ERR_NULL;
    Geom g;
    const int32_t rc = make_geom(desc, &g);
    if (rc != FC_OK) return rc;
    *ho = g.ho;
    *wo = g.wo;
    return FC_OK;
}

int32_t fc_compact_workspace_bytes(int64_t m, size_t *bytes)
{
    if (!bytes) return FC_ERR_NULL;
    if (m <= 0) return FC_ERR_SHAPE;
    if (m >= INT32_MAX) return FC_ERR_RANGE;
    *bytes = compact_ws(m);
    return FC_OK;
}

int32_t fc_workspace_bytes(const fc_conv_desc *desc, size_t *bytes)
{
    if (!desc || !bytes) return FC_ERR_NULL;
    Geom g;
    const int32_t rc = make_geom(desc, &g);
    if (rc != FC_OK) return rc;
    *bytes = conv_ws_layout(g).total;
    return FC_OK;
}

int32_t fc_mask_downsample(const uint8_t *mask_in, int32_t n, int32_t h, int32_t w, int32_t kh, int32_t kw,
                           int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t dil_h,
                           int32_t dil_w, uint8_t *mask_out, void *stream)
{
    if (!mask_in || !mask_out) return FC_ERR_NULL;
    if (n <= 0 || h <= 0 || w <= 0 || kh <= 0 || kw <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 ||
        pad_w < 0 || dil_h <= 0 || dil_w <= 0)
        return FC_ERR_SHAPE;
    const int32_t ho = out_dim(h, kh, stride_h, pad_h, dil_h), wo = out_dim(w, kw, stride_w, pad_w, dil_w);
    if (ho <= 0 || wo <= 0) return FC_ERR_SHAPE;
    if ((int64_t)n * ho * wo >= INT32_MAX || (int64_t)n * h * w >= INT32_MAX) return FC_ERR_RANGE;
    const hipError_t e = launch_mask_downsample(mask_in, n, h, w, kh, kw, stride_h, stride_w, pad_h, pad_w,
                                                dil_h, dil_w, ho, wo, mask_out, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : FC_ERR_HIP;
}

int32_t fc_mask_downsample_rule(const uint8_t *mask_in, int32_t n, int32_t h, int32_t w, int32_t kh, int32_t kw,
                                int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t dil_h,
                                int32_t dil_w, int32_t rule, uint8_t *mask_out, void *stream)
{
    if (rule == FC_RULE_CENTRE)
        return fc_mask_downsample(mask_in, n, h, w, kh, kw, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, mask_out,
                                  stream);
    if (rule != FC_RULE_ANY && rule != FC_RULE_ALL) return FC_ERR_DTYPE;
    if (!mask_in || !mask_out) return FC_ERR_NULL;
    if (n <= 0 || h <= 0 || w <= 0 || kh <= 0 || kw <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 ||
        pad_w < 0 || dil_h <= 0 || dil_w <= 0)
        return FC_ERR_SHAPE;
    const int32_t ho = out_dim(h, kh, stride_h, pad_h, dil_h), wo = out_dim(w, kw, stride_w, pad_w, dil_w);
    if (ho <= 0 || wo <= 0) return FC_ERR_SHAPE;
    if ((int64_t)n * ho * wo >= INT32_MAX || (int64_t)n * h * w >= INT32_MAX) return FC_ERR_RANGE;
    const hipError_t e = launch_mask_window(mask_in, n, h, w, kh, kw, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                                            ho, wo, rule == FC_RULE_ALL, mask_out, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : FC_ERR_HIP;
}

int32_t fc_active_index_compact(const uint8_t *mask, int64_t m, int32_t *idx, int32_t *count, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    if (!mask || !idx || !count) return FC_ERR_NULL;
    if (m <= 0) return FC_ERR_SHAPE;
    if (m >= INT32_MAX) return FC_ERR_RANGE;
    if (!workspace || workspace_bytes < compact_ws(m)) return FC_ERR_WORKSPACE;
    if (!aligned16(mask) || !aligned16(idx) || !aligned16(workspace)) return FC_ERR_ALIGN;
    // a flat mask is a 1 x 1 x m image seen through a 1x1 stride-1 window
    MaskGeom g = mask_geom(1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1, 1, 1);
    g.w = g.wo = (int32_t)m;
    g.m = m;
    const hipError_t e =
        launch_compact(g, mask, nullptr, idx, count, (int32_t *)workspace, CompactExtras(), (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : FC_ERR_HIP;
}

static int32_t tiled_check(int32_t n, int32_t ho, int32_t wo, int32_t tile_h, int32_t tile_w, int64_t *rows)
{
    if (n <= 0 || ho <= 0 || wo <= 0 || tile_h <= 0 || tile_w <= 0 || tile_w > kMaxListTileWidth) return FC_ERR_SHAPE;
    if ((int64_t)n * ho * wo >= INT32_MAX) return FC_ERR_RANGE;
    if (tile_h > ho) tile_h = ho; // (a taller tile is the same order)
    *rows = tiled_rows(n, ho, wo, tile_h, tile_w);
    if (*rows >= INT32_MAX) return FC_ERR_RANGE;
    return FC_OK;
}

int32_t fc_compact_tiled_workspace_bytes(int32_t n, int32_t ho, int32_t wo, int32_t tile_h, int32_t tile_w,
                                         size_t *bytes)
{
    if (!bytes) return FC_ERR_NULL;
    int64_t rows;
    const int32_t rc = tiled_check(n, ho, wo, tile_h, tile_w, &rows);
    if (rc != FC_OK) return rc;
    *bytes = align_up((size_t)((rows + kCompactBlockThreads - 1) / kCompactBlockThreads) * sizeof(int32_t), 256);
    return FC_OK;
}

int32_t fc_active_index_compact_tiled(const uint8_t *mask, int32_t n, int32_t ho, int32_t wo, int32_t tile_h,
                                      int32_t tile_w, int32_t *idx, int32_t *count, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    if (!mask || !idx || !count) return FC_ERR_NULL;
    int64_t rows;
    const int32_t rc = tiled_check(n, ho, wo, tile_h, tile_w, &rows);
    if (rc != FC_OK) return rc;
    if (tile_h > ho) tile_h = ho;
    const size_t need = align_up((size_t)((rows + kCompactBlockThreads - 1) / kCompactBlockThreads) * sizeof(int32_t), 256);
    if (!workspace || workspace_bytes < need) return FC_ERR_WORKSPACE;
    if (!aligned16(idx) || !aligned16(workspace)) return FC_ERR_ALIGN;
    const hipError_t e = launch_compact_tiled(mask, n, ho, wo, tile_h, tile_w, idx, count, (int32_t *)workspace,
                                              (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : FC_ERR_HIP;
}

int32_t fc_focused_conv2d(const fc_conv_desc *desc, const void *x, const uint8_t *mask_in, const void *w,
                          const float *bias, const uint8_t *mask_out, const int32_t *idx, const int32_t *count,
                          void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    Geom g;
    const int32_t rc = make_geom(desc, &g);
    if (rc != FC_OK) return rc;
    if (!x || !w || !out) return FC_ERR_NULL;
    if ((idx == nullptr) != (count == nullptr)) return FC_ERR_NULL;
    if (!mask_in && (idx || mask_out)) return FC_ERR_NULL; // a kept list without the mask that gates the taps
    if (!aligned16(x) || !aligned16(w) || !aligned16(out) || !aligned16(idx) || !aligned16(bias)) return FC_ERR_ALIGN;
    if (conv_tensors_overlap(g, desc, x, out)) return FC_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;

    const bool mfma = conv_mfma_supported(g, desc->in_dtype, desc->out_dtype);
    const bool packed = (g.flags & FC_PACKED_MASKS) != 0;
    // the kernel for RGB stems reads byte masks image by image
    if (packed && !mfma && conv_stem_supported(g, desc->in_dtype, desc->out_dtype)) return FC_ERR_DTYPE;
    // 8-bit layers exist on the matrix cores only (16 | c_in, 8 | c_out, at most 32 taps)
    if (desc->in_dtype == FC_FP8 && !mfma) return FC_ERR_DTYPE;
    // 8-bit outputs: the matrix-core kernels round to them, the direct kernel does not
    if (desc->out_dtype == FC_FP8 && !mfma && !conv_stem_supported(g, desc->in_dtype, desc->out_dtype))
        return FC_ERR_DTYPE;
    if (g.flags & (FC_COMPACT_OUT | FC_COMPACT_IN)) {
        // compacted activations: rows in list order, so the list must be given
        if (!idx) return FC_ERR_NULL;
        if (!mfma) return FC_ERR_DTYPE;
        if ((g.flags & FC_COMPACT_IN) &&
            !(g.kh == 1 && g.kw == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0))
            return FC_ERR_SHAPE;
        if (g.flags & FC_COMPACT_OUT) g.flags |= FC_SKIP_ZERO_FILL; // there are no irrelevant rows to clear
    }
    const ConvWorkspace l = conv_ws_layout(g);
    // split-K scratch of the matrix-core path, when the layer is small enough to want it and
    // the caller gave room
    float *partials = nullptr;
    int32_t *tile_counters = nullptr;
    if (mfma && split_k_possible(g) && workspace && workspace_bytes >= l.split_only && aligned16(workspace)) {
        tile_counters = (int32_t *)((uint8_t *)workspace + l.counters);
        partials = (float *)((uint8_t *)workspace + l.partials);
    }
    bool counters_cleared = false;

    if (mask_in && !idx) {
        // derive mask_out, the index list and its length here, in the workspace
        if (!workspace || workspace_bytes < l.total) return FC_ERR_WORKSPACE;
        if (!aligned16(workspace)) return FC_ERR_ALIGN;
        uint8_t *ws = (uint8_t *)workspace;
        uint8_t *m_out = ws + l.mask_out;
        const MaskGeom mg = mask_geom(g.n, g.h, g.w, g.kh, g.kw, g.sh, g.sw, g.ph, g.pw, g.dh, g.dw, g.ho, g.wo);
        // a small layer on the matrix-core path ranks its kept positions inside the convolution
        // kernel (16 positions per thread, labels from the centre tap): no compaction launch.
        // Labels the caller brings (mask_out without a list) are compacted as they are, so that
        // the rows computed and the rows cleared follow the same labels.
        const bool rank_in_kernel = mfma && g.m <= kInlineRankPositions && !mask_out;
        if (!rank_in_kernel) {
            CompactExtras ex;
            if (tile_counters) {
                ex.zero = tile_counters;
                ex.zero_n = kSplitGrid;
                counters_cleared = true;
            }
            hipError_t ec;
            if (mask_out) {
                // a flat mask is a 1 x 1 x m image seen through a 1x1 stride-1 window
                MaskGeom fg = mask_geom(1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1, 1, 1);
                fg.w = fg.wo = g.m;
                fg.m = g.m;
                fg.packed_in = packed;
                ec = launch_compact(fg, mask_out, nullptr, (int32_t *)(ws + l.idx), (int32_t *)(ws + l.count),
                                    (int32_t *)(ws + l.scan), ex, s);
            } else {
                MaskGeom pg = mg;
                pg.packed_in = pg.packed_out = packed; // the derived labels take the form of the input mask
                ec = launch_compact(pg, mask_in, m_out, (int32_t *)(ws + l.idx), (int32_t *)(ws + l.count),
                                    (int32_t *)(ws + l.scan), ex, s);
                mask_out = m_out;
            }
            if (ec != hipSuccess) return FC_ERR_HIP;
            idx = (const int32_t *)(ws + l.idx);
            count = (const int32_t *)(ws + l.count);
        }
    }

    hipError_t e;
    const bool pw = mfma && (idx || !mask_in) && conv_pw_wanted(g, desc->in_dtype, desc->out_dtype, mask_in != nullptr);
    if (mfma && idx && !(pw && (g.flags & FC_RESIDENT_WEIGHTS)) &&
        conv_line_wanted(g, desc->in_dtype, desc->out_dtype, mask_in != nullptr)) {
        e = launch_conv_line(g, desc->in_dtype, desc->out_dtype, x, mask_in, mask_out, w, bias, idx, count, out, s);
        if (e != hipSuccess) return FC_ERR_HIP;
    } else if (pw) {
        e = launch_conv_pw(g, desc->in_dtype, desc->out_dtype, x, mask_in, mask_out, w, bias, idx, count, out, s);
        if (e != hipSuccess) return FC_ERR_HIP;
    } else if (mfma) {
        if (tile_counters && !counters_cleared && !(g.flags & FC_WORKSPACE_READY)) {
            e = launch_zero_i32(tile_counters, kSplitGrid, s);
            if (e != hipSuccess) return FC_ERR_HIP;
        }
        // gather + matrix cores + epilogue + zero-fill in one kernel
        e = launch_conv_mfma(g, desc->in_dtype, desc->out_dtype, x, mask_in, mask_out, w, bias, idx, count, out,
                             partials, tile_counters, s);
        if (e != hipSuccess) return FC_ERR_HIP;
    } else {
        if (conv_stem_supported(g, desc->in_dtype, desc->out_dtype))
            e = launch_conv_stem(g, desc->in_dtype, desc->out_dtype, x, mask_in, w, bias, idx, count, out, s);
        else
            e = launch_conv_direct(g, desc->in_dtype, desc->out_dtype, x, mask_in, w, bias, idx, count, out, s);
        if (e != hipSuccess) return FC_ERR_HIP;
        if (mask_in && !(g.flags & FC_SKIP_ZERO_FILL)) {
            e = launch_zero_fill(g, mask_in, mask_out, out, desc->out_dtype, s);
            if (e != hipSuccess) return FC_ERR_HIP;
        }
    }
    return FC_OK;
}

int32_t fc_focused_gconv2d(const fc_conv_desc *desc, int32_t groups, const void *x, const uint8_t *mask_in,
                           const void *w, const float *bias, const uint8_t *mask_out, const int32_t *idx,
                           const int32_t *count, void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (groups == 1)
        return fc_focused_conv2d(desc, x, mask_in, w, bias, mask_out, idx, count, out, workspace, workspace_bytes,
                                 stream);
    Geom g;
    const int32_t rc = make_geom(desc, &g);
    if (rc != FC_OK) return rc;
    if (groups <= 0 || g.c_in % groups != 0 || g.c_out % groups != 0) return FC_ERR_SHAPE;
    if (g.flags & (FC_COMPACT_OUT | FC_COMPACT_IN)) return FC_ERR_DTYPE; // full layers only
    // one channel per group with the labels of the input mask: the depthwise kernel
    if (groups == g.c_in && g.c_in == g.c_out && !idx && !mask_out)
        return fc_focused_dwconv2d(desc, x, mask_in, w, bias, out, stream);
    if (groups == g.c_in && (g.flags & FC_PACKED_MASKS)) return FC_ERR_DTYPE; // (depthwise: byte masks)
    if (desc->in_dtype == FC_FP8 || desc->out_dtype == FC_FP8) return FC_ERR_DTYPE;
    if (!x || !w || !out) return FC_ERR_NULL;
    if ((idx == nullptr) != (count == nullptr)) return FC_ERR_NULL;
    if (!mask_in && (idx || mask_out)) return FC_ERR_NULL;
    if (!aligned16(x) || !aligned16(w) || !aligned16(out) || !aligned16(idx) || !aligned16(bias)) return FC_ERR_ALIGN;
    if (conv_tensors_overlap(g, desc, x, out)) return FC_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (mask_in && !idx) {
        const ConvWorkspace l = conv_ws_layout(g);
        if (!workspace || workspace_bytes < l.total) return FC_ERR_WORKSPACE;
        if (!aligned16(workspace)) return FC_ERR_ALIGN;
        uint8_t *ws = (uint8_t *)workspace;
        const MaskGeom mg = mask_geom(g.n, g.h, g.w, g.kh, g.kw, g.sh, g.sw, g.ph, g.pw, g.dh, g.dw, g.ho, g.wo);
        hipError_t ec;
        const bool packed = (g.flags & FC_PACKED_MASKS) != 0;
        if (mask_out) { // the caller's labels, compacted as they are
            MaskGeom fg = mask_geom(1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1, 1, 1);
            fg.w = fg.wo = g.m;
            fg.m = g.m;
            fg.packed_in = packed;
            ec = launch_compact(fg, mask_out, nullptr, (int32_t *)(ws + l.idx), (int32_t *)(ws + l.count),
                                (int32_t *)(ws + l.scan), CompactExtras(), s);
        } else {
            MaskGeom pg = mg;
            pg.packed_in = pg.packed_out = packed;
            ec = launch_compact(pg, mask_in, ws + l.mask_out, (int32_t *)(ws + l.idx), (int32_t *)(ws + l.count),
                                (int32_t *)(ws + l.scan), CompactExtras(), s);
            mask_out = ws + l.mask_out;
        }
        if (ec != hipSuccess) return FC_ERR_HIP;
        idx = (const int32_t *)(ws + l.idx);
        count = (const int32_t *)(ws + l.count);
    }
    Geom one = g; // the geometry of one group
    one.c_in = g.c_in / groups;
    one.c_out = g.c_out / groups;
    hipError_t e = launch_conv_direct(one, desc->in_dtype, desc->out_dtype, x, mask_in, w, bias, idx, count, out, s,
                                      groups);
    if (e != hipSuccess) return FC_ERR_HIP;
    if (mask_in && !(g.flags & FC_SKIP_ZERO_FILL)) {
        e = launch_zero_fill(g, mask_in, mask_out, out, desc->out_dtype, s);
        if (e != hipSuccess) return FC_ERR_HIP;
    }
    return FC_OK;
}

int32_t fc_expand_group_weights(int32_t c_in, int32_t c_out, int32_t kh, int32_t kw, int32_t groups, int32_t dtype,
                                const void *w_grouped, void *w_full, void *stream)
{
    if (!w_grouped || !w_full) return FC_ERR_NULL;
    if (c_in <= 0 || c_out <= 0 || kh <= 0 || kw <= 0 || groups <= 0 || c_in % groups != 0 || c_out % groups != 0)
        return FC_ERR_SHAPE;
    if (dtype != FC_F32 && dtype != FC_BF16 && dtype != FC_F16 && dtype != FC_FP8) return FC_ERR_DTYPE;
    if ((int64_t)c_out * kh * kw * c_in >= INT32_MAX) return FC_ERR_RANGE;
    const int esize = dtype == FC_F32 ? 4 : (dtype == FC_FP8 ? 1 : 2);
    const hipError_t e =
        launch_expand_group_weights(w_grouped, c_in, c_out, kh * kw, groups, esize, w_full, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : FC_ERR_HIP;
}

int32_t fc_focused_dwconv2d(const fc_conv_desc *desc, const void *x, const uint8_t *mask_in, const void *w,
                            const float *bias, void *out, void *stream)
{
    Geom g;
    const int32_t rc = make_geom(desc, &g);
    if (rc != FC_OK) return rc;
    if (g.c_in != g.c_out) return FC_ERR_SHAPE;
    if (g.flags & (FC_COMPACT_OUT | FC_COMPACT_IN | FC_PACKED_MASKS)) return FC_ERR_DTYPE; // full layers, byte masks
    if (!x || !w || !out) return FC_ERR_NULL;
    if (!aligned16(x) || !aligned16(w) || !aligned16(out) || !aligned16(bias)) return FC_ERR_ALIGN;
    if (conv_tensors_overlap(g, desc, x, out)) return FC_ERR_NULL;
    if (desc->in_dtype == FC_FP8 || desc->out_dtype == FC_FP8) return FC_ERR_DTYPE; // no 8-bit depthwise layer
    if (!conv_depthwise_supported(g, desc->in_dtype)) return FC_ERR_RANGE;
    const hipError_t e = launch_conv_depthwise(g, desc->in_dtype, desc->out_dtype, x, mask_in, w, bias, out,
                                               (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : FC_ERR_HIP;
}

// Fills the geometry part of the pyramid arguments; returns an fc_status.
static int32_t pyramid_geometry(int32_t n, int32_t h, int32_t w, int32_t levels, const fc_mask_step *steps,
                                PyramidArgs *a)
{
    if (!steps) return FC_ERR_NULL;
    if (n <= 0 || h <= 0 || w <= 0 || levels <= 0 || levels > kMaxPyramidLevels) return FC_ERR_SHAPE;
    if ((int64_t)n * h * w >= INT32_MAX) return FC_ERR_RANGE;
    a->levels = levels;
    a->n = n;
    a->h[0] = h;
    a->w[0] = w;
    int64_t blocks = 0;
    for (int l = 0; l < levels; ++l) {
        const fc_mask_step &t = steps[l];
        if (t.kh <= 0 || t.kw <= 0 || t.stride_h <= 0 || t.stride_w <= 0 || t.pad_h < 0 || t.pad_w < 0 ||
            t.dil_h <= 0 || t.dil_w <= 0)
            return FC_ERR_SHAPE;
        const int32_t ho = out_dim(a->h[l], t.kh, t.stride_h, t.pad_h, t.dil_h);
        const int32_t wo = out_dim(a->w[l], t.kw, t.stride_w, t.pad_w, t.dil_w);
        if (ho <= 0 || wo <= 0) return FC_ERR_SHAPE;
        a->h[l + 1] = ho;
        a->w[l + 1] = wo;
        a->sh[l] = t.stride_h;
        a->sw[l] = t.stride_w;
        a->ch0[l] = -t.pad_h + t.dil_h * ((t.kh - 1) / 2);
        a->cw0[l] = -t.pad_w + t.dil_w * ((t.kw - 1) / 2);
        a->m[l] = (int64_t)n * ho * wo;
        a->div_w[l] = make_fastdiv((uint32_t)wo);
        a->div_h[l] = make_fastdiv((uint32_t)ho);
        if (a->m[l] >= INT32_MAX) return FC_ERR_RANGE;
        a->block0[l] = (int32_t)blocks;
        blocks += compact_blocks(a->m[l]);
    }
    if (blocks >= INT32_MAX) return FC_ERR_RANGE;
    a->block0[levels] = (int32_t)blocks;
    a->identity0 = (a->sh[0] == 1 && a->sw[0] == 1 && a->ch0[0] == 0 && a->cw0[0] == 0 && a->h[1] == h && a->w[1] == w) ? 1 : 0;
    return FC_OK;
}

int32_t fc_mask_pyramid_dims(int32_t h, int32_t w, int32_t levels, const fc_mask_step *steps, int32_t *hs,
                             int32_t *ws)
{
    if (!hs || !ws) return FC_ERR_NULL;
    PyramidArgs a;
    const int32_t rc = pyramid_geometry(1, h, w, levels, steps, &a);
    if (rc != FC_OK) return rc;
    for (int l = 0; l < levels; ++l) {
        hs[l] = a.h[l + 1];
        ws[l] = a.w[l + 1];
    }
    return FC_OK;
}

int32_t fc_mask_pyramid_workspace_bytes(int32_t n, int32_t h, int32_t w, int32_t levels,
                                        const fc_mask_step *steps, size_t *bytes)
{
    if (!bytes) return FC_ERR_NULL;
    PyramidArgs a;
    const int32_t rc = pyramid_geometry(n, h, w, levels, steps, &a);
    if (rc != FC_OK) return rc;
    *bytes = align_up((size_t)a.block0[levels] * sizeof(int32_t), 256);
    return FC_OK;
}

static int32_t mask_pyramid_any(const uint8_t *mask_in, int32_t packed_in, int32_t packed_out, int32_t n, int32_t h,
                                int32_t w, int32_t levels, const fc_mask_step *steps, uint8_t *const *mask_out,
                                int32_t *const *idx, int32_t *const *count, void *workspace, size_t workspace_bytes,
                                void *stream)
{
    if (!mask_in || !mask_out || !idx || !count) return FC_ERR_NULL;
    PyramidArgs a;
    const int32_t rc = pyramid_geometry(n, h, w, levels, steps, &a);
    if (rc != FC_OK) return rc;
    a.packed_in = packed_in ? 1 : 0;
    a.packed_out = packed_out ? 1 : 0;
    if (a.packed_in && !aligned16(mask_in)) return FC_ERR_ALIGN;
    for (int l = 0; l < levels; ++l) {
        if (!mask_out[l] || !idx[l] || !count[l]) return FC_ERR_NULL;
        if (!aligned16(mask_out[l]) || !aligned16(idx[l])) return FC_ERR_ALIGN;
        a.mask_out[l] = mask_out[l];
        a.idx[l] = idx[l];
        a.count[l] = count[l];
    }
    if (!aligned16(mask_in)) a.identity0 = 0;
    const size_t need = align_up((size_t)a.block0[levels] * sizeof(int32_t), 256);
    if (!workspace || workspace_bytes < need) return FC_ERR_WORKSPACE;
    if (!aligned16(workspace)) return FC_ERR_ALIGN;
    const hipError_t e = launch_mask_pyramid(a, mask_in, (int32_t *)workspace, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : FC_ERR_HIP;
}

int32_t fc_mask_pyramid(const uint8_t *mask_in, int32_t n, int32_t h, int32_t w, int32_t levels,
                        const fc_mask_step *steps, uint8_t *const *mask_out, int32_t *const *idx,
                        int32_t *const *count, void *workspace, size_t workspace_bytes, void *stream)
{
    return mask_pyramid_any(mask_in, 0, 0, n, h, w, levels, steps, mask_out, idx, count, workspace, workspace_bytes,
                            stream);
}

int32_t fc_mask_pyramid_packed(const void *mask_in, int32_t mask_in_packed, int32_t n, int32_t h, int32_t w,
                               int32_t levels, const fc_mask_step *steps, uint64_t *const *bits_out,
                               int32_t *const *idx, int32_t *const *count, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    return mask_pyramid_any((const uint8_t *)mask_in, mask_in_packed, 1, n, h, w, levels, steps,
                            (uint8_t *const *)bits_out, idx, count, workspace, workspace_bytes, stream);
}

size_t fc_packed_mask_bytes(int64_t m) { return m <= 0 ? 0 : (size_t)((m + 63) / 64) * 8; }

int32_t fc_mask_pack(const uint8_t *mask, int64_t m, uint64_t *bits, void *stream)
{
    if (!mask || !bits) return FC_ERR_NULL;
    if (m <= 0) return FC_ERR_SHAPE;
    if (m >= INT32_MAX) return FC_ERR_RANGE;
    if (!aligned16(bits)) return FC_ERR_ALIGN;
    return launch_mask_pack(mask, m, bits, (hipStream_t)stream) == hipSuccess ? FC_OK : FC_ERR_HIP;
}

int32_t fc_mask_downsample_packed(const uint64_t *bits_in, int32_t n, int32_t h, int32_t w, int32_t kh, int32_t kw,
                                  int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t dil_h,
                                  int32_t dil_w, uint64_t *bits_out, void *stream)
{
    if (!bits_in || !bits_out) return FC_ERR_NULL;
    if (n <= 0 || h <= 0 || w <= 0 || kh <= 0 || kw <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 ||
        pad_w < 0 || dil_h <= 0 || dil_w <= 0)
        return FC_ERR_SHAPE;
    const int32_t ho = out_dim(h, kh, stride_h, pad_h, dil_h), wo = out_dim(w, kw, stride_w, pad_w, dil_w);
    if (ho <= 0 || wo <= 0) return FC_ERR_SHAPE;
    if ((int64_t)n * ho * wo >= INT32_MAX || (int64_t)n * h * w >= INT32_MAX) return FC_ERR_RANGE;
    if (!aligned16(bits_in) || !aligned16(bits_out)) return FC_ERR_ALIGN;
    MaskGeom g = mask_geom(n, h, w, kh, kw, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, ho, wo);
    g.packed_in = g.packed_out = 1;
    return launch_mask_rescale(g, (const uint8_t *)bits_in, (uint8_t *)bits_out, (hipStream_t)stream) == hipSuccess
               ? FC_OK
               : FC_ERR_HIP;
}

int32_t fc_active_index_compact_packed(const uint64_t *bits, int64_t m, int32_t *idx, int32_t *count, void *workspace,
                                       size_t workspace_bytes, void *stream)
{
    if (!bits || !idx || !count) return FC_ERR_NULL;
    if (m <= 0) return FC_ERR_SHAPE;
    if (m >= INT32_MAX) return FC_ERR_RANGE;
    if (!workspace || workspace_bytes < compact_ws(m)) return FC_ERR_WORKSPACE;
    if (!aligned16(bits) || !aligned16(idx) || !aligned16(workspace)) return FC_ERR_ALIGN;
    MaskGeom g = mask_geom(1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1, 1, 1);
    g.w = g.wo = (int32_t)m;
    g.m = m;
    g.packed_in = 1;
    const hipError_t e = launch_compact(g, (const uint8_t *)bits, nullptr, idx, count, (int32_t *)workspace,
                                        CompactExtras(), (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : FC_ERR_HIP;
}

// ---- the entry point that allocates nothing --------------------------------------------
// Its workspace is this file-scope device array.  Every GPU the library is loaded on holds its
// own copy at its own address; the name `noalloc_scratch` is only a handle for
// hipGetSymbolAddress in host code, never a pointer to pass on.
} // extern "C"
static __device__ __align__(256) unsigned char noalloc_scratch[FC_NOALLOC_SCRATCH_BYTES];
namespace {
constexpr int kNoallocMaxDevices = 64;
std::atomic<void *> noalloc_ptr[kNoallocMaxDevices];

// Address of the current device's copy of the array (resolved once per device).
int32_t noalloc_scratch_of_current_device(void **p)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return FC_ERR_HIP;
    if (dev < 0 || dev >= kNoallocMaxDevices) return FC_ERR_RANGE;
    void *q = noalloc_ptr[dev].load(std::memory_order_acquire);
    if (!q) {
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(noalloc_scratch)) != hipSuccess || !q) return FC_ERR_HIP;
        noalloc_ptr[dev].store(q, std::memory_order_release); // (two threads store the same address)
    }
    *p = q;
    return FC_OK;
}
} // namespace
extern "C" {

int32_t fc_noalloc_init(void)
{
    void *p;
    return noalloc_scratch_of_current_device(&p);
}

int32_t fc_focused_conv2d_noalloc(const fc_conv_desc *desc, const void *x, const uint8_t *mask_in, const void *w,
                                  const float *bias, void *out, void *stream)
{
    Geom g;
    const int32_t rc = make_geom(desc, &g);
    if (rc != FC_OK) return rc;
    // the whole workspace of the call (split-K scratch, labels, kept list) must fit the array
    if (conv_ws_layout(g).total > (size_t)FC_NOALLOC_SCRATCH_BYTES) return FC_ERR_RANGE;
    void *scratch;
    const int32_t rs = noalloc_scratch_of_current_device(&scratch);
    if (rs != FC_OK) return rs;
    // the array keeps the last call's contents: the arrival counters are cleared by this call
    // whatever the caller's flags say (everything else in it is written before it is read)
    fc_conv_desc d = *desc;
    d.flags &= ~(uint32_t)FC_WORKSPACE_READY;
    return fc_focused_conv2d(&d, x, mask_in, w, bias, nullptr, nullptr, nullptr, out, scratch,
                             (size_t)FC_NOALLOC_SCRATCH_BYTES, stream);
}

int32_t fc_calibrate_mfma(int32_t dtype, int32_t iters, int32_t blocks, void *sink, double *flop, void *stream)
{
    if (!sink || !flop) return FC_ERR_NULL;
    if (dtype != FC_BF16 && dtype != FC_F16 && dtype != FC_FP8) return FC_ERR_DTYPE;
    if (iters <= 0 || blocks <= 0 || blocks > (1 << 20)) return FC_ERR_SHAPE;
    // 8 instructions a round, 2 * 32 * 32 * K multiply-adds each (K = 16, or 64 for 8-bit operands), 4 waves
    *flop = (double)blocks * 4.0 * (double)iters * 8.0 * 2.0 * 32.0 * 32.0 * (dtype == FC_FP8 ? 64.0 : 16.0);
    return launch_calibrate_mfma(dtype, iters, blocks, (float *)sink, (hipStream_t)stream) == hipSuccess ? FC_OK
                                                                                                            : FC_ERR_HIP;
}

int32_t fc_calibrate_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst) return FC_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return FC_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return FC_ERR_ALIGN;
    if (ranges_overlap(src, bytes, dst, bytes)) return FC_ERR_NULL;
    return launch_calibrate_copy(src, dst, bytes, (hipStream_t)stream) == hipSuccess ? FC_OK : FC_ERR_HIP;
}

int32_t fc_calibrate_issue(int32_t mode, int32_t waves_per_simd, int32_t steps, int32_t blocks, const void *src,
                           size_t src_bytes, int64_t *cycles, void *sink, void *stream)
{
    if (!src || !cycles || !sink) return FC_ERR_NULL;
    if (mode < 0 || mode > 4 || (waves_per_simd != 1 && waves_per_simd != 2 && waves_per_simd != 4)) return FC_ERR_SHAPE;
    if (steps <= 0 || blocks <= 0 || blocks > 65536) return FC_ERR_SHAPE;
    if (src_bytes < ((size_t)1 << 20)) return FC_ERR_WORKSPACE;
    if (!aligned16(src)) return FC_ERR_ALIGN;
    return launch_calibrate_issue(mode, waves_per_simd, steps, blocks, src, (long long *)cycles, (float *)sink,
                                  (hipStream_t)stream) == hipSuccess
               ? FC_OK
               : FC_ERR_HIP;
}

int32_t fc_maxpool2d(const void *x, int32_t n, int32_t h, int32_t w, int32_t c, int32_t dtype, int32_t k,
                     int32_t stride, int32_t pad, void *out, void *stream)
{
    return fc_maxpool2d_masked(x, n, h, w, c, dtype, k, stride, pad, nullptr, out, stream);
}

int32_t fc_maxpool2d_masked(const void *x, int32_t n, int32_t h, int32_t w, int32_t c, int32_t dtype, int32_t k,
                            int32_t stride, int32_t pad, const uint8_t *keep, void *out, void *stream)
{
    if (!x || !out) return FC_ERR_NULL;
    if (n <= 0 || h <= 0 || w <= 0 || c <= 0 || k <= 0 || stride <= 0 || pad < 0 || 2 * pad > k)
        return FC_ERR_SHAPE;
    if (dtype != FC_F32 && dtype != FC_BF16 && dtype != FC_F16) return FC_ERR_DTYPE;
    const int32_t ho = out_dim(h, k, stride, pad, 1), wo = out_dim(w, k, stride, pad, 1);
    if (ho <= 0 || wo <= 0) return FC_ERR_SHAPE;
    const hipError_t e = launch_maxpool(x, n, h, w, c, dtype, k, stride, pad, ho, wo, keep, out, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : FC_ERR_HIP;
}

} // extern "C"
