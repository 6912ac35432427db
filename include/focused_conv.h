/*
 * focused_conv.h - C ABI of the focused convolution library for AMD MI355X
 * (gfx950).
 *
 * The focused convolution (Tung et al., "Irrelevant Pixels are Everywhere",
 * Sec. III-A) is a GEMM convolution whose im2col step skips every patch that a
 * binary pixel mask labels irrelevant, so that the matrix product has fewer
 * columns; weights and bias are those of the dense layer, and with no mask the
 * layer is the standard convolution.  Sec. III-B carries the mask through a
 * network by rescaling it to each layer's spatial size.
 *
 * Semantics fixed by this library (the paper leaves them open):
 *   - mask: one byte per pixel, per image, [N][H][W]; nonzero = relevant.
 *   - a patch (= an output position) is kept iff the INPUT mask under the
 *     centre tap of its receptive field is relevant:
 *         ih_c = clamp(oh*stride_h - pad_h + dil_h*((KH-1)/2), 0, H-1)
 *     (same for iw_c).  This is nearest-neighbour rescaling of the mask.
 *   - a kept output equals the dense convolution of the input with irrelevant
 *     input pixels (and padding) treated as zero.  Gated taps are skipped, not
 *     multiplied: NaN/Inf at irrelevant input pixels never reach an output.
 *   - an irrelevant output position holds +0.0 in every channel (no bias), or
 *     is left untouched when FC_SKIP_ZERO_FILL is set.
 *   - Ho = floor((H + 2*pad_h - dil_h*(KH-1) - 1)/stride_h) + 1 (same for Wo).
 *   - arithmetic: products of the stored inputs accumulated in fp32, bias added
 *     in fp32, optional ReLU, one round-to-nearest-even to the output type.
 *
 * Layouts (all dense, no strides): x[N][H][W][C_in] (NHWC),
 * w[C_out][KH][KW][C_in], bias[C_out] float32, out[N][Ho][Wo][C_out].
 *
 * Conventions for every entry point:
 *   - pointers marked "device" are HIP device memory owned by the caller; the
 *     library allocates nothing and frees nothing.  What it keeps between calls is
 *     host-side only and per device: which kernel variants have had their dynamic
 *     LDS limit raised, the CU count, and the address of the device array of
 *     fc_focused_conv2d_noalloc.  No result depends on it.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All device work is enqueued on it; no call waits for the device and no
 *     call reads results back to the host.
 *   - the return value is an fc_status.  Argument errors are found on the host
 *     before anything is launched and leave every output untouched.  FC_ERR_HIP
 *     means the HIP runtime refused a launch: launches enqueued before it stay
 *     enqueued, so the workspace (and, for calls that build their own kept list,
 *     nothing else) may have been written; `out` is written by the last launch
 *     of a call only.
 *   - device base pointers must be 16-byte aligned.
 *   - every call enqueues kernel launches only (no memsets, no copies, no
 *     allocation), so calls can be recorded into a HIP graph.  The first call
 *     on a device that uses a given kernel variant also raises that kernel's
 *     dynamic LDS limit (a host-side attribute call, once per variant and
 *     device): run a call once eagerly before capturing it.
 */
#ifndef FOCUSED_CONV_H
#define FOCUSED_CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FC_OK = 0,
    FC_ERR_NULL = -1,      /* a required pointer is NULL */
    FC_ERR_SHAPE = -2,     /* a size is zero/negative or gives an empty output */
    FC_ERR_DTYPE = -3,     /* unknown or unsupported type combination */
    FC_ERR_ALIGN = -4,     /* a device pointer is not 16-byte aligned */
    FC_ERR_WORKSPACE = -5, /* workspace missing or smaller than fc_workspace_bytes */
    FC_ERR_RANGE = -6,     /* N*Ho*Wo or N*H*W does not fit the 31-bit index type */
    FC_ERR_HIP = -7        /* the HIP runtime refused a launch */
} fc_status;

/* FC_FP8 is the 8-bit E4M3 format of the OCP 8-bit floating point specification (the
 * variant without infinities; bias 7, largest value 448, 0x7F/0xFF = NaN), one byte per
 * value, as the gfx950 matrix cores read it.  The paper's method does not depend on the
 * storage type (Sec. III-A keeps the layer's weights and arithmetic unchanged); the 8-bit
 * form halves the gathered bytes.  Values are used as stored: a caller that quantises with
 * per-tensor scales folds their product into the bias (divide it) and into whatever reads
 * the output (ReLU commutes with a positive scale). */
typedef enum { FC_F32 = 0, FC_BF16 = 1, FC_F16 = 2, FC_FP8 = 3 } fc_dtype;

enum {
    FC_RELU = 1u,           /* max(.,0) at kept positions */
    FC_SKIP_ZERO_FILL = 2u, /* leave irrelevant output positions untouched */
    FC_WORKSPACE_READY = 4u, /* the caller vouches that the counters at the start of `workspace` are
                               zero: true for a workspace that was zeroed once, and from then on
                               after every completed fc_focused_conv2d call that was given it (the
                               library leaves them zero).  Saves the launch that clears them. */
    /* Compacted activations (fc_focused_conv2d with a kept list only, matrix-core layers only,
       else FC_ERR_DTYPE): rows stored in list order, row j = list entry j, nothing for the
       irrelevant positions.  Layers that see the same list can hand each other such tensors. */
    FC_COMPACT_OUT = 8u,     /* out is [count][c_out] (capacity n*ho*wo rows); no zero-fill */
    FC_COMPACT_IN = 16u,     /* x is [count][c_in]; 1x1 kernels with unit stride and no padding only
                               (else FC_ERR_SHAPE): row j of x is the pixel list entry j reads */
    /* Packed masks: mask_in and mask_out of this call are one BIT per pixel instead of one byte
       (see fc_mask_pack for the layout).  fc_focused_conv2d and fc_focused_gconv2d only; layers
       with at most 4 input channels and depthwise layers take byte masks (FC_ERR_DTYPE). */
    FC_PACKED_MASKS = 32u,
    /* Kernel choice.  The library picks the kernel of a matrix-core layer from its shape by rules
       measured on the layers of ResNet, VGG and MobileNet backbones.  With this flag a layer that
       the resident-weights kernel supports (1x1 without padding, and 3x3 whose pixels are 128
       bytes: 64 channels of a 16-bit type or 128 of the 8-bit one; more than 4 096 output
       positions; a kept list or no mask) runs on that kernel whatever the rule says; on any other
       layer the flag changes nothing.  Results are the same to the documented tolerance either
       way (fp32 accumulation in a different order). */
    FC_RESIDENT_WEIGHTS = 64u
};

/* The arrival counters of FC_WORKSPACE_READY live in this many leading bytes of the workspace. */
enum { FC_WORKSPACE_COUNTER_BYTES = 2048 };

/* One convolution layer.  in_dtype is the storage type of x and w; out_dtype is
 * in_dtype or FC_F32 (for FC_FP8 inputs: FC_BF16 or FC_F32), or FC_FP8 for any in_dtype but
 * FC_F32.  FC_FP8 inputs are served by fc_focused_conv2d only, and only for layers with c_in a
 * multiple of 16, c_out a multiple of 8 and at most 32 taps; FC_FP8 outputs by
 * fc_focused_conv2d only, for c_out a multiple of 16 and the layers its matrix-core kernels
 * take (16-bit storage: c_in a multiple of 8 and at most 32 taps, or c_in <= 4); anything
 * else gives FC_ERR_DTYPE.
 * An FC_FP8 output is the fp32 result (bias and ReLU applied) rounded once to the nearest
 * E4M3 value, ties to the even code; magnitudes beyond 448 are stored as 448 with their
 * sign, NaN as one of the two NaN codes: what the next 8-bit layer reads, so that a chain of such layers moves
 * one byte per value (the caller's scales are folded as described at fc_dtype). */
typedef struct fc_conv_desc {
    int32_t n, h, w, c_in, c_out, kh, kw;
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
    int32_t in_dtype, out_dtype; /* fc_dtype */
    uint32_t flags;
} fc_conv_desc;

/* Human-readable name of a status code (static storage, never NULL). */
const char *fc_status_string(int32_t status);

/* Output size of a layer (Sec. III-A operation count; the Fig. 5 caption's 4x6
 * input with a 3x3 kernel giving 8 patches fixes the "+1").  Host only. */
int32_t fc_out_dims(const fc_conv_desc *desc, int32_t *ho, int32_t *wo);

/* Bytes of device workspace fc_focused_conv2d needs when the caller passes no
 * index list (split-K scratch for small layers + mask_out + idx + count + scan
 * scratch), and
 * fc_active_index_compact needs for `m` positions.  Host only. */
int32_t fc_workspace_bytes(const fc_conv_desc *desc, size_t *bytes);
int32_t fc_compact_workspace_bytes(int64_t m, size_t *bytes);

/* Mask propagation (Sec. III-B: the mask is rescaled to each layer's size).
 * mask_out[n][oh][ow] = (mask_in under the centre tap of (oh,ow)) != 0, written
 * as 0/1 bytes.  Takes the geometry of the layer (or pooling window) that
 * changes the resolution.
 *   mask_in  device, [n][h][w] bytes, read only
 *   mask_out device, [n][ho][wo] bytes, fully overwritten */
int32_t fc_mask_downsample(const uint8_t *mask_in, int32_t n, int32_t h, int32_t w,
                           int32_t kh, int32_t kw, int32_t stride_h, int32_t stride_w,
                           int32_t pad_h, int32_t pad_w, int32_t dil_h, int32_t dil_w,
                           uint8_t *mask_out, void *stream);

/* Patch labels by another rule.  Sec. III-A drops the patches that carry an irrelevant
 * label without saying how a per-pixel mask labels a whole patch; this library's reading is the
 * centre tap (fc_mask_downsample, and what fc_focused_conv2d derives by itself).  The
 * other two readings are offered here: FC_RULE_ANY keeps a patch if any pixel of its
 * window is relevant (conservative: a margin of context around the relevant region),
 * FC_RULE_ALL only if all are.  Pixels outside the image are not part of the window; a
 * window wholly outside is irrelevant.  FC_RULE_CENTRE is fc_mask_downsample.
 * To run a layer with such labels, compact them (fc_active_index_compact) and pass
 * mask_out, idx and count to fc_focused_conv2d, with the geometry of that same layer:
 * taps are still gated by mask_in, rows with label 0 are still zero-filled.
 * Arguments as fc_mask_downsample; an unknown rule gives FC_ERR_DTYPE. */
enum { FC_RULE_CENTRE = 0, FC_RULE_ANY = 1, FC_RULE_ALL = 2 };
int32_t fc_mask_downsample_rule(const uint8_t *mask_in, int32_t n, int32_t h, int32_t w,
                                int32_t kh, int32_t kw, int32_t stride_h, int32_t stride_w,
                                int32_t pad_h, int32_t pad_w, int32_t dil_h, int32_t dil_w,
                                int32_t rule, uint8_t *mask_out, void *stream);

/* Packed masks (Sec. III-B's per-layer mask at an eighth of the bytes): one bit per pixel,
 * pixel p of the flat [n][h][w] order is bit p % 64 of the 64-bit word p / 64 (what a 64-lane
 * ballot over 64 consecutive pixels gives; little-endian, so also bit p % 8 of byte p / 8); the
 * bits of the last word past the last pixel are zero.  A packed mask of m pixels occupies
 * fc_packed_mask_bytes(m) = 8 * ceil(m / 64) bytes and must be 16-byte aligned.
 *   fc_mask_pack               bytes -> bits (a nonzero byte is a 1)
 *   fc_mask_downsample_packed  fc_mask_downsample from bits to bits
 *   fc_active_index_compact_packed  fc_active_index_compact from bits (same list, bit for bit)
 *   fc_mask_pyramid_packed     fc_mask_pyramid with the levels' masks written as bits; the input
 *                              mask is bytes (mask_in_packed = 0) or bits (1)
 * and fc_focused_conv2d takes them with FC_PACKED_MASKS.  Arguments otherwise as the byte forms. */
size_t fc_packed_mask_bytes(int64_t m);
int32_t fc_mask_pack(const uint8_t *mask, int64_t m, uint64_t *bits, void *stream);
int32_t fc_mask_downsample_packed(const uint64_t *bits_in, int32_t n, int32_t h, int32_t w,
                                  int32_t kh, int32_t kw, int32_t stride_h, int32_t stride_w,
                                  int32_t pad_h, int32_t pad_w, int32_t dil_h, int32_t dil_w,
                                  uint64_t *bits_out, void *stream);
int32_t fc_active_index_compact_packed(const uint64_t *bits, int64_t m, int32_t *idx, int32_t *count,
                                       void *workspace, size_t workspace_bytes, void *stream);

/* Which patches become columns (Sec. III-A: an irrelevant patch is not
 * converted).  Writes the ascending list of flat positions p in [0,m) with
 * mask[p] != 0 and their number.  One list serves every layer at that
 * resolution.
 *   mask      device, m bytes, read only
 *   idx       device, capacity m int32; idx[0..count) written, rest unspecified
 *   count     device, one int32, overwritten
 *   workspace device, >= fc_compact_workspace_bytes(m) */
int32_t fc_active_index_compact(const uint8_t *mask, int64_t m, int32_t *idx, int32_t *count,
                                void *workspace, size_t workspace_bytes, void *stream);

/* The same positions in tile order.  Sec. III-A fixes WHICH patches become columns, not their
 * order, and fc_focused_conv2d takes the kept positions in any order (each exactly once): every
 * output row gets the same terms, only the order of its fp32 sum may differ.  This list walks every image tile by tile - tiles of
 * tile_h x tile_w positions, row-major over the tiles, row-major inside a tile - so that
 * the rows of one GEMM tile are neighbours in both directions.
 *   mask      device, [n][ho][wo] bytes (a layer's output-resolution mask), read only
 *   tile_w    1..32; tile_h >= 1
 *   idx,count as fc_active_index_compact
 *   workspace device, >= fc_compact_tiled_workspace_bytes(...) */
int32_t fc_compact_tiled_workspace_bytes(int32_t n, int32_t ho, int32_t wo, int32_t tile_h,
                                         int32_t tile_w, size_t *bytes);
int32_t fc_active_index_compact_tiled(const uint8_t *mask, int32_t n, int32_t ho, int32_t wo,
                                      int32_t tile_h, int32_t tile_w, int32_t *idx, int32_t *count,
                                      void *workspace, size_t workspace_bytes, void *stream);

/* Mask pyramid (Sec. III-B: one mask per image, rescaled to every layer's size).  Builds, for
 * `levels` successive resolution changes, the mask and the kept-position list of every level
 * from the input mask in two launches.  steps[l] is the window (kernel, stride, padding,
 * dilation) of the layer that takes level l - 1 (the input mask for l = 0) to level l; level l
 * equals fc_mask_downsample of level l - 1 with that window, and its list equals
 * fc_active_index_compact of it (bit for bit).
 *   mask_in   device, [n][h][w] bytes, read only
 *   mask_out  host array of `levels` device pointers, [n][h_l][w_l] bytes each, overwritten
 *   idx,count host arrays of `levels` device pointers (capacity n*h_l*w_l int32; one int32)
 *   workspace device, >= fc_mask_pyramid_workspace_bytes
 * fc_mask_pyramid_dims gives h_l, w_l (host only). */
#define FC_MAX_PYRAMID_LEVELS 8
typedef struct fc_mask_step {
    int32_t kh, kw, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} fc_mask_step;
int32_t fc_mask_pyramid_dims(int32_t h, int32_t w, int32_t levels, const fc_mask_step *steps,
                             int32_t *hs, int32_t *ws);
int32_t fc_mask_pyramid_workspace_bytes(int32_t n, int32_t h, int32_t w, int32_t levels,
                                        const fc_mask_step *steps, size_t *bytes);
int32_t fc_mask_pyramid(const uint8_t *mask_in, int32_t n, int32_t h, int32_t w, int32_t levels,
                        const fc_mask_step *steps, uint8_t *const *mask_out, int32_t *const *idx,
                        int32_t *const *count, void *workspace, size_t workspace_bytes, void *stream);
int32_t fc_mask_pyramid_packed(const void *mask_in, int32_t mask_in_packed, int32_t n, int32_t h, int32_t w,
                               int32_t levels, const fc_mask_step *steps, uint64_t *const *bits_out,
                               int32_t *const *idx, int32_t *const *count, void *workspace,
                               size_t workspace_bytes, void *stream);

/* The layer (Sec. III-A).  Gathers the receptive fields of the kept positions
 * (implicit im2col), multiplies by the unchanged weights on the matrix cores,
 * adds bias, applies ReLU if asked, writes each kept row, zero-fills the rest.
 *   x         device, NHWC, in_dtype, read only
 *   mask_in   device [n][h][w] bytes, or NULL = every pixel relevant (the dense
 *             layer; idx/count/mask_out must then be NULL too)
 *   w         device, [c_out][kh][kw][c_in], in_dtype, read only
 *   bias      device, c_out floats, or NULL
 *   mask_out  device [n][ho][wo] 0/1 bytes as fc_mask_downsample (or
 *             fc_mask_downsample_rule) writes them for this layer's geometry, or
 *             NULL (then derived from mask_in by the centre tap).  Given without
 *             idx/count, the call compacts these labels itself (into the
 *             workspace): the rows computed and the rows cleared follow them
 *   idx,count device, as fc_active_index_compact writes them from mask_out; both
 *             NULL = computed here into the workspace
 *   out       device, NHWC, out_dtype; its bytes must not overlap those of x
 *             (FC_ERR_NULL)
 *   workspace device, >= fc_workspace_bytes(desc) when idx is NULL and mask_in is
 *             not; otherwise optional: when given (any call, also the dense
 *             layer), layers with few tiles split their reduction over more
 *             workgroups and park fp32 partial tiles there (deterministic:
 *             partials are always added in the same order).  Its first bytes
 *             hold arrival counters that every call finds and leaves at zero;
 *             a call clears them first unless FC_WORKSPACE_READY is set
 * `count` is read on the device only; the launch grid does not depend on it. */
int32_t fc_focused_conv2d(const fc_conv_desc *desc, const void *x, const uint8_t *mask_in,
                          const void *w, const float *bias, const uint8_t *mask_out,
                          const int32_t *idx, const int32_t *count, void *out,
                          void *workspace, size_t workspace_bytes, void *stream);

/* The same layer for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It is
 * fc_focused_conv2d(desc, x, mask_in, w, bias, NULL, NULL, NULL, out, <scratch>, ..., stream),
 * i.e. the labels, the kept list and the split-K scratch of the call live in a device array
 * of FC_NOALLOC_SCRATCH_BYTES that is part of the library's code object (every GPU the library
 * runs on holds one copy until the process ends).  The call allocates and frees nothing,
 * enqueues kernel launches only, and gives bit for bit the result of that fc_focused_conv2d
 * call.
 *   - layers whose fc_workspace_bytes(desc) exceeds FC_NOALLOC_SCRATCH_BYTES (five bytes per
 *     output position: more than about 8 million positions) are refused with FC_ERR_RANGE
 *     before anything is launched.
 *   - FC_WORKSPACE_READY is ignored (the call always clears the arrival counters itself);
 *     FC_COMPACT_OUT / FC_COMPACT_IN need a caller's list and give FC_ERR_NULL here.
 *   - all calls on one GPU share that GPU's array: calls that may overlap in time on one GPU
 *     (different streams, parallel graph branches) race and must be ordered by the caller.
 *   - the address of the array is looked up on the first call on each device (or by
 *     fc_noalloc_init, with that device current); do either once, eagerly, before capturing
 *     a call into a graph. */
#define FC_NOALLOC_SCRATCH_BYTES (40u << 20)
int32_t fc_noalloc_init(void);
int32_t fc_focused_conv2d_noalloc(const fc_conv_desc *desc, const void *x, const uint8_t *mask_in,
                                  const void *w, const float *bias, void *out, void *stream);

/* The grouped layer: channels cut into `groups` equal slices, output slice g sees input slice
 * g only (the layer type between fc_focused_conv2d, groups = 1, and fc_focused_dwconv2d, one
 * channel per group; both are what this call runs in those two cases).  Sec. III-A unchanged
 * otherwise.  Arguments as fc_focused_conv2d, with
 *   desc      c_in and c_out are the totals; both must be multiples of groups (FC_ERR_SHAPE)
 *   w         device, [c_out][kh][kw][c_in / groups]
 *   workspace needed (>= fc_workspace_bytes(desc)) only when mask_in is given without a list
 * Layers with more than one channel per group run on the vector ALUs, not on the matrix
 * cores, and take the 32- and 16-bit storage types only (FC_FP8: FC_ERR_DTYPE). */
int32_t fc_focused_gconv2d(const fc_conv_desc *desc, int32_t groups, const void *x,
                           const uint8_t *mask_in, const void *w, const float *bias,
                           const uint8_t *mask_out, const int32_t *idx, const int32_t *count,
                           void *out, void *workspace, size_t workspace_bytes, void *stream);

/* A grouped layer is the full layer with block-diagonal weights (the terms outside the blocks
 * are zeros and change no sum).  This writes those weights: w_full[c_out][kh][kw][c_in] from
 * w_grouped[c_out][kh][kw][c_in / groups], any storage type, both device.  With them
 * fc_focused_conv2d runs the grouped layer on the matrix cores, which for the group counts of
 * common networks is several times faster than fc_focused_gconv2d in spite of the `groups`
 * times larger multiply count (and is the only way to run a grouped layer in FC_FP8).  Expand
 * once when the weights are loaded. */
int32_t fc_expand_group_weights(int32_t c_in, int32_t c_out, int32_t kh, int32_t kw, int32_t groups,
                                int32_t dtype, const void *w_grouped, void *w_full, void *stream);

/* The depthwise layer: one KH x KW filter per channel, the layer type most of
 * the two networks of Sec. IV consist of (depthwise-separable blocks; their
 * 1x1 halves are fc_focused_conv2d).  Sec. III-A unchanged otherwise: a
 * position whose centre-tap mask byte is zero gets +0.0 in every channel (or is
 * left untouched with FC_SKIP_ZERO_FILL), a kept position sees zero at
 * irrelevant input pixels and outside the image; exact products, fp32
 * accumulation over the taps in the order kh, kw (16-bit 3x3 layers add the
 * taps two at a time), one rounding to out_dtype.
 *   desc      c_out must equal c_in (else FC_ERR_SHAPE); flags FC_RELU and
 *             FC_SKIP_ZERO_FILL apply
 *   x         device, NHWC, in_dtype, read only; one image must stay below
 *             0xF0000000 bytes and n below 65536 (else FC_ERR_RANGE)
 *   mask_in   device [n][h][w] bytes, or NULL = every pixel relevant
 *   w         device, [c][kh][kw], in_dtype, read only
 *   bias      device, c floats, or NULL
 *   out       device, NHWC [n][ho][wo][c], out_dtype; must not overlap x
 * The label of a position is read from mask_in directly, so the call needs no
 * kept-position list and no workspace; one kernel launch on `stream`. */
int32_t fc_focused_dwconv2d(const fc_conv_desc *desc, const void *x, const uint8_t *mask_in,
                            const void *w, const float *bias, void *out, void *stream);

/* Calibration of the two rooflines the layers are priced against (measurement support, not
 * part of the paper's method; Sec. III-A's operation count is what `flop` counts for a layer).
 * fc_calibrate_mfma enqueues one launch in which `blocks` workgroups of four waves each run
 * `iters` rounds of eight independent matrix instructions of the storage type `dtype`
 * (FC_BF16, FC_F16 or FC_FP8) on register operands, and writes the FLOP of the launch to
 * *flop (host); `sink` is a device buffer of at least blocks * 256 floats that is never
 * written in practice.  fc_calibrate_copy enqueues one streaming copy of `bytes` bytes (a
 * multiple of 16; both buffers device, 16-byte aligned, not overlapping).  The caller times the
 * launches with events on `stream`. */
int32_t fc_calibrate_mfma(int32_t dtype, int32_t iters, int32_t blocks, void *sink, double *flop,
                          void *stream);
int32_t fc_calibrate_copy(const void *src, void *dst, size_t bytes, void *stream);

/* What a wave can issue beside its matrix instructions (measurement support as above; it is
 * what decides how many waves per SIMD the layer kernels need).  One launch of `blocks`
 * workgroups with `waves_per_simd` (1, 2 or 4) waves on every SIMD; every wave runs `steps`
 * steps of two independent 32x32x16 bf16 matrix instructions plus the item `mode` names:
 *   0 nothing, 1 one 1 KB load from `src` into LDS, 2 twelve dependent integer instructions,
 *   3 one 16-byte-per-lane LDS read of the next operand, 4 items 1 and 3.
 *   src       device, at least 1 MiB (src_bytes; else FC_ERR_WORKSPACE), 16-byte aligned, read only
 *   cycles    device, `blocks` 64-bit integers: shader cycles the loop took in the first wave
 *             of every workgroup (divide by `steps`)
 *   sink      device, `blocks` floats, never written in practice
 * Errors: FC_ERR_NULL, FC_ERR_SHAPE (mode, waves_per_simd, steps or blocks out of range),
 * FC_ERR_WORKSPACE, FC_ERR_ALIGN, FC_ERR_HIP. */
int32_t fc_calibrate_issue(int32_t mode, int32_t waves_per_simd, int32_t steps, int32_t blocks,
                           const void *src, size_t src_bytes, int64_t *cycles, void *sink, void *stream);

/* Helper for conv stacks with pooling between layers (not part of the paper's
 * method): NHWC max-pool over the full tensor, window k, stride s, padding p
 * (padding never wins the max).  x/out device, dtype as given. */
int32_t fc_maxpool2d(const void *x, int32_t n, int32_t h, int32_t w, int32_t c, int32_t dtype,
                     int32_t k, int32_t stride, int32_t pad, void *out, void *stream);

/* The same helper for a stack that carries a mask: positions whose byte in `keep`
 * ([n][ho][wo], as fc_mask_downsample writes it for the pool's window) is zero get
 * +0.0 in every channel and their window is not read - no feature is computed at an
 * irrelevant position (Sec. III-A), and a focused layer that reads the pooled tensor
 * with that mask never looks at it.  keep == NULL is fc_maxpool2d. */
int32_t fc_maxpool2d_masked(const void *x, int32_t n, int32_t h, int32_t w, int32_t c, int32_t dtype,
                            int32_t k, int32_t stride, int32_t pad, const uint8_t *keep, void *out,
                            void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FOCUSED_CONV_H */
