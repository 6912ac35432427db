// Focused 1x1 convolution on the gfx950 matrix cores with the layer's weights resident in LDS
// (Sec. III-A: a GEMM over the kept patches only, with the dense layer's weights).
//
// A 1x1 layer without padding is a plain GEMM of the kept pixels with a [C_in x C_out] matrix:
// one gathered row per kept position, a short reduction, and as many bytes written as read or
// more (a bottleneck's 64 -> 256 expansion writes four times what it reads).  The tiled kernel
// spends such a layer on fixed costs: set-up, the one or few stages and the epilogue of a tile
// follow one another, and every tile fetches its own weights.  Here a workgroup (one per CU)
// keeps one slice of the output channels' weights (at most 88 KB) in LDS for the whole launch,
// and every one of its eight or twelve waves is a pipeline of its own over units of 32 kept
// rows: the next 128-byte chunk of its rows is on its way (a wave-wide load into LDS, counted
// and waited for by the wave itself) while the current one is multiplied against the slice.
// Waves do not cooperate after the prologue: no barrier in the loop, two or three waves per SIMD
// cover each other's waits.  16-bit outputs leave through LDS as whole 128-byte lines (the
// accumulator layout by itself gives 32-byte pieces, which cost a 64 -> 256 layer a third of its
// time), 8-bit ones the same way.  Storage is bf16, f16 or E4M3 (the 8-bit matrix instruction);
// rows are whole 16-byte pieces; which layers the library sends here is decided
// in fc_api.hip (conv_pw_wanted), from measurements against the tiled kernel.
//
// Rows = kept output positions (from the list, or all positions of a dense layer); a row's pixel
// is the position's centre tap (stride allowed, no padding), or row j of a compacted input.  The
// pixel that decided to keep a position is the only one the position reads, so no mask byte is
// looked at in the loop.  fp32 accumulators, bias added after the reduction, one rounding.
//
// 3x3 layers whose pixels are one 128-byte chunk (64 channels of a 16-bit type, 128 of the 8-bit
// one) run here as the 1x1 layer of their nine-pixel patches (TAPS = 9): nine chunks per row,
// chunk t the pixel under tap t, slices of 64 output channels (72 KB of weights).  A tap outside
// the image or under an irrelevant pixel is not read (its chunk arrives as zeros): the mask bytes
// under the nine taps of a unit's rows are fetched into LDS a unit ahead, and every gathered row
// carries a nine-bit set of the taps it reads.  Any stride, padding and dilation.
#include "fc_dma_util.hpp"
#include <atomic>

namespace fc {

constexpr uint32_t kPwChunkBytes = 32u * 128u;  // a chunk buffer: 32 rows x 64 channels
// LDS of a wave: RING chunk buffers + the list entries of a unit
constexpr uint32_t pw_wave_bytes(int ring) { return (uint32_t)ring * kPwChunkBytes + 256u; }
// 3x3 layers: + the mask bytes under the nine taps of a unit's rows (five wave loads of a dword per lane)
constexpr uint32_t kPwTapMaskBytes = 5u * 256u;
constexpr uint32_t pw_wave_bytes_of(int ring, int taps) { return pw_wave_bytes(ring) + (taps > 1 ? kPwTapMaskBytes : 0u); }

struct PwDivs {
    FastDiv wo, ho, cpr; // output width, output height, 16-byte pieces per output row
};

__device__ __forceinline__ void pw_dma_load4(const u32x4_t &rsrc, uint32_t byte_offset, uint32_t lds_addr)
{
    __asm__ volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                     :
                     : "s"(lds_addr), "v"(byte_offset), "s"(rsrc)
                     : "memory");
}

// one byte per lane, zero-extended into the lane's dword of LDS (out of range: zero)
__device__ __forceinline__ void pw_dma_load1(const u32x4_t &rsrc, uint32_t byte_offset, uint32_t lds_addr)
{
    __asm__ volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_ubyte %1, %2, 0 offen lds"
                     :
                     : "s"(lds_addr), "v"(byte_offset), "s"(rsrc)
                     : "memory");
}

// s_waitcnt takes its count as an immediate, and n (wave-uniform) is known at run time only: a
// jump into a table of 16 waits for the even counts 0 .. 30 (each followed by a branch to the
// end), taking the largest even count that is not above n.
#define FC_WJ(k) "s_waitcnt vmcnt(" #k ")\n\ts_branch 1f\n\t"
__device__ __forceinline__ void pw_wait_vmcnt(int n)
{
    // the table starts 12 bytes after the address s_getpc_b64 returns; an entry is 8 bytes
    // (n is wave-uniform; the scalar operand below must not be handed a vector register)
    const uint32_t off = (uint32_t)(min(__builtin_amdgcn_readfirstlane(n), 30) >> 1) * 8u + 12u;
    __asm__ volatile("s_getpc_b64 vcc\n\t"
                     "s_add_u32 vcc_lo, vcc_lo, %0\n\t"
                     "s_addc_u32 vcc_hi, vcc_hi, 0\n\t"
                     "s_setpc_b64 vcc\n\t"
                     FC_WJ(0) FC_WJ(2) FC_WJ(4) FC_WJ(6) FC_WJ(8) FC_WJ(10) FC_WJ(12) FC_WJ(14)
                     FC_WJ(16) FC_WJ(18) FC_WJ(20) FC_WJ(22) FC_WJ(24) FC_WJ(26) FC_WJ(28) FC_WJ(30)
                     "1:"
                     :
                     : "s"(off)
                     : "vcc", "scc", "memory");
}
#undef FC_WJ

// Before a load into LDS is issued: every LDS read this wave has issued has returned.  The reads
// of the area the load overwrites come earlier in program order, but issued is not done: the
// compiler places the matrix instructions that wait for them after the (asynchronous, to it
// opaque) load, and the LDS queue of a workgroup whose waves all read weights can hold a read
// back for longer than a load that hits in the cache takes to come back.  Measured before this
// wait was there: in about one launch of ten of a 512 -> 2048 layer one unit's last k-step of a
// chunk was multiplied with the data of the chunk two stages later, on a prefix of its rows.
__device__ __forceinline__ void pw_lds_reads_done()
{
    __asm__ volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// DT: storage type (bf16 / f16 / E4M3); TO: float or the 16-bit / 8-bit carrier of the output;
// NCB: 32-channel blocks of a workgroup's slice of the output channels; KCT: the number of
// 128-byte chunks of an input row (64 channels of a 16-bit type, 128 of the 8-bit one) where the
// chunk loop is unrolled (1, 2, 4, 8: 10 % faster on layers of several chunks), 0 = a launch
// parameter.  The waves of the workgroup (blockDim.x / 64) are a launch parameter.  Rows are whole
// 16-byte pieces on both sides: the pieces of the last chunk past c_in and the channels of the
// last slice past c_out are read as zeros and never stored.
template <int DT, typename TO, int NCB, int KCT, int TAPS>
__global__ __launch_bounds__(768, 1)
void k_conv_pw(Geom g, PwDivs dv, int kch_arg, const unsigned char *__restrict__ x, const uint8_t *__restrict__ mask_in,
               const uint8_t *__restrict__ mask_out, const unsigned char *__restrict__ w,
               const float *__restrict__ bias, const int32_t *__restrict__ idx,
               const int32_t *__restrict__ count, TO *__restrict__ out)
{
    constexpr int ES = DT == FC_FP8 ? 1 : 2;            // bytes per stored element
    constexpr int ODT = DT == FC_FP8 ? FC_BF16 : DT;    // 16-bit output format
    constexpr uint32_t KSTEP = kStepBytes<DT>;          // bytes of a chunk row per matrix instruction
    constexpr int KK = 128 / (int)KSTEP;                // matrix instructions per chunk and block
    static_assert(TAPS == 1 || (TAPS == 9 && NCB == 2), "1x1, or 3x3 with a pixel of one 128-byte chunk");
    constexpr int RING = 2;                   // chunk buffers per wave
    constexpr uint32_t WAVEB = pw_wave_bytes_of(RING, TAPS);
    constexpr int COUT = NCB * 32;
    constexpr int GB = NCB < 4 ? NCB : 4;     // channel blocks multiplied at a time
    // (with several input chunks all accumulators of a row are live at once: the host gives
    // slices of eight blocks to layers of one chunk only)
    static_assert(NCB <= 4 || KCT == 1, "slices of eight blocks: one chunk");
    const int kch = KCT ? KCT : kch_arg;
    const uint32_t wbytes = (uint32_t)kch * COUT * 128u;
    const int nw = (int)blockDim.x >> 6;

    extern __shared__ __align__(16) unsigned char smem_raw[];
    const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>(smem_raw);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const float *bias_s = reinterpret_cast<const float *>(smem_raw + wbytes);
    unsigned char *const my = smem_raw + wbytes + 1024u + (size_t)wave * WAVEB;
    const uint32_t my0 = lds0 + wbytes + 1024u + (uint32_t)wave * WAVEB;
    const int32_t *const idx_w = reinterpret_cast<const int32_t *>(my + RING * kPwChunkBytes);

    const bool packed_masks = (g.flags & FC_PACKED_MASKS) != 0;
    const bool compact_in = (g.flags & FC_COMPACT_IN) != 0, compact_out = (g.flags & FC_COMPACT_OUT) != 0;
    const int rows = idx ? *count : g.m;
    // rows compacted on both sides are row j in, row j out: a plain GEMM, the list is not read
    const bool use_list = idx && !(compact_in && compact_out);
    // A workgroup multiplies by one slice of COUT output channels.  Workgroup b runs on XCD
    // b mod 8; the workgroups of an XCD form groups of n_slices neighbours that share their rows
    // (each takes another slice, so the rows come out of that XCD's L2 for all but the first),
    // and XCD j takes the j-th contiguous eighth of the rows.  Workgroups left over when the
    // slices do not divide an XCD's workgroups take no rows (they still clear rows below).
    const int n_slices = (g.c_out + COUT - 1) / COUT;
    const int in_xcd = (int)blockIdx.x >> 3, groups_per_xcd = ((int)gridDim.x >> 3) / n_slices;
    const bool spare = in_xcd >= groups_per_xcd * n_slices;
    const int co0 = spare ? 0 : (in_xcd % n_slices) * COUT;
    const int group = ((int)blockIdx.x & 7) * groups_per_xcd + in_xcd / n_slices;
    const int co_left = g.c_out - co0; // channels of this slice and after it
    // an output larger than the memory-side cache (256 MB) is streamed past it: measured on a
    // 64 -> 256 layer, 314 MB of rows leave 22 % faster that way, 164 MB of rows 10 % slower
    const bool stream_out = (int64_t)rows * g.c_out * (int)sizeof(TO) > (256ll << 20);
    // 16-byte pieces of a weight row (a 3x3 layer's row is its nine taps' pixels, one chunk each:
    // the layer is the 1x1 layer of the 9 C_in-channel patch)
    const int cin8 = (TAPS * g.c_in * ES) >> 4;

    // ---- the weights: LDS row (chunk, output channel) holds that channel's 128 bytes of input
    // channels of the chunk, its 16-byte pieces swizzled by the channel ----
    if (!spare) {
        const u32x4_t rsrc_w = make_rsrc_words(w, (uint32_t)g.c_out * (uint32_t)(TAPS * g.c_in) * (uint32_t)ES);
        const int loads = kch * (COUT / 8); // wave loads of 8 rows each
        for (int ii = wave; ii < loads; ii += nw) {
            const int ch = ii / (COUT / 8), co = (ii - ch * (COUT / 8)) * 8 + (lane >> 3);
            const int piece = ch * 8 + ((lane & 7) ^ (int)FC_SWZ(co));
            const bool ok = co < co_left && piece < cin8;
            const uint32_t off = ((uint32_t)(co0 + co) * (uint32_t)(TAPS * g.c_in)) * (uint32_t)ES + (uint32_t)piece * 16u;
            dma_load16(rsrc_w, ok ? off : kOutOfRange, lds0 + (uint32_t)ii * 1024u);
        }
        for (int c = tid; c < COUT; c += nw * 64)
            reinterpret_cast<float *>(smem_raw + wbytes)[c] = (bias && c < co_left) ? bias[co0 + c] : 0.f;
    }
    wait_vmcnt<0>();
    __syncthreads();

    // ---- my share of the kept rows: units of 32 rows, the same number (+-1) for every wave of
    // the groups ----
    const int nwv = 8 * groups_per_xcd * nw;
    const int wv = group * nw + wave;
    const int nb = (rows + 31) >> 5;
    const int share_q = nb / nwv, share_r = nb - share_q * nwv;
    const int b0 = wv * share_q + (wv * share_r) / nwv;
    const int b1 = (wv + 1) * share_q + ((wv + 1) * share_r) / nwv;
    const int nu = spare ? 0 : b1 - b0;

    const uint32_t x_rows = compact_in ? (uint32_t)g.m : (uint32_t)g.n * g.h * g.w;
    const uint32_t row_bytes = (uint32_t)g.c_in * (uint32_t)ES;
    const u32x4_t rsrc_x = make_rsrc_words(x, x_rows * row_bytes);
    const u32x4_t rsrc_i = make_rsrc_words(idx, (uint32_t)rows * 4u);
    const bool unit_step = g.sh == 1 && g.sw == 1; // (no padding: the pixel of a position is the position)
    // the last chunk of a row may be short: bit j says whether the piece this lane gathers in
    // wave load j lies inside the row there
    const int tail8 = cin8 - (kch - 1) * 8;
    uint32_t tail_ok = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        tail_ok |= (uint32_t)(((lane & 7) ^ (int)FC_SWZ(j * 8 + (lane >> 3))) < tail8) << j;

    // loads issued so far by this wave, and that count right after the last load of what is awaited
    int issued = 0, mark_idx = 0, mark_x[RING] = {};
    [[maybe_unused]] int mark_m = 0;

    auto issue_idx = [&](int v) {
        if (!use_list) return;
        const uint32_t r = (uint32_t)(b0 + v) * 32u + (uint32_t)lane;
        pw_lds_reads_done();
        pw_dma_load4(rsrc_i, lane < 32 ? r * 4u : kOutOfRange, my0 + RING * kPwChunkBytes);
        issued += 1;
        mark_idx = issued;
    };
    // a unit's rows: where this lane's row is stored (-1: no row), and the byte offsets of the
    // four rows whose pieces this lane gathers (row 8j + lane / 8 in wave load j)
    int st_p[2] = {-1, -1};
    int st_pr[2][4]; // where row 8j + lane / 8 is stored (16-bit outputs leave through LDS, in the gather's row order)
    uint32_t st_off[2][4];
    // 3x3 only: per gathered row the taps that are read (inside the image and relevant: bit kh * 3 + kw;
    // st_off is then the row's origin, tap (0, 0), which may lie before the tensor), and the
    // position of this lane's row in the unit after the next set-up
    [[maybe_unused]] uint32_t st_val[2][4] = {};
    [[maybe_unused]] int st_pn = -1;
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) st_off[k][j] = kOutOfRange, st_pr[k][j] = -1;

    // ---- 3x3: a unit is set up in two steps.  presetup (a unit ahead of setup) takes the list
    // entries and sends for the mask bytes under the nine taps of every row: wave load q brings
    // tap 2q of row (lane & 31) for lanes 0 .. 31 and tap 2q + 1 for lanes 32 .. 63 ----
    const uint32_t mask0 = my0 + RING * kPwChunkBytes + 256u;
    const uint32_t *const mask_w = reinterpret_cast<const uint32_t *>(my + RING * kPwChunkBytes + 256u);
    const u32x4_t rsrc_m = make_rsrc_words(mask_in, packed_masks ? (uint32_t)(((int64_t)g.n * g.h * g.w + 7) >> 3)
                                                                 : (uint32_t)g.n * g.h * g.w);
    // pixel index under tap t of the position (n, oh, ow), or -1 outside the image
    auto tap_pixel = [&](int n, int oh, int ow, int t) -> int {
        const int kh = (t * 11) >> 5, kw = t - kh * 3; // t / 3 for t < 10
        const int ih = oh * g.sh - g.ph + kh * g.dh, iw = ow * g.sw - g.pw + kw * g.dw;
        const bool in = t < 9 && (uint32_t)ih < (uint32_t)g.h && (uint32_t)iw < (uint32_t)g.w;
        return in ? (n * g.h + ih) * g.w + iw : -1;
    };
    [[maybe_unused]] auto presetup = [&](int v) {
        const int r = (b0 + v) * 32 + l32;
        const bool valid = r < rows;
        int p = r;
        if (use_list) {
            pw_wait_vmcnt(issued - mark_idx);
            p = idx_w[l32];
        }
        st_pn = valid ? p : -1;
        if (mask_in) {
            const int q1 = (int)fast_div((uint32_t)(valid ? p : 0), dv.wo);
            const int ow = (valid ? p : 0) - q1 * g.wo;
            const int n = (int)fast_div((uint32_t)q1, dv.ho);
            const int oh = q1 - n * g.ho;
            pw_lds_reads_done();
#pragma unroll
            for (int q = 0; q < 5; ++q) {
                const int px = valid ? tap_pixel(n, oh, ow, 2 * q + half) : -1;
                pw_dma_load1(rsrc_m, px < 0 ? kOutOfRange : (uint32_t)(packed_masks ? px >> 3 : px), mask0 + (uint32_t)q * 256u);
            }
            issued += 5;
            mark_m = issued;
        }
    };
    auto setup = [&](int v, int k) {
        const int r = (b0 + v) * 32 + l32;
        if constexpr (TAPS == 9) {
            const int p = st_pn;
            const bool valid = p >= 0;
            const int q1 = (int)fast_div((uint32_t)(valid ? p : 0), dv.wo);
            const int ow = (valid ? p : 0) - q1 * g.wo;
            const int n = (int)fast_div((uint32_t)q1, dv.ho);
            const int oh = q1 - n * g.ho;
            // this lane's taps (2q + half): inside the image, and relevant
            uint32_t bits = 0;
            if (mask_in) {
                pw_wait_vmcnt(issued - mark_m);
            }
#pragma unroll
            for (int q = 0; q < 5; ++q) {
                const int t = 2 * q + half;
                const int px = valid ? tap_pixel(n, oh, ow, t) : -1;
                uint32_t on = px >= 0;
                if (mask_in) {
                    const uint32_t b = mask_w[q * 64 + lane];
                    on &= packed_masks ? (b >> (px & 7)) & 1u : (uint32_t)(b != 0);
                }
                bits |= on << t;
            }
            bits |= (uint32_t)__shfl((int)bits, lane ^ 32, 64);
            // the row's origin (tap (0, 0)); it may be outside the image, the taps read are not
            const int pix0 = (n * g.h + oh * g.sh - g.ph) * g.w + ow * g.sw - g.pw;
            const uint32_t off = (uint32_t)pix0 * row_bytes;
            st_p[k] = valid ? (compact_out ? r : p) : -1;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = j * 8 + (lane >> 3);
                st_off[k][j] = (uint32_t)__shfl((int)off, row, 64) + (uint32_t)((lane & 7) ^ FC_SWZ(row)) * 16u;
                st_val[k][j] = (uint32_t)__shfl((int)bits, row, 64);
                if constexpr (sizeof(TO) <= 2) st_pr[k][j] = __shfl(st_p[k], row, 64);
            }
            return;
        }
        const bool valid = r < rows;
        int p = r;
        if (use_list) {
            pw_wait_vmcnt(issued - mark_idx);
            p = idx_w[l32];
        }
        int pix = p;
        if (compact_in) {
            pix = r;
        } else if (!unit_step) {
            const int q1 = (int)fast_div((uint32_t)(valid ? p : 0), dv.wo);
            const int ow = (valid ? p : 0) - q1 * g.wo;
            const int n = (int)fast_div((uint32_t)q1, dv.ho);
            const int oh = q1 - n * g.ho;
            pix = (n * g.h + oh * g.sh) * g.w + ow * g.sw;
        }
        const uint32_t off = valid ? (uint32_t)pix * row_bytes : kOutOfRange;
        st_p[k] = valid ? (compact_out ? r : p) : -1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = j * 8 + (lane >> 3);
            const uint32_t o = (uint32_t)__shfl((int)off, row, 64);
            st_off[k][j] = o == kOutOfRange ? o : o + (uint32_t)((lane & 7) ^ FC_SWZ(row)) * 16u;
            if constexpr (sizeof(TO) <= 2) st_pr[k][j] = __shfl(st_p[k], row, 64);
        }
    };
    // one stage: chunk c of the unit with state k, into ring buffer `buf`
    auto issue_x = [&](int k, int c, int buf) {
        pw_lds_reads_done();
        if constexpr (TAPS == 9) {
            // chunk c is the pixel under tap c: the row's origin + (kh dil_h W + kw dil_w) pixels
            const int kh = (c * 11) >> 5, kw = c - kh * 3;
            const uint32_t delta = (uint32_t)((kh * g.dh * g.w + kw * g.dw) * (int)row_bytes);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t o = ((st_val[k][j] >> c) & 1u) ? st_off[k][j] + delta : kOutOfRange;
                dma_load16_s(rsrc_x, o, 0u, my0 + (uint32_t)buf * kPwChunkBytes + (uint32_t)j * 1024u);
            }
        } else {
            const bool last = c == kch - 1;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t o = (last && !((tail_ok >> j) & 1u)) ? kOutOfRange : st_off[k][j];
                dma_load16_s(rsrc_x, o, (uint32_t)c * 128u, my0 + (uint32_t)buf * kPwChunkBytes + (uint32_t)j * 1024u);
            }
        }
        issued += 4;
#pragma unroll
        for (int r = 0; r < RING; ++r) mark_x[r] = buf == r ? issued : mark_x[r];
    };

    // fragment addressing: lane reads row (lane & 31); in k-step kk that is the 16-byte piece
    // 2 kk + (lane >> 5) (8-bit storage: the pieces 4 kk + 2 (lane >> 5) and the one after it),
    // stored at slot piece ^ swizzle(row)
    const uint32_t frag = (uint32_t)l32 * 128u + (uint32_t)((half * (int)(KSTEP / 32u)) ^ FC_SWZ(l32)) * 16u;

    // fp32 outputs: one rounding, ReLU, and every lane stores its four channels
    auto store_block = [&](const f32x16_t &a, int cb, int p_mine) {
        float v[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 bq = *reinterpret_cast<const float4 *>(bias_s + cb * 32 + q * 8 + half * 4);
            v[q * 4 + 0] = a[q * 4 + 0] + bq.x;
            v[q * 4 + 1] = a[q * 4 + 1] + bq.y;
            v[q * 4 + 2] = a[q * 4 + 2] + bq.z;
            v[q * 4 + 3] = a[q * 4 + 3] + bq.w;
        }
        TO *row = out + (int64_t)(p_mine < 0 ? 0 : p_mine) * g.c_out + co0 + cb * 32;
        if constexpr (sizeof(TO) == 4) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v0 = v[q * 4], v1 = v[q * 4 + 1], v2 = v[q * 4 + 2], v3 = v[q * 4 + 3];
                if (g.flags & FC_RELU) {
                    v0 = relu_keep_nan(v0); v1 = relu_keep_nan(v1);
                    v2 = relu_keep_nan(v2); v3 = relu_keep_nan(v3);
                }
                if (p_mine >= 0 && cb * 32 + q * 8 + half * 4 < co_left)
                    store4<ODT, TO>(row + q * 8 + half * 4, v0, v1, v2, v3);
            }
        }
    };

    // 16-bit outputs: two blocks of 32 channels (128 bytes of every row) go through LDS, laid out
    // like a gathered chunk, and leave as whole 128-byte lines: eight lanes per row, 16 bytes each.
    // The staging area is the ring buffer of the chunk just consumed (its fragments are in
    // registers); a wave's LDS accesses execute in order, so no barrier is needed.
    auto store_pair = [&](const f32x16_t &a0, const f32x16_t &a1, int cb, unsigned char *stg) {
        if constexpr (sizeof(TO) == 2) {
            if (cb * 32 >= co_left) return; // (a pair wholly past the last channel)
#pragma unroll
            for (int bl = 0; bl < 2; ++bl) {
                const f32x16_t &a = bl ? a1 : a0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 bq = *reinterpret_cast<const float4 *>(bias_s + (cb + bl) * 32 + q * 8 + half * 4);
                    uint2 pk;
                    store4<ODT, TO>(reinterpret_cast<TO *>(&pk), a[q * 4] + bq.x, a[q * 4 + 1] + bq.y,
                                   a[q * 4 + 2] + bq.z, a[q * 4 + 3] + bq.w);
                    if (g.flags & FC_RELU) {
                        pk.x = relu_packed16(pk.x);
                        pk.y = relu_packed16(pk.y);
                    }
                    const uint32_t at = (uint32_t)l32 * 128u + (uint32_t)((bl * 4 + q) ^ FC_SWZ(l32)) * 16u + (uint32_t)half * 8u;
                    *reinterpret_cast<uint2 *>(stg + at) = pk;
                }
            }
            __asm__ volatile("" ::: "memory");
            u32x4_t piece[4];
            u32x4_t *at16[4];
            const bool inside = cb * 32 + (lane & 7) * 8 < co_left; // this lane's 8 channels exist
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = j * 8 + (lane >> 3);
                const uint32_t at = (uint32_t)row * 128u + (uint32_t)((lane & 7) ^ FC_SWZ(row)) * 16u;
                piece[j] = *reinterpret_cast<const u32x4_t *>(stg + at);
                const int pr = st_pr[0][j];
                at16[j] = reinterpret_cast<u32x4_t *>(out + (int64_t)(pr < 0 ? 0 : pr) * g.c_out + co0 + cb * 32 + (lane & 7) * 8);
            }
            // (the non-temporal stores are written out: the compiler folds a store and its
            // non-temporal twin into one plain store when they sit in the two arms of a branch)
            if (stream_out) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (st_pr[0][j] >= 0 && inside)
                        __asm__ volatile("global_store_dwordx4 %0, %1, off nt" : : "v"(at16[j]), "v"(piece[j]) : "memory");
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (st_pr[0][j] >= 0 && inside) *at16[j] = piece[j];
            }
            __asm__ volatile("" ::: "memory");
        }
    };

    // 8-bit outputs: the (two or four) blocks of a group, 32 bytes of a row each, go through LDS the
    // same way and leave as 16-byte pieces, up to 128 bytes of a row per store instruction.
    auto store_bytes = [&](const f32x16_t *a, int cb, unsigned char *stg) {
        if constexpr (sizeof(TO) == 1) {
            if (cb * 32 >= co_left) return; // (a group wholly past the last channel)
#pragma unroll
            for (int bl = 0; bl < GB; ++bl) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 bq = *reinterpret_cast<const float4 *>(bias_s + (cb + bl) * 32 + q * 8 + half * 4);
                    uint32_t pk;
                    store4<ODT, TO>(reinterpret_cast<TO *>(&pk), a[bl][q * 4] + bq.x, a[bl][q * 4 + 1] + bq.y,
                                    a[bl][q * 4 + 2] + bq.z, a[bl][q * 4 + 3] + bq.w);
                    if (g.flags & FC_RELU) pk = relu_packed8(pk);
                    const uint32_t at = (uint32_t)l32 * 128u + (uint32_t)((bl * 2 + (q >> 1)) ^ FC_SWZ(l32)) * 16u +
                                        (uint32_t)((q & 1) * 8 + half * 4);
                    *reinterpret_cast<uint32_t *>(stg + at) = pk;
                }
            }
            __asm__ volatile("" ::: "memory");
            const bool inside = (lane & 7) < GB * 2 && cb * 32 + (lane & 7) * 16 < co_left; // this lane's 16 channels exist
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = j * 8 + (lane >> 3);
                const uint32_t at = (uint32_t)row * 128u + (uint32_t)((lane & 7) ^ FC_SWZ(row)) * 16u;
                const u32x4_t piece = *reinterpret_cast<const u32x4_t *>(stg + at);
                const int pr = st_pr[0][j];
                if (pr >= 0 && inside)
                    *reinterpret_cast<u32x4_t *>(out + (int64_t)pr * g.c_out + co0 + cb * 32 + (lane & 7) * 16) = piece;
            }
            __asm__ volatile("" ::: "memory");
        }
    };

    // ---- the pipeline: stage t = (unit t / kch, chunk t % kch) lives in ring buffer t % 2, and
    // stage t + 1 is issued when stage t is about to be consumed ----
    if (nu > 0) {
        issue_idx(0);
        if constexpr (TAPS == 9) presetup(0);
        setup(0, 0);
        if (nu > 1) issue_idx(1);
        issue_x(0, 0, 0);
    }
    f32x16_t acc[GB];
    int buf = 0;
    for (int u = 0; u < nu; ++u) {
        const int p_mine = st_p[0];
#pragma unroll(KCT ? KCT : 1)
        for (int c = 0; c < kch; ++c) {
            // a stage goes out first, into the buffer freed last: the next chunk of this unit, or
            // the first chunk of the next unit (whose rows are looked up before it)
            const int bufn = buf ^ 1;
            if (c + 1 < kch) {
                issue_x(0, c + 1, bufn);
                if constexpr (TAPS == 9) {
                    // the next unit's list entries have long arrived: its mask bytes go out now,
                    // and the entries of the unit after it
                    if (c == 0 && u + 1 < nu) {
                        presetup(u + 1);
                        if (u + 2 < nu) issue_idx(u + 2);
                    }
                }
            } else if (u + 1 < nu) {
                setup(u + 1, 1);
                if constexpr (TAPS == 1) {
                    if (u + 2 < nu) issue_idx(u + 2);
                }
                issue_x(1, 0, bufn);
            }
            pw_wait_vmcnt(issued - (buf == 0 ? mark_x[0] : mark_x[1]));
            const unsigned char *xs = my + (size_t)buf * kPwChunkBytes;
            Frag<DT> xf[KK];
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) xf[kk].load(xs, frag ^ ((uint32_t)kk * KSTEP));
#pragma unroll
            for (int gb = 0; gb < NCB; gb += GB) {
                if (c == 0 || NCB > GB) {
#pragma unroll
                    for (int b = 0; b < GB; ++b)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
                }
                const unsigned char *ws = smem_raw + (size_t)(c * COUT + gb * 32) * 128u;
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    Frag<DT> wf[GB];
#pragma unroll
                    for (int b = 0; b < GB; ++b) wf[b].load(ws + b * 4096, frag ^ ((uint32_t)kk * KSTEP));
#pragma unroll
                    for (int b = 0; b < GB; ++b) acc[b] = mfma32<DT>(wf[b], xf[kk], acc[b]);
                }
                if (c == kch - 1) {
                    if constexpr (sizeof(TO) == 2) {
#pragma unroll
                        for (int b = 0; b < GB; b += 2)
                            store_pair(acc[b], acc[b + 1], gb + b, my + (size_t)buf * kPwChunkBytes);
                    } else if constexpr (sizeof(TO) == 1) {
                        store_bytes(acc, gb, my + (size_t)buf * kPwChunkBytes);
                    } else {
#pragma unroll
                        for (int b = 0; b < GB; ++b) store_block(acc[b], gb + b, p_mine);
                    }
                }
            }
            buf ^= 1;
        }
        st_p[0] = st_p[1];
#pragma unroll
        for (int j = 0; j < 4; ++j) st_off[0][j] = st_off[1][j], st_pr[0][j] = st_pr[1][j], st_val[0][j] = st_val[1][j];
    }

    // ---- zero-fill of the irrelevant output rows.  An item is 64 consecutive positions, or one
    // of `parts` interleaved shares of their 16-byte pieces when there are fewer such blocks than
    // waves (wide rows, few positions); a wave goes on to its items as soon as its own units are
    // done and lists the dropped positions of a block in its own (now idle) chunk buffer ----
    if (mask_in && !(g.flags & FC_SKIP_ZERO_FILL) && !compact_out) {
        int32_t *dropped = reinterpret_cast<int32_t *>(my);
        u32x4_t *o4 = reinterpret_cast<u32x4_t *>(out);
        const u32x4_t zero4 = {0u, 0u, 0u, 0u};
        const int cpr = g.c_out * (int)sizeof(TO) / 16; // 16-byte pieces per row
        const int workers = (int)gridDim.x * nw;
        const int nblocks = (g.m + 63) >> 6;
        const int parts = min(max(workers / nblocks, 1), 16);
        for (int item = (int)blockIdx.x * nw + wave; item < nblocks * parts; item += workers) {
            const int blk = item / parts, part = item - blk * parts;
            const int pp = blk * 64 + lane;
            bool kept = true; // (positions past the end count as kept: nothing to clear)
            if (pp < g.m) {
                if (mask_out) {
                    kept = mask_at(mask_out, pp, packed_masks);
                } else {
                    const int q = (int)fast_div((uint32_t)pp, dv.wo);
                    const int ow = pp - q * g.wo;
                    const int b = (int)fast_div((uint32_t)q, dv.ho);
                    const int oh = q - b * g.ho;
                    // (the centre tap, clamped into the image)
                    const int ihc = min(max(oh * g.sh - g.ph + g.dh * ((g.kh - 1) / 2), 0), g.h - 1);
                    const int iwc = min(max(ow * g.sw - g.pw + g.dw * ((g.kw - 1) / 2), 0), g.w - 1);
                    kept = mask_at(mask_in, (int64_t)(b * g.h + ihc) * g.w + iwc, packed_masks);
                }
            }
            const uint64_t drop = __ballot(!kept);
            if (!kept) dropped[__popcll(drop & ((1ull << lane) - 1ull))] = pp; // in position order
            const int total = __popcll(drop) * cpr;
            for (int c = part * 64 + lane; c < total; c += parts * 64) {
                const int rk = (int)fast_div((uint32_t)c, dv.cpr), pc = c - rk * cpr;
                __builtin_nontemporal_store(zero4, o4 + (int64_t)dropped[rk] * cpr + pc);
            }
        }
    }
}

// ---------------------------------------------------------------------------

constexpr uint32_t kPwLdsBytes = 160u * 1024u;

// 32-channel blocks in a workgroup's slice of the output channels, 0 if the layer does not fit.
// A layer of one input chunk takes slices of up to 256 channels (a row's accumulators are then
// computed in two halves) and so reads every row once for up to 256 output channels; with more
// chunks all accumulators of a row are live at once and a slice is 128 channels, or 64 where
// 128 would not leave room for eight waves beside the weights.
// 3x3 layers whose pixels are one chunk (128 bytes) run as the 1x1 layer of their nine-pixel
// patches: nine chunks, slices of 64 output channels (72 KB of weights)
static bool pw_is_3x3(const Geom &g, int es) { return g.kh == 3 && g.kw == 3 && g.c_in * es == 128; }

static int pw_slice_blocks(const Geom &g, int es)
{
    if (pw_is_3x3(g, es)) return 2;
    const int kch = (g.c_in * es + 127) / 128; // chunks of 128 bytes
    if (kch == 1) return g.c_out <= 64 ? 2 : g.c_out <= 128 ? 4 : 8;
    for (int ncb = g.c_out <= 64 ? 2 : 4; ncb >= 2; ncb -= 2)
        if ((uint32_t)kch * ncb * 32u * 128u + 1024u + 8u * pw_wave_bytes(2) <= kPwLdsBytes) return ncb;
    return 0;
}

static int pw_grid()
{
    // one workgroup per CU (the count is read once per process; all devices of a node are alike)
    static std::atomic<int> cus{0};
    int v = cus.load(std::memory_order_relaxed);
    if (v == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            v = prop.multiProcessorCount;
        if (v <= 0) v = 256;
        v &= ~7; // a multiple of the XCD count
        if (v < 8) v = 8;
        cus.store(v, std::memory_order_relaxed);
    }
    return v;
}

bool conv_pw_supported(const Geom &g, int in_dtype, int out_dtype)
{
    if (in_dtype != FC_BF16 && in_dtype != FC_F16 && in_dtype != FC_FP8) return false;
    if (out_dtype != (in_dtype == FC_FP8 ? FC_BF16 : in_dtype) && out_dtype != FC_F32 && out_dtype != FC_FP8) return false;
    const int es = in_dtype == FC_FP8 ? 1 : 2;
    if (!(g.kh == 1 && g.kw == 1 && g.ph == 0 && g.pw == 0) && !pw_is_3x3(g, es)) return false;
    if (pw_is_3x3(g, es) && (g.flags & FC_COMPACT_IN)) return false;
    // rows of whole 16-byte pieces on both sides
    if (g.c_in * es < 16 || (g.c_in * es) % 16 != 0 || g.c_out < 8 || g.c_out % 8 != 0) return false;
    if (out_dtype == FC_FP8 && g.c_out % 16 != 0) return false;
    const int ncb = pw_slice_blocks(g, es);
    if (ncb == 0) return false;
    // the slices of a group of workgroups sit on one XCD
    const int n_slices = (g.c_out + ncb * 32 - 1) / (ncb * 32), per_xcd = pw_grid() >> 3;
    if (n_slices > per_xcd) return false;
    if ((uint64_t)g.n * g.h * g.w * g.c_in * (uint64_t)es >= kBufferLimit) return false;
    if ((uint64_t)g.c_out * g.c_in * (uint64_t)es >= kBufferLimit) return false;
    if ((uint64_t)g.m * 4u >= kBufferLimit) return false; // the list goes through a descriptor as well
    return true;
}

template <int DT, typename TO, int NCB, int KCT, int TAPS = 1>
static hipError_t launch_pw(const Geom &g, const void *x, const uint8_t *mask_in, const uint8_t *mask_out,
                            const void *w, const float *bias, const int32_t *idx, const int32_t *count, void *out,
                            hipStream_t s)
{
    // twelve waves per CU where the weights leave room for their buffers, else eight
    constexpr int es = DT == FC_FP8 ? 1 : 2;
    const int kch = TAPS * ((g.c_in * es + 127) / 128);
    const uint32_t wbytes = (uint32_t)kch * NCB * 32u * 128u;
    const int fit = (int)((kPwLdsBytes - wbytes - 1024u) / pw_wave_bytes_of(2, TAPS));
    if (fit < 8) return hipErrorInvalidValue;
    const int nw = fit >= 12 ? 12 : 8;
    const size_t lds = wbytes + 1024u + (size_t)nw * pw_wave_bytes_of(2, TAPS);
    auto kern = k_conv_pw<DT, TO, NCB, KCT, TAPS>;
    PwDivs dv;
    dv.wo = make_fastdiv((uint32_t)g.wo);
    dv.ho = make_fastdiv((uint32_t)g.ho);
    dv.cpr = make_fastdiv((uint32_t)g.c_out * (uint32_t)sizeof(TO) / 16u);
    // the dynamic LDS limit is raised once per function and device
    static std::atomic<uint64_t> attr_devices{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t dev_bit = 1ull << (dev & 63);
    if (!(attr_devices.load(std::memory_order_acquire) & dev_bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)kPwLdsBytes);
        if (e != hipSuccess) return e;
        attr_devices.fetch_or(dev_bit, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(pw_grid()), dim3(nw * 64), lds, s, g, dv, kch, (const unsigned char *)x, mask_in, mask_out,
                       (const unsigned char *)w, bias, idx, count, (TO *)out);
    return hipGetLastError();
}

template <int DT, typename TO>
static hipError_t launch_pw_shape(const Geom &g, const void *x, const uint8_t *mask_in, const uint8_t *mask_out,
                                  const void *w, const float *bias, const int32_t *idx, const int32_t *count,
                                  void *out, hipStream_t s)
{
#define FC_PW_ARGS g, x, mask_in, mask_out, w, bias, idx, count, out, s
    constexpr int es = DT == FC_FP8 ? 1 : 2;
    if (pw_is_3x3(g, es)) return launch_pw<DT, TO, 2, 9, 9>(FC_PW_ARGS);
    const int ncb = pw_slice_blocks(g, es), kch = (g.c_in * es + 127) / 128;
    if (ncb == 8) return launch_pw<DT, TO, 8, 1>(FC_PW_ARGS);
    if (ncb == 4) {
        if (kch == 1) return launch_pw<DT, TO, 4, 1>(FC_PW_ARGS);
        if (kch == 2) return launch_pw<DT, TO, 4, 2>(FC_PW_ARGS);
        if (kch == 4) return launch_pw<DT, TO, 4, 4>(FC_PW_ARGS);
        return launch_pw<DT, TO, 4, 0>(FC_PW_ARGS);
    }
    if (ncb == 2) {
        if (kch == 1) return launch_pw<DT, TO, 2, 1>(FC_PW_ARGS);
        if (kch == 2) return launch_pw<DT, TO, 2, 2>(FC_PW_ARGS);
        if (kch == 4) return launch_pw<DT, TO, 2, 4>(FC_PW_ARGS);
        if (kch == 8) return launch_pw<DT, TO, 2, 8>(FC_PW_ARGS);
        return launch_pw<DT, TO, 2, 0>(FC_PW_ARGS);
    }
    return hipErrorInvalidValue;
#undef FC_PW_ARGS
}

hipError_t launch_conv_pw(const Geom &g, int in_dtype, int out_dtype, const void *x, const uint8_t *mask_in,
                          const uint8_t *mask_out, const void *w, const float *bias, const int32_t *idx,
                          const int32_t *count, void *out, hipStream_t s)
{
#define FC_PW_CALL(DT, TO) launch_pw_shape<DT, TO>(g, x, mask_in, mask_out, w, bias, idx, count, out, s)
    if (in_dtype == FC_BF16) {
        if (out_dtype == FC_F32) return FC_PW_CALL(FC_BF16, float);
        if (out_dtype == FC_FP8) return FC_PW_CALL(FC_BF16, uint8_t);
        return FC_PW_CALL(FC_BF16, uint16_t);
    }
    if (in_dtype == FC_FP8) {
        if (out_dtype == FC_F32) return FC_PW_CALL(FC_FP8, float);
        if (out_dtype == FC_FP8) return FC_PW_CALL(FC_FP8, uint8_t);
        return FC_PW_CALL(FC_FP8, uint16_t);
    }
    if (out_dtype == FC_F32) return FC_PW_CALL(FC_F16, float);
    if (out_dtype == FC_FP8) return FC_PW_CALL(FC_F16, uint8_t);
    return FC_PW_CALL(FC_F16, uint16_t);
#undef FC_PW_CALL
}

} // namespace fc
