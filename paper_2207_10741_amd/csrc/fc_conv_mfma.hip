// Focused convolution on the gfx950 matrix cores (Sec. III-A: a GEMM over the
// kept patches only, with the dense layer's weights).
//
// GEMM view: rows = kept output positions (from the index list), reduction
// K = (tap, input channel), columns = output channels.  The patch matrix is never
// stored: for every (tap, 128-byte chunk of channels) = one pipeline stage, the workgroup
// gathers, for each of its TM positions, the 128 contiguous bytes of that tap's NHWC
// pixel into LDS (zeros where the tap falls outside the image or on an irrelevant
// input pixel), next to the TN x 128-byte slab of weights for the same tap, and feeds
// both to the matrix cores with fp32 accumulators: v_mfma_f32_32x32x16 for bf16 / f16
// storage (64 channels per stage, four instructions per 32 x 32 block), and
// v_mfma_f32_32x32x64_f8f6f4 for 8-bit E4M3 storage (128 channels per stage, two
// instructions of twice the length).  Everything outside the multiply itself - gather,
// swizzle, pipeline, epilogue - moves bytes and is the same code for both.
//
// Data path.  The gathers go straight from global memory into LDS ("buffer_load ...
// lds", 16 bytes per lane) without passing through registers: measured on this chip a
// 128-bit LDS write from registers costs three times a 128-bit LDS read, and staging
// through registers also serialises the workgroup behind bursts of loads.  A wave-wide
// load writes 64 x 16 contiguous bytes of LDS, i.e. 8 tile rows of 128 bytes with no
// padding; bank conflicts on the fragment reads are avoided instead by an XOR swizzle
// applied on the global side: LDS slot c of row r holds the row's 16-byte piece
// c ^ ((r >> 1) & 7).  The loads are issued from inline assembly and waited for with
// explicit s_waitcnt vmcnt(N), so that NB-1 stages stay in flight while one is being
// multiplied (left to itself the compiler drains every outstanding LDS-bound load
// before each LDS read).  A gated lane (padding, irrelevant input pixel, channel
// tail, stage past the end) gets an offset that is out of range for its buffer
// descriptor, for which the hardware writes zeros without touching memory; nothing
// in the gather branches.
//
// The weights are the MFMA's A operand (rows = output channel) and the gathered
// activations its B operand (columns = position), so a lane's accumulators hold 4
// consecutive output channels of one position.  The accumulators start from the bias;
// the epilogue rounds once to the output type, applies ReLU, transposes the tile
// through LDS and stores each kept row as whole 16-byte pieces.  The same kernel clears
// the irrelevant rows (the workgroups that have no tile do it).
//
// The launch grid never depends on the kept count: workgroups stride over the tiles
// and read the count on the device.  Layers with few tiles split every tile's reduction
// over several workgroups, which meet through fp32 partial tiles in the workspace; the
// one that arrives last adds them in a fixed order and writes the tile.
#include "fc_dma_util.hpp"
#include <type_traits>
#include <atomic>

namespace fc {

constexpr int kMaxSplits = 16;                 // most K-splits of one tile
constexpr int kMinSplitStages = 8;            // fewest stages a K-split is left with
constexpr int kBusySplitStages = 64;          // shortest reduction that is split on a busy chip
constexpr int kSmallLayerTiles = 64;  // layers with at most this many 128 x 64 tiles use 64 x 64 tiles
[[maybe_unused]] constexpr int kMaxTaps = 32;                   // tap-valid bits per row live in one 32-bit word

// Bytes of the LDS stage region: NB buffers of (TM + TN) rows for the tap-by-tap loop; with the
// shared-halo loop (SL > 0) also room for two buffers of SL pixel slots and NBW weight buffers.
template <int TM, int TN, int NB, int SL, int NBW>
constexpr size_t dma_stage_region_bytes()
{
    const size_t classic = (size_t)NB * (TM + TN) * 128;
    const size_t halo = SL > 0 ? (size_t)2 * SL * 128 + (size_t)NBW * TN * 128 : 0;
    return classic > halo ? classic : halo;
}

template <int TM, int TN, int NB, int SL, int NBW>
constexpr size_t dma_lds_bytes()
{
    return dma_stage_region_bytes<TM, TN, NB, SL, NBW>() + (size_t)TM * 5 * sizeof(int32_t) +
           (SL > 0 ? (size_t)(TM + 3 * SL + 8) * sizeof(int32_t) : 0);
}

// DT: storage type of x and w; TO: float or a 16-bit carrier; TM x TN: workgroup tile
// (positions x output channels); WM x WN: wave grid inside it; TAPC: 1 (1x1 kernels),
// 9 (3x3 kernels) or 32 (any kernel of up to 32 taps); NB: LDS stage buffers (NB-1
// stages of loads in flight); MINW: waves per SIMD the register budget leaves room for.
//
// SL > 0 (3x3 kernels with unit horizontal stride and dilation only) adds the shared-halo
// loop.  The three horizontal taps of a kept position read the pixels left of, at and right
// of its centre column, and the kept positions of a tile are sorted, so along a run of
// horizontally adjacent kept positions the left pixel of one is the centre pixel of the one
// before it.  The tile therefore lays its pixels out on a line of "slots": one per kept
// position, plus one before the first and one after the last position of every run; position
// r's taps kw = 0, 1, 2 are then slots cs(r) - 1, cs(r), cs(r) + 1.  For every (kernel row,
// 64-channel chunk) the line is gathered into LDS once and multiplied three times, each time
// against the weights of another horizontal tap, which cuts the gathered bytes by up to three.
// A tile whose line would need more than SL slots (a fragmented mask) runs the tap-by-tap
// loop instead.  NBW: LDS buffers for the per-tap weight slabs of the shared-halo loop.
//
// CMP: the instances that serve compacted activations (FC_COMPACT_IN / FC_COMPACT_OUT: rows
// stored in list order).  Separate instances, so that the ordinary ones do not change by a
// register: the 128 x 64 three-buffer instance loses 20 % with a handful more.
template <int DT, typename TO, int TM, int TN, int WM, int WN, int TAPC, int NB, int MINW, int SL, int NBW, bool CMP>
__global__ __launch_bounds__(WM *WN * 64, MINW) void k_conv_dma(Geom g, const uint16_t *__restrict__ x,
                                                                 const uint8_t *__restrict__ mask_in,
                                                                 const uint8_t *__restrict__ mask_out,
                                                                 const uint16_t *__restrict__ w,
                                                                 const float *__restrict__ bias,
                                                                 const int32_t *__restrict__ idx,
                                                                 const int32_t *__restrict__ count,
                                                                 TO *__restrict__ out,
                                                                 float *__restrict__ partials,
                                                                 int32_t *__restrict__ tile_counters)
{
    constexpr int NT = WM * WN * 64;
    constexpr int RPP = NT / 8;        // rows covered by one pass of wave loads
    constexpr int XR = TM / RPP;       // wave loads per thread for the activation tile
    constexpr int WR = TN / RPP;       // ... for the weight tile
    constexpr int L = XR + WR;         // loads per thread per stage
    constexpr int WTM = TM / WM, WTN = TN / WN;
    constexpr int PB = WTM / 32, CB = WTN / 32;
    constexpr int ES = DT == FC_FP8 ? 1 : 2;               // bytes per stored element
    constexpr int TK = kStageBytes / ES;                   // reduction elements per stage
    constexpr int EPP = 16 / ES;                           // elements per 16-byte piece
    constexpr uint32_t KSTEP = kStepBytes<DT>;             // bytes of a row per matrix instruction
    constexpr int KK = kStageBytes / (int)KSTEP;           // matrix instructions per stage and block pair
    constexpr int ODT = DT == FC_FP8 ? FC_BF16 : DT;       // 16-bit output format
    // register sets of operand fragments: the 16-bit types fetch step kk + 1 while step kk is
    // multiplied; fp8 fragments are twice as large and its instructions twice as long, so one set,
    // refilled behind the multiplies of a step, keeps the kernel inside the register file
    constexpr int FB = (DT == FC_FP8 && TM * TN >= 128 * 128) ? 1 : 2;
    constexpr int PAIR_IT = (TM * TAPC + NT - 1) / NT;
    constexpr int PAIR_CH = PAIR_IT < 5 ? PAIR_IT : 5;
    constexpr int STAGE_BYTES = (TM + TN) * 128;
    static_assert(TM % RPP == 0 && TN % RPP == 0 && WTM % 32 == 0 && WTN % 32 == 0, "tile shape");
    static_assert(TM <= NT && TN <= NT, "set-up assumes one thread per row / channel");
    static_assert(NB >= 2 && (NB - 1) * L <= 63, "vmcnt is a 6-bit counter");
    constexpr bool HALO = SL > 0;
    constexpr size_t REGION = dma_stage_region_bytes<TM, TN, NB, SL, NBW>();
    static_assert(!HALO || (TAPC == 9 && SL % RPP == 0 && SL <= NT && SL > TM && (NBW == 2 || NBW == 3)),
                  "shared-halo loop: 3x3 kernels, whole load passes, one thread per slot");

    extern __shared__ __align__(16) unsigned char smem_raw[];
    unsigned char *stage0 = smem_raw;                                   // [NB][TM + TN][128]
    int32_t *row_p = reinterpret_cast<int32_t *>(smem_raw + REGION);
    int32_t *row_base = row_p + TM;
    int32_t *row_img = row_base + TM;
    int32_t *row_hw = row_img + TM;
    uint32_t *row_bits = reinterpret_cast<uint32_t *>(row_hw + TM);
    // shared-halo loop only: centre slot of every row, and per slot the pixel of kernel row 0,
    // its packed (ih, iw) and one "inside the image and relevant" bit per kernel row
    int32_t *row_cs = reinterpret_cast<int32_t *>(row_bits + TM);
    int32_t *slot_pix = row_cs + TM;
    int32_t *slot_hw = slot_pix + SL;
    uint32_t *slot_bits = reinterpret_cast<uint32_t *>(slot_hw + SL);
    int32_t *scan_part = reinterpret_cast<int32_t *>(slot_bits + SL);
    const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>(smem_raw); // LDS byte address of the stage buffers

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave % WM, wave_n = wave / WM;
    const int slot = tid & 7, prow = tid >> 3;

    // Kept rows.  With a list they are given.  Without one but with a mask (the launcher does
    // this only for layers of at most 16 positions per thread) the workgroup ranks the kept
    // positions itself: thread t labels positions 16t .. 16t+15 (centre tap, Sec. III-B) and a
    // prefix sum over the workgroup gives the rank of its first kept position; the set-up of a
    // tile then has every thread drop its positions of that tile's rank range into row_p.  A
    // small layer so needs no compaction launch before this one.
    const bool packed_masks = (g.flags & FC_PACKED_MASKS) != 0; // masks are one bit per pixel
    const bool inline_rank = !idx && mask_in;
    uint32_t rank_flags = 0;
    int rank_base = 0;
    int rows = g.m;
    if (inline_rank) {
        MaskGeom mg = mask_geom(g.n, g.h, g.w, g.kh, g.kw, g.sh, g.sw, g.ph, g.pw, g.dh, g.dw, g.ho, g.wo);
        mg.packed_in = (g.flags & FC_PACKED_MASKS) ? 1 : 0;
        if (!mg.packed_in && (reinterpret_cast<uintptr_t>(mask_in) & 15u)) mg.identity = 0; // the 128-bit path needs alignment
        rank_flags = kept_flags16(mg, mask_in, (int64_t)tid * 16);
        const int cnt = __popc(rank_flags);
        const int incl = wave_inclusive_scan(cnt);
        if (lane == 63) row_p[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int v = 0; v < NT / 64; ++v) {
            const int t = row_p[v];
            before += v < wave ? t : 0;
            total += t;
        }
        rank_base = before + incl - cnt;
        rows = total;
        __syncthreads(); // row_p is free again
    } else if (idx) {
        rows = *count;
    }
    const int n_nt = (g.c_out + TN - 1) / TN;
    const int ntiles = ((rows + TM - 1) / TM) * n_nt;
    const int taps = TAPC == 32 ? g.kh * g.kw : TAPC;
    const int kwid = TAPC == 32 ? g.kw : (TAPC == 9 ? 3 : 1);
    const int cchunks = (g.c_in + TK - 1) / TK;
    const int stages = taps * cchunks;
    const bool self_tap = TAPC == 1 && g.ph == 0 && g.pw == 0;
    const u32x4_t rsrc_x = make_rsrc_words(x, (uint32_t)g.n * g.h * g.w * g.c_in * (uint32_t)ES);
    const u32x4_t rsrc_w = make_rsrc_words(w, (uint32_t)g.c_out * taps * g.c_in * (uint32_t)ES);

    // fragment addressing: lane reads row (lane & 31) of a 32-row block; in step kk that is
    // the 16-byte piece 2*kk + (lane >> 5) (fp8: the pieces 4*kk + 2*(lane >> 5) and the one
    // after it), stored at slot piece ^ ((row >> 1) & 7); all block bases are multiples of 32
    // rows, so the swizzle term depends on the lane only
    constexpr uint32_t HALF = KSTEP / 32u; // piece index of the upper half-wave within a step
    const uint32_t frag_row = (uint32_t)(lane & 31) * 128u;
    const uint32_t frag_t16 = (uint32_t)(((lane >> 5) * HALF) ^ FC_SWZ(lane & 31)) * 16u;

    // Tile order: all row tiles of channel tile 0, then of channel tile 1, ...  Workgroups
    // are dispatched round-robin over the 8 XCDs, each with its own L2, so XCD j takes the
    // j-th contiguous eighth of that order: its tiles share one weight slab and
    // neighbouring image rows (the halo of the 3x3 taps) in that L2.
    const int n_mt = (rows + TM - 1) / TM;
    // Split-K: when there are fewer tiles than workgroups (small layers, or few kept rows)
    // the reduction of every tile is cut into S equal runs of stages, one work unit each, so
    // that the serial K loop of a workgroup gets S times shorter and the chip fills up.
    // Units of one tile are adjacent in the order, so they share an XCD.  S is the same in
    // every workgroup (it depends on the kept count and the grid only).
    int S = 1;
    if (partials && ntiles > 0) {
        S = (int)gridDim.x / ntiles;
        const int work = HALO ? g.kh * cchunks : stages; // (kernel row, chunk) groups or stages
        S = S < 1 ? 1 : (S > work ? work : S);
        if (S > kMaxSplits) S = kMaxSplits;
        // the exchange of partial tiles costs about as much as twenty stages, so a unit keeps at
        // least kMinSplitStages of them: short reductions are not split at all (a 3x3 layer with
        // 64 input channels: 8.4 us unsplit against 19.3 us split three ways)
        const int s_cap = stages / kMinSplitStages;
        if (S > s_cap) S = s_cap < 1 ? 1 : s_cap;
        // when the tiles alone already fill more than a quarter of the grid, the exchange also
        // competes with the other tiles' traffic and only long reductions gain (512 channels at
        // 16 x 16, batch 16: 72 stages split three ways 31 -> 26 us, 36 stages 20 -> 28 us)
        if (ntiles * 4 > (int)gridDim.x && stages < kBusySplitStages) S = 1;
    }
    const int nunits = ntiles * S;
    const int per_xcd = (nunits + 7) >> 3;
    const int xcd = blockIdx.x & 7;

    // ---- zero-fill of the irrelevant output rows (none for the dense layer) ----
    // The grid is sized for the dense row count, so with a kept share r about 1 - r of
    // the workgroups have no tile: when there are enough of them they alone clear the
    // irrelevant rows (about one tile's worth of rows each, off the critical path of the
    // tiles); otherwise every workgroup clears its share before its tiles.  A wave looks
    // at 64 positions at a time and stores whole 16-byte pieces with all lanes.
    if (mask_in && !(g.flags & FC_SKIP_ZERO_FILL)) {
        const int slots = gridDim.x >> 3;
        const int idle_slots = slots > per_xcd ? slots - per_xcd : 0;
        const bool idle_only = idle_slots > 0 && idle_slots * 8 >= (int)(gridDim.x >> 4);
        const int my_slot = blockIdx.x >> 3;
        if (!idle_only || my_slot >= per_xcd) {
            const int nworkers = (idle_only ? idle_slots * 8 : (int)gridDim.x) * (NT / 64);
            const int worker = (idle_only ? (my_slot - per_xcd) * 8 + xcd : (int)blockIdx.x) * (NT / 64) + wave;
            int32_t *dropped = reinterpret_cast<int32_t *>(smem_raw) + wave * 64; // per-wave list
            const int cpr = g.c_out * (int)sizeof(TO) / 16; // 16-byte pieces per row
            u32x4_t *o4 = reinterpret_cast<u32x4_t *>(out);
            const u32x4_t zero4 = {0u, 0u, 0u, 0u};
            const int ch0 = -g.ph + g.dh * ((g.kh - 1) / 2), cw0 = -g.pw + g.dw * ((g.kw - 1) / 2);
            for (int p0 = worker * 64; p0 < g.m; p0 += nworkers * 64) {
                const int pp = p0 + lane;
                bool kept = true;
                if (pp < g.m) {
                    if (mask_out) {
                        kept = mask_at(mask_out, pp, packed_masks);
                    } else {
                        const int ow = pp % g.wo;
                        const int q = pp / g.wo;
                        const int oh = q % g.ho;
                        const int b = q / g.ho;
                        const int ih = min(max(oh * g.sh + ch0, 0), g.h - 1);
                        const int iw = min(max(ow * g.sw + cw0, 0), g.w - 1);
                        kept = mask_at(mask_in, (int64_t)(b * g.h + ih) * g.w + iw, packed_masks);
                    }
                }
                const uint64_t drop = __ballot(!kept);
                const int nd = __popcll(drop);
                if (!kept) dropped[__popcll(drop & ((1ull << lane) - 1ull))] = pp; // in position order
                // (same wave wrote and reads the list: program order suffices)
                const int total = nd * cpr;
                for (int c = lane; c < total; c += 64) {
                    const int rk = c / cpr, pc = c - rk * cpr;
                    __builtin_nontemporal_store(zero4, o4 + (int64_t)dropped[rk] * cpr + pc);
                }
            }
        }
    }
    for (int slot_t = blockIdx.x >> 3; slot_t < per_xcd; slot_t += gridDim.x >> 3) {
        const int unit = xcd * per_xcd + slot_t;
        if (unit >= nunits) break;
        const int tile = unit / S, split = unit - tile * S;
        const int s_begin = (int)((int64_t)split * stages / S), s_end = (int)((int64_t)(split + 1) * stages / S);
        const int nst = s_end - s_begin; // stages of this unit
        const int nt = tile / n_mt, mt = tile - nt * n_mt;
        const int co0 = nt * TN;

        __syncthreads(); // the previous tile's epilogue is done with LDS
        if (inline_rank) {
            // every thread drops its kept positions whose rank falls into this tile
            if (tid < TM) row_p[tid] = -1;
            __syncthreads();
            const int lo = mt * TM;
            int r = rank_base;
            uint32_t f = rank_flags;
            if (r < lo + TM && r + __popc(f) > lo) {
                while (f) {
                    const int j = __ffs((int)f) - 1;
                    f &= f - 1;
                    if (r >= lo && r < lo + TM) row_p[r - lo] = tid * 16 + j;
                    ++r;
                }
            }
            __syncthreads();
        }
        int sa_p = -1, sa_ow = 0, sa_ih0 = 0, sa_iw0 = 0, sa_b = 0; // this thread's row (tid < TM)
        if (tid < TM) {
            const int m = mt * TM + tid;
            int p = -1, base = 0, b = 0, hw = 0;
            if (m < rows) {
                p = inline_rank ? row_p[tid] : (idx ? idx[m] : m);
                const int ow = p % g.wo;
                const int q = p / g.wo;
                const int oh = q % g.ho;
                b = q / g.ho;
                const int ih0 = oh * g.sh - g.ph, iw0 = ow * g.sw - g.pw;
                sa_p = p; sa_ow = ow; sa_ih0 = ih0; sa_iw0 = iw0; sa_b = b;
                base = (b * g.h + ih0) * g.w + iw0;
                // compacted input (1x1, unit stride, no padding): the row's pixel is row m of x
                if constexpr (CMP) {
                    if (g.flags & FC_COMPACT_IN) base = m;
                }
                hw = (int)(((uint32_t)ih0 & 0xffffu) | ((uint32_t)iw0 << 16));
            }
            row_p[tid] = p;
            row_base[tid] = base;
            row_img[tid] = b;
            row_hw[tid] = hw;
            // an unpadded 1x1 kernel reads exactly the pixel that decided to keep the position:
            // inside the image and relevant by construction, nothing to look up
            row_bits[tid] = (self_tap && p >= 0) ? 1u : 0u;
        }
        // The accumulators start from the bias (in the first K-split only), so the epilogue has
        // nothing to add: every lane fetches the bias of its own channels now and the loads
        // are long back when the set-up is done.
        float4 bias_q[CB][4];
#pragma unroll
        for (int b = 0; b < CB; ++b)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int co = co0 + wave_n * WTN + b * 32 + q * 8 + (lane >> 5) * 4;
                bias_q[b][q] = (bias && split == 0 && co < g.c_out) ? *reinterpret_cast<const float4 *>(bias + co)
                                                                    : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        __syncthreads();
        bool use_halo = false;
        int ns = 0; // slots on this tile's pixel line
        if constexpr (HALO) {
            int cnt = 0, lead = 0;
            bool ladj = false, radj = false;
            if (tid < TM) {
                cnt = 1;
                if (sa_p >= 0) {
                    ladj = tid > 0 && row_p[tid - 1] == sa_p - 1 && sa_ow > 0;
                    radj = tid < TM - 1 && row_p[tid + 1] == sa_p + 1 && sa_ow < g.wo - 1;
                    lead = ladj ? 0 : 1;
                    cnt = 1 + lead + (radj ? 0 : 1);
                }
            }
            const int incl = wave_inclusive_scan(cnt);
            if (lane == 63) scan_part[wave] = incl;
            if (tid < SL) slot_bits[tid] = 0;
            __syncthreads();
            int before = 0;
#pragma unroll
            for (int v = 0; v < NT / 64; ++v) {
                const int t = scan_part[v];
                before += v < wave ? t : 0;
                ns += t;
            }
            // (one slot to spare: a row past the end of the list still reads "its" three slots)
            use_halo = ns + 1 <= SL;
            if (use_halo && tid < TM) {
                const int cs = before + incl - cnt + lead;
                row_cs[tid] = cs;
                if (sa_p >= 0) {
                    const int iwc = sa_iw0 + 1; // kw = 1, unit dilation
                    const int pixc = (sa_b * g.h + sa_ih0) * g.w + iwc;
                    const int ih16 = (int)((uint32_t)sa_ih0 & 0xffffu);
                    slot_pix[cs] = pixc;
                    slot_hw[cs] = ih16 | (int)((uint32_t)iwc << 16);
                    if (!ladj) {
                        slot_pix[cs - 1] = pixc - 1;
                        slot_hw[cs - 1] = ih16 | (int)((uint32_t)(iwc - 1) << 16);
                    }
                    if (!radj) {
                        slot_pix[cs + 1] = pixc + 1;
                        slot_hw[cs + 1] = ih16 | (int)((uint32_t)(iwc + 1) << 16);
                    }
                } else {
                    slot_pix[cs] = 0;
                    slot_hw[cs] = (int)((uint32_t)(-20000) << 16); // never inside an image
                }
            }
            __syncthreads();
            if (use_halo) {
                // one thread per (slot, kernel row): inside the image and relevant?
                constexpr int SIT = (SL * 3 + NT - 1) / NT;
                int ssl_[SIT], skh_[SIT], spix_[SIT];
                bool sin_[SIT];
#pragma unroll
                for (int i = 0; i < SIT; ++i) {
                    const int pair = tid + i * NT;
                    const int sl = pair / 3, kh_i = pair - sl * 3;
                    const bool live = sl < ns;
                    const int s2 = live ? sl : 0;
                    const int hw = slot_hw[s2];
                    const int ih = (int)(int16_t)(hw & 0xffff) + kh_i * g.dh;
                    const int iw = hw >> 16;
                    const bool inb = live && ih >= 0 && ih < g.h && iw >= 0 && iw < g.w;
                    ssl_[i] = s2;
                    skh_[i] = kh_i;
                    sin_[i] = inb;
                    spix_[i] = inb ? slot_pix[s2] + kh_i * g.dh * g.w : 0;
                }
                uint8_t smv[SIT];
#pragma unroll
                for (int i = 0; i < SIT; ++i) smv[i] = mask_in ? (uint8_t)mask_at(mask_in, spix_[i], packed_masks) : (uint8_t)1;
#pragma unroll
                for (int i = 0; i < SIT; ++i)
                    if (sin_[i] && smv[i]) atomicOr(&slot_bits[ssl_[i]], 1u << skh_[i]);
            }
        }
        // set-up B: one thread per (row, tap) decides "inside the image and relevant" (for a
        // masked layer it fetches the mask byte under the tap; all of a thread's bytes are in
        // flight together)
        for (int i0 = 0; i0 < ((use_halo || self_tap) ? 0 : PAIR_IT); i0 += PAIR_CH) {
            int prow_[PAIR_CH], ptap_[PAIR_CH], ppix_[PAIR_CH];
            bool pin_[PAIR_CH];
#pragma unroll
            for (int i = 0; i < PAIR_CH; ++i) {
                const int pair = tid + (i0 + i) * NT;
                const int r = pair / taps, t = pair - r * taps;
                const bool live = pair < TM * taps;
                const int rr = live ? r : 0;
                const int kh = t / kwid, kw = t - kh * kwid;
                const int hw = row_hw[rr];
                const int ih = (int)(int16_t)(hw & 0xffff) + kh * g.dh;
                const int iw = (hw >> 16) + kw * g.dw;
                const bool inb = live && row_p[rr] >= 0 && ih >= 0 && ih < g.h && iw >= 0 && iw < g.w;
                prow_[i] = rr;
                ptap_[i] = t;
                pin_[i] = inb;
                ppix_[i] = inb ? (row_img[rr] * g.h + ih) * g.w + iw : 0;
            }
            uint8_t mv[PAIR_CH];
#pragma unroll
            for (int i = 0; i < PAIR_CH; ++i) mv[i] = mask_in ? (uint8_t)mask_at(mask_in, ppix_[i], packed_masks) : (uint8_t)1;
#pragma unroll
            for (int i = 0; i < PAIR_CH; ++i)
                if (pin_[i] && mv[i]) atomicOr(&row_bits[prow_[i]], 1u << ptap_[i]);
        }

        // per-thread, loop-invariant byte offsets; gp = the global 16-byte piece this lane
        // fetches for its LDS slot (the swizzle)
        uint32_t woff[WR];
        int wgp[WR];
#pragma unroll
        for (int j = 0; j < WR; ++j) {
            const int r = prow + j * RPP;
            const int co = co0 + r;
            wgp[j] = slot ^ FC_SWZ(r);
            woff[j] = co < g.c_out ? ((uint32_t)co * (uint32_t)(taps * g.c_in) + (uint32_t)wgp[j] * EPP) * ES
                                   : kOutOfRange;
        }

        f32x16_t acc[PB][CB];
#pragma unroll
        for (int a = 0; a < PB; ++a)
#pragma unroll
            for (int b = 0; b < CB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc[a][b][q * 4 + 0] = bias_q[b][q].x;
                    acc[a][b][q * 4 + 1] = bias_q[b][q].y;
                    acc[a][b][q * 4 + 2] = bias_q[b][q].z;
                    acc[a][b][q * 4 + 3] = bias_q[b][q].w;
                }

        if (HALO && use_halo) {
            // ---------------- shared-halo loop ----------------
            // LDS: two buffers of SL pixel slots, then NBW buffers of TN weight rows.  A group =
            // one (kernel row, 64-channel chunk): its pixel line is gathered once (XL wave loads
            // per thread, issued a whole group ahead), its three taps are three stages, each
            // with its own weight slab (WR wave loads per thread, issued NBW - 1 stages ahead).
            __syncthreads(); // slot_bits complete
            constexpr int XL = HALO ? SL / RPP : 1;
            constexpr uint32_t XB = (uint32_t)SL * 128u;
            constexpr uint32_t WB = (uint32_t)TN * 128u;
            // A slot's offset is that of its first kernel row, which may lie above or left of the
            // image; the load instruction adds the kernel row's offset itself and range-checks
            // the per-lane part alone, so that part must not be negative: the line is gathered
            // through a descriptor that starts (pad_h rows + pad_w pixels) before the tensor.
            // (Nothing in front of the tensor is ever read: those taps are switched off.)
            const uint32_t xbias = (uint32_t)(g.ph * g.w + g.pw) * (uint32_t)g.c_in * (uint32_t)ES;
            const u32x4_t rsrc_xb = make_rsrc_words(reinterpret_cast<const unsigned char *>(x) - xbias,
                                                    (uint32_t)g.n * g.h * g.w * g.c_in * (uint32_t)ES + xbias);
            uint32_t hxoff[XL], hxbits[XL];
            int hxgp[XL];
#pragma unroll
            for (int j = 0; j < XL; ++j) {
                const int sl = prow + j * RPP;
                hxgp[j] = slot ^ FC_SWZ(sl);
                hxoff[j] = ((uint32_t)slot_pix[sl] * (uint32_t)g.c_in + (uint32_t)hxgp[j] * EPP) * ES + xbias;
                hxbits[j] = slot_bits[sl];
            }
            // fragment addressing: the three slots of this lane's rows
            uint32_t xfa[PB][3];
#pragma unroll
            for (int a = 0; a < PB; ++a) {
                const int cs = row_cs[wave_m * WTM + a * 32 + (lane & 31)];
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    const int sl = cs + t - 1;
                    xfa[a][t] = (uint32_t)sl * 128u + (uint32_t)(((lane >> 5) * HALF) ^ FC_SWZ(sl)) * 16u;
                }
            }
            const int groups = g.kh * cchunks;
            const int g_begin = (int)((int64_t)split * groups / S), g_end = (int)((int64_t)(split + 1) * groups / S);
            const int ng = g_end - g_begin;
            // cursors: next pixel line to gather, next weight slab to fetch
            int xkh = g_begin / cchunks, xcc = g_begin - xkh * cchunks, xleft = ng;
            int wkh = xkh, wcc = xcc, wkw = 0, wleft = 3 * ng;
            uint32_t ld_off[WR + XL];
            // (buffer numbers are compile-time values throughout: the group loop is unrolled over
            // the two line buffers, so fragment and gather addresses inside LDS need no arithmetic)
            // Offsets of a stage's loads: a per-lane part (ld_off) and a wave-uniform part that the
            // load instruction adds itself (ld_sx for the line, ld_sw for the slab).  When the
            // input channels are whole 64-channel chunks the per-lane part of a weight row never
            // changes and that of a slot only depends on its tap-valid bit; with a channel tail
            // the lanes past the last channel are switched off one by one.
            const bool k_tail = (g.c_in % TK) != 0;
            uint32_t ld_sx = 0, ld_sw = 0;
#define FC_HALO_PREP_X(at)                                                                                \
    {                                                                                                     \
        const uint32_t sx = (uint32_t)((xkh * g.dh) * g.w * g.c_in + xcc * TK) * ES;                      \
        const bool in_k = xleft > 0;                                                                      \
        --xleft;                                                                                          \
        if (k_tail) {                                                                                     \
            ld_sx = 0;                                                                                    \
            _Pragma("unroll") for (int j = 0; j < XL; ++j)                                                \
            {                                                                                             \
                const bool ok = in_k && xcc * TK + hxgp[j] * EPP < g.c_in && ((hxbits[j] >> (xkh & 31)) & 1u); \
                ld_off[(at) + j] = ok ? hxoff[j] + sx : kOutOfRange;                                      \
            }                                                                                             \
        } else {                                                                                          \
            ld_sx = in_k ? sx : 0u;                                                                       \
            const uint32_t sel = in_k ? 1u << (xkh & 31) : 0u;                                            \
            _Pragma("unroll") for (int j = 0; j < XL; ++j)                                                \
                ld_off[(at) + j] = (hxbits[j] & sel) ? hxoff[j] : kOutOfRange;                            \
        }                                                                                                 \
        const int wrap = (xcc + 1 == cchunks);                                                            \
        xcc = wrap ? 0 : xcc + 1;                                                                         \
        xkh += wrap;                                                                                      \
    }
#define FC_HALO_PREP_W()                                                                                  \
    {                                                                                                     \
        const uint32_t sw = (uint32_t)((wkh * 3 + wkw) * g.c_in + wcc * TK) * ES;                         \
        const bool in_k = wleft > 0;                                                                      \
        --wleft;                                                                                          \
        if (k_tail) {                                                                                     \
            ld_sw = 0;                                                                                    \
            _Pragma("unroll") for (int j = 0; j < WR; ++j)                                                \
            {                                                                                             \
                const bool ok = in_k && wcc * TK + wgp[j] * EPP < g.c_in;                                 \
                ld_off[j] = ok ? woff[j] + sw : kOutOfRange;                                              \
            }                                                                                             \
        } else {                                                                                          \
            ld_sw = in_k ? sw : 0u;                                                                       \
            _Pragma("unroll") for (int j = 0; j < WR; ++j) ld_off[j] = in_k ? woff[j] : kOutOfRange;      \
        }                                                                                                 \
        const int w3 = (wkw == 2);                                                                        \
        wkw = w3 ? 0 : wkw + 1;                                                                           \
        const int wc = w3 & (wcc + 1 == cchunks);                                                         \
        wcc = w3 ? (wc ? 0 : wcc + 1) : wcc;                                                              \
        wkh += wc;                                                                                        \
    }
            // wave loads j in [first, last) of a stage's issue list: the weight slab (to ring
            // position wb) first, then, where the stage has one, the pixel line (to line buffer xb)
            const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)wave * 1024u);
#define FC_HALO_ISSUE(first, last, total, xb, wb)                                                         \
    _Pragma("unroll") for (int j = (first); j < (last); ++j)                                              \
        if (j < (total))                                                                                  \
            dma_load16_s(j < WR ? rsrc_w : rsrc_xb, ld_off[j], j < WR ? ld_sw : ld_sx,                    \
                         lds_wave + (j < WR ? 2u * XB + (uint32_t)(wb) * WB + (uint32_t)j * (RPP * 128)   \
                                            : (uint32_t)(xb) * XB + (uint32_t)(j - WR) * (RPP * 128)));

            // prologue, in this order: first pixel line (to buffer 0), then NBW - 1 weight slabs
            FC_HALO_PREP_X(WR)
            FC_HALO_ISSUE(WR, WR + XL, WR + XL, 0, 0)
#pragma unroll
            for (int d = 0; d < NBW - 1; ++d) {
                FC_HALO_PREP_W()
                FC_HALO_ISSUE(0, WR, WR, 0, d)
            }
            // one group: line buffer CXB is multiplied three times; the slab of tap t sits at ring
            // position (CW0 + t) % NBW
            auto group = [&](auto cxb_c, auto cw0_c) __attribute__((always_inline)) {
                constexpr int CXB = decltype(cxb_c)::value, CW0 = decltype(cw0_c)::value;
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    const int cwb = (CW0 + t) % NBW;            // (compile-time after unrolling)
                    const int iwb = (cwb + NBW - 1) % NBW;      // ring position the slab issued now goes to
                    // this stage issues the weight slab NBW - 1 stages ahead and, on the first
                    // tap, after it, the next group's pixel line
                    FC_HALO_PREP_W()
                    if (t == 0) FC_HALO_PREP_X(WR)
                    constexpr int kBehindW = (NBW - 2) * WR; // loads issued after this stage's slab ...
                    // ... on tap 0 (the line of this group was issued before that slab); on taps
                    // 1 and 2 the next group's line is in flight behind it as well
                    if (t == 0) wait_vmcnt<kBehindW>();
                    if (t == 1) wait_vmcnt<kBehindW + XL>();
                    if (t == 2) wait_vmcnt<(NBW == 3 ? WR + XL : 0)>();
                    __syncthreads();
                    const unsigned char *xs = stage0 + (uint32_t)CXB * XB;
                    const unsigned char *ws =
                        stage0 + 2u * XB + (uint32_t)cwb * WB + (wave_n * WTN) * 128 + frag_row;
                    const int nld = t == 0 ? WR + XL : WR;
                    const int lpk = t == 0 ? (WR + XL + KK - 1) / KK : (WR + KK - 1) / KK;
                    Frag<DT> wf[FB][CB], xf[FB][PB];
#pragma unroll
                    for (int b = 0; b < CB; ++b) wf[0][b].load(ws + b * 4096, frag_t16);
#pragma unroll
                    for (int a = 0; a < PB; ++a) xf[0][a].load(xs, xfa[a][t]);
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) {
                        if (FB == 2 && kk + 1 < KK) {
                            const uint32_t o = ((uint32_t)(kk + 1) * KSTEP) ^ frag_t16;
#pragma unroll
                            for (int b = 0; b < CB; ++b) wf[(kk + 1) & 1][b].load(ws + b * 4096, o);
#pragma unroll
                            for (int a = 0; a < PB; ++a)
                                xf[(kk + 1) & 1][a].load(xs, xfa[a][t] ^ ((uint32_t)(kk + 1) * KSTEP));
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        FC_HALO_ISSUE(kk * lpk, (kk + 1) * lpk, nld, CXB ^ 1, iwb)
#pragma unroll
                        for (int a = 0; a < PB; ++a)
#pragma unroll
                            for (int b = 0; b < CB; ++b)
                                acc[a][b] = mfma32<DT>(wf[kk % FB][b], xf[kk % FB][a], acc[a][b]);
                        if (FB == 1 && kk + 1 < KK) {
                            __builtin_amdgcn_sched_barrier(0);
                            const uint32_t o = ((uint32_t)(kk + 1) * KSTEP) ^ frag_t16;
#pragma unroll
                            for (int b = 0; b < CB; ++b) wf[0][b].load(ws + b * 4096, o);
#pragma unroll
                            for (int a = 0; a < PB; ++a) xf[0][a].load(xs, xfa[a][t] ^ ((uint32_t)(kk + 1) * KSTEP));
                        }
                    }
                }
            };
            // groups alternate between the two line buffers; with a ring of two slabs the ring
            // position of a group's first slab alternates as well (three stages per group), with
            // a ring of three it is always position 0
            static_assert(NBW == 2 || NBW == 3, "weight ring of the shared-halo loop");
            for (int gi = 0; gi < ng; gi += 2) {
                group(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
                if (gi + 1 < ng) group(std::integral_constant<int, 1>{}, std::integral_constant<int, (NBW == 2 ? 1 : 0)>{});
            }
#undef FC_HALO_ISSUE
#undef FC_HALO_PREP_W
#undef FC_HALO_PREP_X
        } else {
        __syncthreads(); // row_bits complete
        uint32_t xoff[XR], xbits[XR];
        int xgp[XR];
#pragma unroll
        for (int j = 0; j < XR; ++j) {
            const int r = prow + j * RPP;
            xgp[j] = slot ^ FC_SWZ(r);
            xoff[j] = ((uint32_t)row_base[r] * (uint32_t)g.c_in + (uint32_t)xgp[j] * EPP) * ES;
            xbits[j] = row_bits[r];
        }
        // cursor: the next stage to be issued (starts at this unit's first stage)
        int tap = s_begin / cchunks, cc = s_begin - tap * cchunks;
        int kh = tap / kwid, kw = tap - kh * kwid;
        int to_issue = nst; // stages of this unit not yet issued
        int ibuf = 0;       // LDS buffer the next stage goes to

        // Offsets and LDS targets of the cursor's stage (L wave loads), then advance the cursor.
        uint32_t ld_off[L], ld_lds[L];
#define FC_PREPARE_STAGE()                                                                                \
    {                                                                                                     \
        const uint32_t sx = (uint32_t)(((kh * g.dh) * g.w + kw * g.dw) * g.c_in + cc * TK) * ES;          \
        const uint32_t sw = (uint32_t)(tap * g.c_in + cc * TK) * ES;                                      \
        const uint32_t ldsx = lds0 + (uint32_t)ibuf * STAGE_BYTES + (uint32_t)wave * 1024u;               \
        const bool in_k = to_issue > 0;                                                                   \
        --to_issue;                                                                                       \
        _Pragma("unroll") for (int j = 0; j < XR; ++j)                                                    \
        {                                                                                                 \
            const bool ok = in_k && cc * TK + xgp[j] * EPP < g.c_in && ((xbits[j] >> (tap & 31)) & 1u);   \
            ld_off[j] = ok ? xoff[j] + sx : kOutOfRange;                                                  \
            ld_lds[j] = ldsx + (uint32_t)j * (RPP * 128);                                                 \
        }                                                                                                 \
        _Pragma("unroll") for (int j = 0; j < WR; ++j)                                                    \
        {                                                                                                 \
            const bool ok = in_k && cc * TK + wgp[j] * EPP < g.c_in;                                      \
            ld_off[XR + j] = ok ? woff[j] + sw : kOutOfRange;                                             \
            ld_lds[XR + j] = ldsx + (uint32_t)(TM * 128 + j * (RPP * 128));                               \
        }                                                                                                 \
        const int wrap_c = (cc + 1 == cchunks);                                                           \
        cc = wrap_c ? 0 : cc + 1;                                                                         \
        tap += wrap_c;                                                                                    \
        const int wrap_w = wrap_c & (kw + 1 == kwid);                                                     \
        kw = wrap_c ? (wrap_w ? 0 : kw + 1) : kw;                                                         \
        kh += wrap_w;                                                                                     \
        ibuf = (ibuf + 1 == NB) ? 0 : ibuf + 1;                                                           \
    }
#define FC_ISSUE_LOADS(first, last)                                                                       \
    _Pragma("unroll") for (int j = (first); j < (last); ++j)                                              \
        if (j < L) dma_load16(j < XR ? rsrc_x : rsrc_w, ld_off[j], __builtin_amdgcn_readfirstlane(ld_lds[j]));

        // prologue: NB-1 stages in flight (stages past the end are all out of range: free)
#pragma unroll
        for (int d = 0; d < NB - 1; ++d) {
            FC_PREPARE_STAGE()
            FC_ISSUE_LOADS(0, L)
        }

        constexpr int LPK = (L + KK - 1) / KK; // wave loads issued per 16-wide k-step
        int cbuf = 0;                          // buffer of the stage being multiplied
        for (int s = 0; s < nst; ++s) {
            FC_PREPARE_STAGE()          // stage s + NB - 1: addresses only
            wait_vmcnt<(NB - 2) * L>(); // this thread's loads of stage s have landed
            __syncthreads();            // ... and everyone else's; buffer (s-1) % NB is free
            const unsigned char *xs = stage0 + cbuf * STAGE_BYTES + (wave_m * WTM) * 128 + frag_row;
            const unsigned char *ws = stage0 + cbuf * STAGE_BYTES + (TM + wave_n * WTN) * 128 + frag_row;
            Frag<DT> wf[FB][CB], xf[FB][PB];
#pragma unroll
            for (int b = 0; b < CB; ++b) wf[0][b].load(ws + b * 4096, frag_t16);
#pragma unroll
            for (int a = 0; a < PB; ++a) xf[0][a].load(xs + a * 4096, frag_t16);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                if (FB == 2 && kk + 1 < KK) {
                    const uint32_t o = ((uint32_t)(kk + 1) * KSTEP) ^ frag_t16;
#pragma unroll
                    for (int b = 0; b < CB; ++b) wf[(kk + 1) & 1][b].load(ws + b * 4096, o);
#pragma unroll
                    for (int a = 0; a < PB; ++a) xf[(kk + 1) & 1][a].load(xs + a * 4096, o);
                }
                // keep the order "fetch step kk+1, then multiply step kk": the LDS latency
                // then hides under the MFMAs
                __builtin_amdgcn_sched_barrier(0);
                // the gathers of stage s + NB - 1 are spread over the k-steps, so that the
                // wave never queues behind a burst of loads with its matrix pipe idle
                FC_ISSUE_LOADS(kk * LPK, (kk + 1) * LPK)
#pragma unroll
                for (int a = 0; a < PB; ++a)
#pragma unroll
                    for (int b = 0; b < CB; ++b) acc[a][b] = mfma32<DT>(wf[kk % FB][b], xf[kk % FB][a], acc[a][b]);
                if (FB == 1 && kk + 1 < KK) {
                    __builtin_amdgcn_sched_barrier(0);
                    const uint32_t o = ((uint32_t)(kk + 1) * KSTEP) ^ frag_t16;
#pragma unroll
                    for (int b = 0; b < CB; ++b) wf[0][b].load(ws + b * 4096, o);
#pragma unroll
                    for (int a = 0; a < PB; ++a) xf[0][a].load(xs + a * 4096, o);
                }
            }
            cbuf = (cbuf + 1 == NB) ? 0 : cbuf + 1;
        }
#undef FC_ISSUE_LOADS
#undef FC_PREPARE_STAGE
        } // tap-by-tap loop

        // ---- epilogue: one rounding, ReLU; the tile is transposed through LDS so that every
        // lane stores 16 contiguous bytes.  First let every LDS write in flight land. ----
        wait_vmcnt<0>();
        __syncthreads();
        if (S > 1) {
            // Park this unit's fp32 partial tile (accumulator order, coalesced), then count
            // in; the unit that arrives last adds the S partials in split order - a fixed
            // order, so the result does not depend on which unit that is - and finishes the
            // tile.  Nobody waits for anybody.  The partials and the counter are written and
            // read with device-scope accesses, which go through to the memory side of the
            // per-XCD L2s, so no cache-wide write-back or invalidate is needed.
            // (16 bytes per access with the device-scope cache policy, the form a relaxed
            // agent-scope atomic store / load of 8 bytes compiles to, at twice the width)
            const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(
                partials, 0, (uint32_t)((size_t)kSplitGrid * kSplitTileFloats * sizeof(float)), 0x00020000);
            const uint32_t mine = (uint32_t)unit * (uint32_t)(TM * TN * 4);
#pragma unroll
            for (int a = 0; a < PB; ++a)
#pragma unroll
                for (int b = 0; b < CB; ++b)
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        u32x4_t v;
                        v.x = __float_as_uint(acc[a][b][4 * h]);
                        v.y = __float_as_uint(acc[a][b][4 * h + 1]);
                        v.z = __float_as_uint(acc[a][b][4 * h + 2]);
                        v.w = __float_as_uint(acc[a][b][4 * h + 3]);
                        __builtin_amdgcn_raw_buffer_store_b128(
                            v, rp, mine + (uint32_t)(((a * CB + b) * 4 + h) * NT + tid) * 16u, 0, kDeviceScope);
                    }
            wait_vmcnt<0>(); // this thread's partial stores have been acknowledged
            __syncthreads(); // ... and every other thread's
            if (tid == 0)
                row_bits[0] = (uint32_t)__hip_atomic_fetch_add(&tile_counters[tile], 1, __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            const bool last = (int)row_bits[0] == S - 1;
            if (!last) continue; // uniform: the whole workgroup moves on
            if (tid == 0)        // leave the counters as they were found
                __hip_atomic_store(&tile_counters[tile], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int a = 0; a < PB; ++a)
#pragma unroll
                for (int b = 0; b < CB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
            for (int sp = 0; sp < S; ++sp) {
                const uint32_t theirs = (uint32_t)(tile * S + sp) * (uint32_t)(TM * TN * 4);
#pragma unroll
                for (int a = 0; a < PB; ++a)
#pragma unroll
                    for (int b = 0; b < CB; ++b)
#pragma unroll
                        for (int h = 0; h < 4; ++h) {
                            const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(
                                rp, theirs + (uint32_t)(((a * CB + b) * 4 + h) * NT + tid) * 16u, 0, kDeviceScope);
                            acc[a][b][4 * h] += __uint_as_float(v.x);
                            acc[a][b][4 * h + 1] += __uint_as_float(v.y);
                            acc[a][b][4 * h + 2] += __uint_as_float(v.z);
                            acc[a][b][4 * h + 3] += __uint_as_float(v.w);
                        }
            }
        }
        constexpr int OP = TN * (int)sizeof(TO) + 16;
        static_assert((size_t)TM * OP <= REGION, "output tile fits");
        unsigned char *Os = smem_raw;
#pragma unroll
        for (int a = 0; a < PB; ++a) {
            const int r = wave_m * WTM + a * 32 + (lane & 31);
#pragma unroll
            for (int b = 0; b < CB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int cl = wave_n * WTN + b * 32 + q * 8 + (lane >> 5) * 4;
                    float v0 = acc[a][b][q * 4 + 0], v1 = acc[a][b][q * 4 + 1];
                    float v2 = acc[a][b][q * 4 + 2], v3 = acc[a][b][q * 4 + 3];
                    if constexpr (sizeof(TO) == 4) {
                        if (g.flags & FC_RELU) {
                            v0 = relu_keep_nan(v0); v1 = relu_keep_nan(v1);
                            v2 = relu_keep_nan(v2); v3 = relu_keep_nan(v3);
                        }
                        store4<ODT, TO>(reinterpret_cast<TO *>(Os + r * OP) + cl, v0, v1, v2, v3);
                    } else if constexpr (sizeof(TO) == 1) {
                        // 8-bit outputs: four codes per word, the same sign-bit rule
                        uint32_t pk;
                        store4<ODT, TO>(reinterpret_cast<TO *>(&pk), v0, v1, v2, v3);
                        if (g.flags & FC_RELU) pk = relu_packed8(pk);
                        *reinterpret_cast<uint32_t *>(Os + r * OP + cl) = pk;
                    } else {
                        // 16-bit outputs: round first, then clear the values whose sign bit is set, two
                        // at a time (rounding keeps the sign, so this is max(., 0) of the rounded value)
                        uint2 pk;
                        store4<ODT, TO>(reinterpret_cast<TO *>(&pk), v0, v1, v2, v3);
                        if (g.flags & FC_RELU) {
                            pk.x = relu_packed16(pk.x);
                            pk.y = relu_packed16(pk.y);
                        }
                        *reinterpret_cast<uint2 *>(Os + r * OP + cl * 2) = pk;
                    }
                }
        }
        __syncthreads();
        constexpr int PPR = TN * (int)sizeof(TO) / 16;
        constexpr int EPT = 16 / (int)sizeof(TO);
        // a thread keeps its 16-byte column and walks down the rows; all LDS reads of the walk
        // are issued before the first store
        constexpr int RPI = NT / PPR;   // rows per pass of the workgroup
        constexpr int NPASS = TM / RPI;
        static_assert(NT % PPR == 0 && TM % RPI == 0, "store walk");
        {
            const int pc = tid % PPR, r0 = tid / PPR;
            const int co = co0 + pc * EPT;
            int pp[NPASS];
            u32x4_t pv[NPASS];
#pragma unroll
            for (int k = 0; k < NPASS; ++k) {
                const int r = r0 + k * RPI;
                pp[k] = row_p[r];
                pv[k] = *reinterpret_cast<const u32x4_t *>(Os + r * OP + pc * 16);
            }
            // streaming stores: the output is not read again by this kernel
#pragma unroll
            for (int k = 0; k < NPASS; ++k)
                if (pp[k] >= 0 && co < g.c_out) {
                    // compacted output: row = place in the list, else the position itself
                    int64_t orow = (int64_t)pp[k];
                    if constexpr (CMP) {
                        if (g.flags & FC_COMPACT_OUT) orow = (int64_t)mt * TM + r0 + k * RPI;
                    }
                    __builtin_nontemporal_store(pv[k], reinterpret_cast<u32x4_t *>(out + orow * g.c_out + co));
                }
        }
    }

}

// ---------------------------------------------------------------------------

#if !defined(FC_MFMA_PART) || FC_MFMA_PART == 0
bool conv_mfma_supported(const Geom &g, int in_dtype, int out_dtype)
{
    if (in_dtype != FC_BF16 && in_dtype != FC_F16 && in_dtype != FC_FP8) return false;
    // fp8 layers round to bfloat16 (or stay fp32), the 16-bit types keep their own format; all can
    // round to fp8
    if (out_dtype != (in_dtype == FC_FP8 ? FC_BF16 : in_dtype) && out_dtype != FC_F32 && out_dtype != FC_FP8)
        return false;
    const uint64_t es = in_dtype == FC_FP8 ? 1u : 2u;
    if ((g.c_in * es) % 16 != 0 || g.c_out % 8 != 0) return false; // 16-byte gathers, 4-channel stores
    if (out_dtype == FC_FP8 && g.c_out % 16 != 0) return false;     // rows are stored in 16-byte pieces
    if (g.kh * g.kw > kMaxTaps) return false;
    // row origins are packed into signed 16-bit halves
    if (g.h > 16384 || g.w > 16384 || g.ph > 8192 || g.pw > 8192) return false;
    // x and w are each addressed through one buffer descriptor with 32-bit byte offsets
    // (the shared pixel line reads x through a descriptor that starts pad_h rows + pad_w pixels early)
    if (((uint64_t)g.n * g.h * g.w + (uint64_t)g.ph * g.w + g.pw) * g.c_in * es >= kBufferLimit) return false;
    if ((uint64_t)g.c_out * g.kh * g.kw * g.c_in * es >= kBufferLimit) return false;
    return true;
}
#endif

template <int DT, typename TO, bool CMP, int TM, int TN, int WM, int WN, int TAPC, int NB, int MINW, int SL = 0, int NBW = 2>
static hipError_t launch_dma(const Geom &g, const void *x, const uint8_t *mask_in, const uint8_t *mask_out,
                             const void *w, const float *bias, const int32_t *idx, const int32_t *count,
                             void *out, float *partials, int32_t *tile_counters, hipStream_t s)
{
    auto kern = k_conv_dma<DT, TO, TM, TN, WM, WN, TAPC, NB, MINW, SL, NBW, CMP>;
    constexpr size_t lds = dma_lds_bytes<TM, TN, NB, SL, NBW>();
    // more than 64 KB of dynamic LDS has to be allowed once per function and device; two
    // threads that both find the bit clear both set the attribute, which is harmless
    static std::atomic<uint64_t> attr_devices{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t dev_bit = 1ull << (dev & 63);
    if (!(attr_devices.load(std::memory_order_acquire) & dev_bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds);
        if (e != hipSuccess) return e;
        attr_devices.fetch_or(dev_bit, std::memory_order_release);
    }
    const int64_t max_tiles = (int64_t)((g.m + TM - 1) / TM) * ((g.c_out + TN - 1) / TN);
    const int64_t cap = 256 * 8;
    int blocks = (int)((max_tiles < cap ? max_tiles : cap) + 7) & ~7; // a multiple of the XCD count
    if (partials) blocks = kSplitGrid; // few tiles: enough workgroups for the K-split to fill the chip
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(WM * WN * 64), lds, s, g, (const uint16_t *)x, mask_in, mask_out,
                       (const uint16_t *)w, bias, idx, count, (TO *)out, partials, tile_counters);
    return hipGetLastError();
}

#define FC_ARGS g, x, mask_in, mask_out, w, bias, idx, count, out, partials, tile_counters, s

template <int DT, typename TO, int TAPC, bool CMP>
static hipError_t launch_tile(const Geom &g, const void *x, const uint8_t *mask_in, const uint8_t *mask_out,
                              const void *w, const float *bias, const int32_t *idx, const int32_t *count,
                              void *out, float *partials, int32_t *tile_counters, hipStream_t s)
{
    // 128 x 128 tiles when there are enough of them to give every CU two workgroups;
    // otherwise 128 x 64, which doubles the tile count (the kept count is not known here,
    // so the dense row count decides)
    const int64_t tiles128 = (int64_t)((g.m + 127) / 128) * ((g.c_out + 127) / 128);
    // Layers with only a handful of tiles (the late layers of a network at batch 1) are all
    // latency: 64 x 64 tiles put them on more CUs and four stage buffers keep three gathers in
    // flight (a ResNet-18 stack at batch 1: 0.243 -> 0.221 ms dense, 0.266 -> 0.245 ms focused)
    if constexpr (TAPC != 32) {
        const int64_t tiles64w = (int64_t)((g.m + 127) / 128) * ((g.c_out + 63) / 64);
        if (tiles64w <= kSmallLayerTiles) return launch_dma<DT, TO, CMP, 64, 64, 2, 2, TAPC, 4, 2>(FC_ARGS);
    }
    // 3x3 kernels that step one pixel at a time horizontally share the gathered pixels
    // between their three horizontal taps (worth it when image rows are long enough for runs
    // of adjacent kept positions; narrow layers with many tiles do better with three
    // workgroups per CU, see below)
    if constexpr (TAPC == 9) {
        if (g.sw == 1 && g.dw == 1 && g.wo >= 16) {
            // (with many 128 x 128 tiles it pays down to 16-pixel rows: C512@16 at batch 128 is
            // 13 % faster dense and 17 % faster focused than tap by tap)
            if (g.c_out > 64 && tiles128 >= 512)
                return launch_dma<DT, TO, CMP, 128, 128, 2, 2, TAPC, 2, 2, 160, 2>(FC_ARGS);
            // narrow layers: only with very many tiles (C64@128: -7 % focused, -4..8 % dense from batch
            // 128 on, 16 384 row tiles; at 4 800 row tiles, 64 -> 64 on 32 x 120 x 160 positions, three
            // workgroups per CU, below, are 7 % faster, and at batch 16 as fast)
            const bool many_narrow_tiles = (int64_t)((g.m + 127) / 128) >= 8192;
            if (g.wo >= 32 && (g.c_out > 64 || partials || many_narrow_tiles))
                return launch_dma<DT, TO, CMP, 128, 64, 2, 2, TAPC, 3, 2, 160, 3>(FC_ARGS);
            // shorter image rows, wide layers, a few hundred tiles (C512 on 32 x 15 x 20 positions:
            // 66 us dense / 45 us chained against 102 / 49 us tap by tap; with 128 tiles, C512@16 at
            // batch 16, tap by tap stays ahead)
            if (g.c_out > 64 && tiles128 >= 256)
                return launch_dma<DT, TO, CMP, 128, 64, 2, 2, TAPC, 3, 2, 160, 3>(FC_ARGS);
        }
    }
    // (1x1 layers keep the wide tiles down to 256 of them: 2048 -> 512 on 32 x 15 x 20 positions,
    // 300 tiles, 37 us dense / 29 us chained against 51 / 32 us with 128 x 64 tiles)
    if (g.c_out > 64 && tiles128 >= (TAPC == 1 ? 256 : 512))
        return launch_dma<DT, TO, CMP, 128, 128, 2, 2, TAPC, (sizeof(TO) == 4 ? 3 : 2), 2>(FC_ARGS);
    // narrow layers with many tiles: two stage buffers, so that three workgroups fit a CU
    // and overlap each other's set-up and epilogue
    if (g.c_out <= 64 && !partials) return launch_dma<DT, TO, CMP, 128, 64, 2, 2, TAPC, 2, 3>(FC_ARGS);
    return launch_dma<DT, TO, CMP, 128, 64, 2, 2, TAPC, 3, 2>(FC_ARGS);
}
#undef FC_ARGS

#define FC_ARGS2 g, x, mask_in, mask_out, w, bias, idx, count, out, partials, tile_counters, s

template <int DT, typename TO, bool CMP>
static hipError_t launch_cmp(const Geom &g, const void *x, const uint8_t *mask_in, const uint8_t *mask_out,
                            const void *w, const float *bias, const int32_t *idx, const int32_t *count,
                            void *out, float *partials, int32_t *tile_counters, hipStream_t s)
{
    if (g.kh == 1 && g.kw == 1) return launch_tile<DT, TO, 1, CMP>(FC_ARGS2);
    if (g.kh == 3 && g.kw == 3) return launch_tile<DT, TO, 9, CMP>(FC_ARGS2);
    return launch_tile<DT, TO, 32, CMP>(FC_ARGS2);
}

// The instances of one storage type, with or without compacted activations.
template <int DT, bool CMP>
static hipError_t launch_part(const Geom &g, int out_dtype, const void *x, const uint8_t *mask_in,
                              const uint8_t *mask_out, const void *w, const float *bias, const int32_t *idx,
                              const int32_t *count, void *out, float *partials, int32_t *tile_counters,
                              hipStream_t s)
{
    if (out_dtype == FC_F32) return launch_cmp<DT, float, CMP>(FC_ARGS2);
    if (out_dtype == FC_FP8) return launch_cmp<DT, uint8_t, CMP>(FC_ARGS2);
    return launch_cmp<DT, uint16_t, CMP>(FC_ARGS2);
}

// The kernel instances are spread over six translation units so that a build can compile them
// side by side: a unit compiled with -DFC_MFMA_PART=p (p = 2 * storage type index + compacted)
// holds the instances of part p, part 0 also the two entry points below; without the macro
// this file is one unit that holds everything.
#define FC_PART_PARAMS                                                                                     \
    const Geom &g, int out_dtype, const void *x, const uint8_t *mask_in, const uint8_t *mask_out,         \
        const void *w, const float *bias, const int32_t *idx, const int32_t *count, void *out,             \
        float *partials, int32_t *tile_counters, hipStream_t s
#define FC_PART_ARGS g, out_dtype, x, mask_in, mask_out, w, bias, idx, count, out, partials, tile_counters, s
hipError_t launch_mfma_bf16(FC_PART_PARAMS);
hipError_t launch_mfma_bf16_compact(FC_PART_PARAMS);
hipError_t launch_mfma_f16(FC_PART_PARAMS);
hipError_t launch_mfma_f16_compact(FC_PART_PARAMS);
hipError_t launch_mfma_fp8(FC_PART_PARAMS);
hipError_t launch_mfma_fp8_compact(FC_PART_PARAMS);

#ifndef FC_MFMA_PART
#define FC_MFMA_PART -1
#endif
#define FC_IN_PART(p) (FC_MFMA_PART < 0 || FC_MFMA_PART == (p))

#if FC_IN_PART(0)
hipError_t launch_mfma_bf16(FC_PART_PARAMS) { return launch_part<FC_BF16, false>(FC_PART_ARGS); }
#endif
#if FC_IN_PART(1)
hipError_t launch_mfma_bf16_compact(FC_PART_PARAMS) { return launch_part<FC_BF16, true>(FC_PART_ARGS); }
#endif
#if FC_IN_PART(2)
hipError_t launch_mfma_f16(FC_PART_PARAMS) { return launch_part<FC_F16, false>(FC_PART_ARGS); }
#endif
#if FC_IN_PART(3)
hipError_t launch_mfma_f16_compact(FC_PART_PARAMS) { return launch_part<FC_F16, true>(FC_PART_ARGS); }
#endif
#if FC_IN_PART(4)
hipError_t launch_mfma_fp8(FC_PART_PARAMS) { return launch_part<FC_FP8, false>(FC_PART_ARGS); }
#endif
#if FC_IN_PART(5)
hipError_t launch_mfma_fp8_compact(FC_PART_PARAMS) { return launch_part<FC_FP8, true>(FC_PART_ARGS); }
#endif

#if FC_IN_PART(0)
hipError_t launch_conv_mfma(const Geom &g, int in_dtype, int out_dtype, const void *x, const uint8_t *mask_in,
                            const uint8_t *mask_out, const void *w, const float *bias, const int32_t *idx,
                            const int32_t *count, void *out, float *partials, int32_t *tile_counters,
                            hipStream_t s)
{
    const bool compact = (g.flags & (FC_COMPACT_IN | FC_COMPACT_OUT)) != 0;
    if (in_dtype == FC_BF16) return compact ? launch_mfma_bf16_compact(FC_PART_ARGS) : launch_mfma_bf16(FC_PART_ARGS);
    if (in_dtype == FC_FP8) return compact ? launch_mfma_fp8_compact(FC_PART_ARGS) : launch_mfma_fp8(FC_PART_ARGS);
    return compact ? launch_mfma_f16_compact(FC_PART_ARGS) : launch_mfma_f16(FC_PART_ARGS);
}
#endif

} // namespace fc
