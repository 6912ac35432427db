// Focused convolution on the gfx950 matrix cores, one resident workgroup per CU
// (Sec. III-A: a GEMM over the kept patches only, with the dense layer's weights).
//
// Same GEMM view and the same data path as the tiled kernel next door (rows = kept output
// positions, reduction = (tap, input channel), gathers straight from global memory into
// swizzled LDS rows, 32x32x16 matrix instructions with fp32 accumulators, bias-initialised
// accumulators, one rounding in the epilogue), built for 3x3 layers with so few kept rows that
// the chip holds about one tile per CU.  There the run time is one tile latency, and "a few
// tiles more than CUs" costs a whole second round.  Here the launch is as many workgroups as
// CUs, and the kept rows (known on the device only) are dealt out evenly in blocks of 32:
// every workgroup gets the same share, one round whatever the kept count, so that the time
// follows the kept share instead of moving in steps.
//
// A workgroup is eight waves, WM x WN over the rows and output channels of a tile.  The number
// of 32-row blocks a wave multiplies is a run-time value (up to PBW), which is what lets the
// shares be even; the stage loop is instantiated once per block count, so that the loads and
// multiplies of a stage stay straight-line code.
//
// Set-up is done once per "macro tile" of up to NSUB tiles: list entries -> positions ->
// pixel line -> tap-valid bits are two dependent memory round trips, paid once for several
// tiles; the tiles of a macro tile then only read tables in LDS.  The first weight slabs are
// requested before the set-up starts.
//
// Pixel line (unit horizontal stride and dilation): the kept positions of a tile are sorted,
// so along a run of horizontally adjacent kept positions the left pixel of one is the centre
// pixel of the one before.  A tile lays its pixels out on a line of slots: one per kept
// position plus one before the first and one after the last position of every run; position
// r's taps kw = 0, 1, 2 are slots cs(r) - 1, cs(r), cs(r) + 1.  For every (kernel row,
// 64-channel chunk) the line is gathered once and multiplied three times.  A macro tile whose
// lines would not fit (fragmented masks), and every other 3x3 geometry, runs tap by tap: one
// slot per position, one tap per gathered line.
#include "fc_dma_util.hpp"
#include <atomic>
#include <type_traits>

namespace fc {

constexpr int kLineWaves = 8;
constexpr int kLineThreads = kLineWaves * 64;
constexpr int kLineRPP = kLineThreads / 8; // LDS rows one pass of wave loads covers (16 bytes per lane)

constexpr int line_round_up(int v, int to) { return (v + to - 1) / to * to; }
// slots of one tile's pixel line: its rows, two run ends, one spare, in whole load passes
constexpr int line_slots(int tm) { return line_round_up(tm + 32, kLineRPP); }

// LDS bytes: two pixel-line buffers, the ring of weight slabs, then the tables of a macro tile.
template <int TM, int TN, int NSUB>
constexpr size_t line_table_bytes()
{
    // row_p, row_cs [NSUB * TM]; slot_pix, slot_hw, slot_bits [NSUB * SL]; sub_slot; scan parts
    return (size_t)(2 * NSUB * TM + 3 * NSUB * line_slots(TM) + (NSUB + 1) + 64) * sizeof(int32_t);
}
template <int TM, int TN, int NSUB, int NBW>
constexpr size_t line_lds_bytes()
{
    return (size_t)2 * line_slots(TM) * 128 + (size_t)NBW * TN * 128 + line_table_bytes<TM, TN, NSUB>();
}

// divisors of the position decode, prepared on the host
struct LineDivs {
    FastDiv wo, ho;
    int32_t n_nt, n_rs_max; // channel tiles; workgroups per channel tile (the most row shares)
    FastDiv rs;            // by n_rs_max
};

// DT: storage type (bf16 / f16); TO: float or the 16-bit / 8-bit carrier of the output; TN: output
// channels per tile; WM x WN: waves; PBW: most 32-row blocks per wave (tile height up to
// WM * PBW * 32); NSUB: tiles per macro tile; NBW: ring of weight slabs (NBW - 1 stages ahead).
//
// Stage order (both loops): kernel row, 64-channel chunk, horizontal tap.  On a shared line the
// three horizontal taps of one (kernel row, chunk) read one gathered line; tap by tap every
// stage gathers its own.  The weight stream is the same either way, so its first slabs are
// requested before the set-up knows which loop a macro tile takes.
template <int DT, typename TO, int TN, int WM, int WN, int PBW, int NSUB, int NBW, int MINW>
__global__ __launch_bounds__(kLineThreads, MINW) void k_conv_line(Geom g, LineDivs dv, const uint16_t *__restrict__ x,
                                                                  const uint8_t *__restrict__ mask_in,
                                                                  const uint8_t *__restrict__ mask_out,
                                                                  const uint16_t *__restrict__ w,
                                                                  const float *__restrict__ bias,
                                                                  const int32_t *__restrict__ idx,
                                                                  const int32_t *__restrict__ count,
                                                                  TO *__restrict__ out)
{
    static_assert(WM * WN == kLineWaves, "eight waves");
    static_assert(DT == FC_BF16 || DT == FC_F16, "16-bit storage");
    static_assert(NBW >= 3, "weight ring");
    constexpr int NT = kLineThreads;
    constexpr int RPP = kLineRPP;
    constexpr int TM = WM * PBW * 32;          // most rows of a tile
    constexpr int RMAX = NSUB * TM;            // most rows of a macro tile
    constexpr int SL = line_slots(TM);         // slots of a line buffer
    constexpr int SMAX = NSUB * SL;
    constexpr int XL = SL / RPP, WR = TN / RPP; // wave loads per thread: one line, one weight slab
    constexpr int CB = TN / (WN * 32);
    constexpr int ES = 2, TK = kStageBytes / ES, EPP = 16 / ES;
    constexpr uint32_t KSTEP = kStepBytes<DT>;
    constexpr int KK = kStageBytes / (int)KSTEP; // matrix instructions per stage and block pair
    constexpr int RIT = (RMAX + NT - 1) / NT;  // rows per thread in the set-up
    constexpr uint32_t XB = (uint32_t)SL * 128u, WB = (uint32_t)TN * 128u;
    constexpr int KW = 3, TAPC = 9;            // 3x3 kernels: horizontal taps = stages per (kernel row, chunk)
    static_assert(TN % RPP == 0 && TN % (WN * 32) == 0, "tile shape");
    // a 128-row piece of the output tile passes through the front of LDS when the loop is over
    constexpr size_t FRONT = (size_t)2 * XB + (size_t)NBW * WB;
    constexpr int OP = TN * (int)sizeof(TO) + 16;
    static_assert((size_t)128 * OP <= FRONT, "front of LDS");

    extern __shared__ __align__(16) unsigned char smem_raw[];
    const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>(smem_raw);
    const int cchunks = (g.c_in + TK - 1) / TK;
    const int nstage = TAPC * cchunks;
    const uint32_t wbuf_bytes = (uint32_t)NBW * WB;
    unsigned char *const wbuf = smem_raw + 2 * XB;
    int32_t *row_p = reinterpret_cast<int32_t *>(smem_raw + 2 * XB + wbuf_bytes);
    int32_t *row_cs = row_p + RMAX;
    int32_t *slot_pix = row_cs + RMAX;
    int32_t *slot_hw = slot_pix + SMAX;
    uint32_t *slot_bits = reinterpret_cast<uint32_t *>(slot_hw + SMAX);
    int32_t *sub_slot = reinterpret_cast<int32_t *>(slot_bits + SMAX); // first slot of every tile, [NSUB + 1]
    int32_t *scan_part = sub_slot + (NSUB + 1);                        // [RIT][8] wave totals

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // (wave-uniform: kept in a scalar register)
    // (waves w and w + 4 share a SIMD: with the channel index fastest they take different rows
    // of the tile, so a SIMD's two waves together hold an even number of row blocks)
    const int wave_n = wave % WN, wave_m = wave / WN;
    const int slot = tid & 7, prow = tid >> 3;

    const int rows = idx ? *count : g.m;
    const int n_nt = dv.n_nt;
    const int nb = (rows + 31) >> 5;          // 32-row blocks of the kept rows
    // Row shares: as many as there are workgroups per channel tile (but no share below WM
    // blocks, which would leave waves without rows); share i takes the blocks
    // [i * nb / n_rs, (i + 1) * nb / n_rs).  Units are ordered channel tile first, and XCD j
    // (workgroup b runs on XCD b mod 8) takes the j-th contiguous eighth, so that the units
    // which share an L2 share one weight slab and neighbouring image rows.
    // (divisions by the usual share count go through a divisor prepared on the host)
    int n_rs = dv.n_rs_max;
    const bool few_blocks = n_rs > (nb + WM - 1) / WM;
    if (few_blocks) n_rs = (nb + WM - 1) / WM;
    const int nunits = n_rs * n_nt;
    const int per_xcd = (nunits + 7) >> 3;
    const int xcd = blockIdx.x & 7;
    const int share_q = few_blocks ? (n_rs > 0 ? nb / n_rs : 0) : (int)fast_div((uint32_t)nb, dv.rs);
    const int share_r = nb - share_q * n_rs; // nb = q * n_rs + r
    const u32x4_t rsrc_x = make_rsrc_words(x, (uint32_t)g.n * g.h * g.w * g.c_in * (uint32_t)ES);
    const u32x4_t rsrc_w = make_rsrc_words(w, (uint32_t)g.c_out * TAPC * g.c_in * (uint32_t)ES);

    // fragment addressing (see the tiled kernel): lane reads row (lane & 31) of a 32-row
    // block; in k-step q that is the 16-byte piece 2q + (lane >> 5), stored at slot
    // piece ^ swizzle(row)
    const uint32_t frag_row = (uint32_t)(lane & 31) * 128u;
    const uint32_t frag_t16 = (uint32_t)((lane >> 5) ^ FC_SWZ(lane & 31)) * 16u;
    const int xgp = slot ^ FC_SWZ(prow); // 16-byte piece this lane fetches for its LDS slot (rows 64 apart share it)

    // ---- zero-fill of the irrelevant output rows: every wave takes 64 positions at a time.
    // The labels of a wave's first 64 positions are asked for now, so that this round trip runs
    // beside the set-up's; the rows are cleared after the tiles, when nothing waits on the
    // memory counter any more (loads and stores share it: a store issued earlier would make the
    // next wait for gathered data wait for its acknowledgement as well). ----
    const bool packed_masks = (g.flags & FC_PACKED_MASKS) != 0; // masks are one bit per pixel
    const bool zero_fill = mask_in && !(g.flags & FC_SKIP_ZERO_FILL);
    const int zf_workers = (int)gridDim.x * kLineWaves;
    const int zf_first = ((int)blockIdx.x * kLineWaves + wave) * 64;
    auto label_of = [&](int pp) -> bool {
        // kept?  (positions past the end count as kept: nothing to clear)
        if (pp >= g.m) return true;
        if (mask_out) return mask_at(mask_out, pp, packed_masks);
        const int ch0 = -g.ph + g.dh * ((g.kh - 1) / 2), cw0 = -g.pw + g.dw * ((g.kw - 1) / 2);
        const int q = (int)fast_div((uint32_t)pp, dv.wo);
        const int ow = pp - q * g.wo;
        const int b = (int)fast_div((uint32_t)q, dv.ho);
        const int oh = q - b * g.ho;
        const int ih = min(max(oh * g.sh + ch0, 0), g.h - 1);
        const int iw = min(max(ow * g.sw + cw0, 0), g.w - 1);
        return mask_at(mask_in, (int64_t)(b * g.h + ih) * g.w + iw, packed_masks);
    };
    auto clear_rows = [&](int pp, uint64_t drop, int32_t *dropped) {
        const int cpr = g.c_out * (int)sizeof(TO) / 16; // 16-byte pieces per row
        u32x4_t *o4 = reinterpret_cast<u32x4_t *>(out);
        const u32x4_t zero4 = {0u, 0u, 0u, 0u};
        const bool kept = !((drop >> lane) & 1ull);
        const int nd = __popcll(drop);
        if (!kept) dropped[__popcll(drop & ((1ull << lane) - 1ull))] = pp; // in position order
        // (same wave wrote and reads the list: program order suffices)
        const int total = nd * cpr;
        for (int c = lane; c < total; c += 64) {
            const int rk = c / cpr, pc = c - rk * cpr;
            __builtin_nontemporal_store(zero4, o4 + (int64_t)dropped[rk] * cpr + pc);
        }
    };
    bool zf_kept = true;
    const bool zf_pending = zero_fill && zf_first < g.m;
    if (zf_pending) zf_kept = label_of(zf_first + lane);
    uint64_t zf_drop = 0; // (taken from the labels once the first tile's list entries are on their way)
    bool zf_have = false;


    for (int slot_t = blockIdx.x >> 3; slot_t < per_xcd; slot_t += gridDim.x >> 3) {
        const int unit = xcd * per_xcd + slot_t;
        if (unit >= nunits) break;
        const int nt = few_blocks ? unit / n_rs : (int)fast_div((uint32_t)unit, dv.rs), rs = unit - nt * n_rs;
        const int co0 = nt * TN;
        // blocks [rs * nb / n_rs, (rs + 1) * nb / n_rs) without a 64-bit division
        const int ub0 = rs * share_q + (few_blocks ? (rs * share_r) / n_rs : (int)fast_div((uint32_t)(rs * share_r), dv.rs));
        const int ub1 = (rs + 1) * share_q +
                        (few_blocks ? ((rs + 1) * share_r) / n_rs : (int)fast_div((uint32_t)((rs + 1) * share_r), dv.rs));

        // per-thread weight rows (loop-invariant): LDS row r of a slab holds output channel co0 + r
        uint32_t woff[WR];
#pragma unroll
        for (int j = 0; j < WR; ++j) {
            const int co = co0 + prow + j * RPP;
            woff[j] = co < g.c_out ? ((uint32_t)co * (uint32_t)(TAPC * g.c_in) + (uint32_t)xgp * EPP) * ES : kOutOfRange;
        }
        __syncthreads(); // the previous unit is done with LDS

        float4 bias_q[CB][4];
#pragma unroll
        for (int b = 0; b < CB; ++b)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int co = co0 + wave_n * (CB * 32) + b * 32 + q * 8 + (lane >> 5) * 4;
                bias_q[b][q] = (bias && co < g.c_out) ? *reinterpret_cast<const float4 *>(bias + co)
                                                      : make_float4(0.f, 0.f, 0.f, 0.f);
            }

        // weight-slab cursor of the tile being prepared (kernel row, chunk, horizontal tap)
        int wkh = 0, wcc = 0, wkw = 0, wleft = 0, wbuf_i = 0;
        uint32_t ldw_off[WR];
        auto prep_w = [&]() {
            const uint32_t sw = (uint32_t)((wkh * KW + wkw) * g.c_in + wcc * TK) * ES;
            const bool in_k = wleft > 0 && wcc * TK + xgp * EPP < g.c_in;
            --wleft;
#pragma unroll
            for (int j = 0; j < WR; ++j) ldw_off[j] = in_k ? woff[j] + sw : kOutOfRange;
        };
        auto issue_w = [&](int j) {
            dma_load16(rsrc_w, ldw_off[j],
                       __builtin_amdgcn_readfirstlane(lds0 + 2u * XB + (uint32_t)wbuf_i * WB + (uint32_t)wave * 1024u +
                                                      (uint32_t)j * (RPP * 128)));
        };
        auto advance_w = [&]() {
            const int last_t = (wkw + 1 == KW);
            wkw = last_t ? 0 : wkw + 1;
            const int wc = last_t & (wcc + 1 == cchunks);
            wcc = last_t ? (wc ? 0 : wcc + 1) : wcc;
            wkh += wc;
            wbuf_i = (wbuf_i + 1 == NBW) ? 0 : wbuf_i + 1;
        };
        // the first NBW - 1 slabs of a tile: asked for as early as LDS is free
        auto weight_prologue = [&]() {
            wkh = 0; wcc = 0; wkw = 0; wleft = nstage; wbuf_i = 0;
#pragma unroll
            for (int d = 0; d < NBW - 1; ++d) {
                prep_w();
#pragma unroll
                for (int j = 0; j < WR; ++j) issue_w(j);
                advance_w();
            }
        };

        // ---- macro tiles of this unit: rows [mm0, mm1) of the kept list ----
        for (int mb0 = ub0; mb0 < ub1; mb0 += NSUB * WM * PBW) {
            const int mb1 = min(ub1, mb0 + NSUB * WM * PBW);
            const int nblk_all = mb1 - mb0;
            const int mm0 = mb0 * 32, mm1 = min(rows, mb1 * 32);
            const int rpad = nblk_all * 32;                                   // rows incl. the padding of the last block
            const int nsub = (nblk_all + WM * PBW - 1) / (WM * PBW);           // tiles, even in blocks
            // first block of tile s: s * nblk_all / nsub
            int tile_b[NSUB + 1];
#pragma unroll
            for (int s = 0; s <= NSUB; ++s) {
                // s * nblk_all / nsub with the divisor a compile-time constant in every branch
                int v = nblk_all;
                if (s < nsub) {
                    const int num = s * nblk_all;
                    v = nsub == 1 ? num : nsub == 2 ? num / 2 : nsub == 3 ? num / 3 : nsub == 4 ? num / 4 : num / nsub;
                }
                tile_b[s] = v;
            }

            if (mb0 != ub0) __syncthreads(); // the previous macro tile is done with LDS and the tables
            weight_prologue();

            // A: the rows' positions and those of their list neighbours in one round trip (thread t
            // takes rows t, t + NT, ...); cnt = slots a row adds to its tile's pixel line: itself,
            // one before it unless its left neighbour is the row before it (in the same tile), one
            // after it unless its right neighbour is the row after it.
            int sa_p[RIT], sa_prev[RIT], sa_next[RIT];
#pragma unroll
            for (int i = 0; i < RIT; ++i) {
                const int r = tid + i * NT;
                const int m = mm0 + r;
                const bool live = r < rpad && m < mm1;
                sa_p[i] = live ? (idx ? idx[m] : m) : -1;
                sa_prev[i] = (live && r > 0) ? (idx ? idx[m - 1] : m - 1) : -2;
                sa_next[i] = (live && m + 1 < mm1) ? (idx ? idx[m + 1] : m + 1) : -2;
            }
            if (zf_pending && !zf_have) {
                zf_drop = __ballot(!zf_kept);
                zf_have = true;
            }
            int sa_ow[RIT], sa_ih0[RIT], sa_iw0[RIT], sa_b[RIT], cnt[RIT], lead[RIT];
            bool ladj[RIT], radj[RIT];
#pragma unroll
            for (int i = 0; i < RIT; ++i) {
                const int r = tid + i * NT;
                const int p = sa_p[i];
                int ow = 0, ih0 = 0, iw0 = 0, b = 0;
                cnt[i] = r < rpad ? 1 : 0; lead[i] = 0; ladj[i] = false; radj[i] = false;
                if (p >= 0) {
                    const int q = (int)fast_div((uint32_t)p, dv.wo);
                    ow = p - q * g.wo;
                    b = (int)fast_div((uint32_t)q, dv.ho);
                    const int oh = q - b * g.ho;
                    ih0 = oh * g.sh - g.ph;
                    iw0 = ow * g.sw - g.pw;
                    // first and last row of this row's tile
                    int st = 0;
#pragma unroll
                    for (int s = 1; s < NSUB; ++s) st += (s < nsub && (r >> 5) >= tile_b[s]) ? 1 : 0;
                    int first = 0, last = 0;
#pragma unroll
                    for (int s = 0; s < NSUB; ++s)
                        if (s == st) { first = tile_b[s] * 32; last = tile_b[s + 1] * 32 - 1; }
                    ladj[i] = r > first && sa_prev[i] == p - 1 && ow > 0;
                    radj[i] = r < last && sa_next[i] == p + 1 && ow < g.wo - 1;
                    lead[i] = ladj[i] ? 0 : 1;
                    cnt[i] = 1 + lead[i] + (radj[i] ? 0 : 1);
                }
                sa_ow[i] = ow; sa_ih0[i] = ih0; sa_iw0[i] = iw0; sa_b[i] = b;
                if (r < RMAX) row_p[r] = p;
                const int incl = wave_inclusive_scan(cnt[i]);
                if (lane == 63) scan_part[i * kLineWaves + wave] = incl;
                cnt[i] = incl - cnt[i]; // exclusive, inside the wave
            }
            __syncthreads();
            // B: slot tables in the shared-line form (kept if every tile's line fits)
            const bool shared_geom = g.sw == 1 && g.dw == 1;
            {
                int carry = 0;
#pragma unroll
                for (int i = 0; i < RIT; ++i) {
                    int mine = carry;
#pragma unroll
                    for (int v = 0; v < kLineWaves; ++v) {
                        const int t = scan_part[i * kLineWaves + v];
                        mine += v < wave ? t : 0;
                        carry += t;
                    }
                    cnt[i] += mine; // slots before this row's first
                }
                if (tid == 0) sub_slot[nsub] = carry;
#pragma unroll
                for (int i = 0; i < RIT; ++i) {
                    const int r = tid + i * NT;
                    if (r < rpad) {
                        // first slot of every tile = the first slot of its first row
#pragma unroll
                        for (int s = 0; s < NSUB; ++s)
                            if (s < nsub && r == tile_b[s] * 32) sub_slot[s] = cnt[i];
                        const int cs = cnt[i] + lead[i];
                        if (shared_geom && cs + 1 < SMAX) {
                            row_cs[r] = cs;
                            if (sa_p[i] >= 0) {
                                const int iwc = sa_iw0[i] + 1; // kw = 1, unit dilation
                                const int pixc = (sa_b[i] * g.h + sa_ih0[i]) * g.w + iwc;
                                const int ih16 = (int)((uint32_t)sa_ih0[i] & 0xffffu);
                                slot_pix[cs] = pixc;
                                slot_hw[cs] = ih16 | (int)((uint32_t)iwc << 16);
                                if (!ladj[i]) {
                                    slot_pix[cs - 1] = pixc - 1;
                                    slot_hw[cs - 1] = ih16 | (int)((uint32_t)(iwc - 1) << 16);
                                }
                                if (!radj[i]) {
                                    slot_pix[cs + 1] = pixc + 1;
                                    slot_hw[cs + 1] = ih16 | (int)((uint32_t)(iwc + 1) << 16);
                                }
                            } else {
                                slot_pix[cs] = 0;
                                slot_hw[cs] = (int)((uint32_t)(-20000) << 16); // never inside an image
                            }
                        }
                    }
                }
            }
            __syncthreads();
            bool use_shared = shared_geom;
            int tile_s[NSUB + 1]; // first slot of every tile
#pragma unroll
            for (int s = 0; s <= NSUB; ++s) tile_s[s] = sub_slot[s <= nsub ? s : nsub];
#pragma unroll
            for (int s = 0; s < NSUB; ++s)
                if (s < nsub && tile_s[s + 1] - tile_s[s] + 1 > SL) use_shared = false;
            if (!use_shared) {
                // tap by tap: one slot per row, holding the pixel of the row's first tap
#pragma unroll
                for (int i = 0; i < RIT; ++i) {
                    const int r = tid + i * NT;
                    if (r < rpad) {
                        row_cs[r] = r;
                        if (sa_p[i] >= 0) {
                            slot_pix[r] = (sa_b[i] * g.h + sa_ih0[i]) * g.w + sa_iw0[i];
                            slot_hw[r] = (int)(((uint32_t)sa_ih0[i] & 0xffffu) | ((uint32_t)sa_iw0[i] << 16));
                        } else {
                            slot_pix[r] = 0;
                            slot_hw[r] = (int)((uint32_t)(-20000) << 16);
                        }
                    }
                }
#pragma unroll
                for (int s = 0; s <= NSUB; ++s) tile_s[s] = tile_b[s] * 32;
                __syncthreads();
            }

            // C: one thread per (slot, q): inside the image and relevant?  q = kernel row on a
            // shared line (the slot's own column), tap otherwise
            auto tap_bits = [&](auto nq_c, const int nsl) {
                constexpr int NQ = decltype(nq_c)::value;
                for (int sl = tid; sl < nsl; sl += NT) {
                    const int hw = slot_hw[sl];
                    const int pix = slot_pix[sl];
                    const int ih0 = (int)(int16_t)(hw & 0xffff), iw0 = hw >> 16;
                    bool inb[NQ];
                    uint8_t mv[NQ];
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        const int kh_i = NQ == 3 ? q : q / KW, kw_i = NQ == 3 ? 0 : q - (q / KW) * KW;
                        const int ih = ih0 + kh_i * g.dh, iw = iw0 + kw_i * g.dw;
                        inb[q] = ih >= 0 && ih < g.h && iw >= 0 && iw < g.w;
                        mv[q] = mask_in
                                    ? (uint8_t)mask_at(mask_in, inb[q] ? pix + kh_i * g.dh * g.w + kw_i * g.dw : 0, packed_masks)
                                    : (uint8_t)1;
                    }
                    uint32_t bits = 0;
#pragma unroll
                    for (int q = 0; q < NQ; ++q) bits |= (inb[q] && mv[q]) ? (1u << q) : 0u;
                    slot_bits[sl] = bits;
                }
            };
            if (use_shared) tap_bits(std::integral_constant<int, 3>{}, tile_s[NSUB]);
            else tap_bits(std::integral_constant<int, TAPC>{}, rpad);
            __syncthreads();

            // ---- the tiles of this macro tile ----
#pragma unroll 1
            for (int st = 0; st < nsub; ++st) {
                int r0 = 0, r1 = 0, s0 = 0, s1 = 0;
#pragma unroll
                for (int s = 0; s < NSUB; ++s)
                    if (s == st) { r0 = tile_b[s] * 32; r1 = tile_b[s + 1] * 32; s0 = tile_s[s]; s1 = tile_s[s + 1]; }
                const int nsl = s1 - s0; // (a shared line has one spare slot after these: zeros)
                const int nblk = (r1 - r0) >> 5;
                const int nblk_w = (nblk + WM - 1) / WM;                 // blocks per wave row
                const int nb_mine = __builtin_amdgcn_readfirstlane(min(max(nblk - wave_m * nblk_w, 0), nblk_w));
                if (st > 0) weight_prologue(); // (the first tile's went out before the set-up)

                // this thread's line loads: slot prow + j * RPP of the tile's line
                uint32_t hxoff[XL], hxbits[XL];
#pragma unroll
                for (int j = 0; j < XL; ++j) {
                    const int l = prow + j * RPP;
                    const bool live = l < nsl;
                    const int sl = live ? s0 + l : 0;
                    hxoff[j] = ((uint32_t)slot_pix[sl] * (uint32_t)g.c_in + (uint32_t)xgp * EPP) * ES;
                    hxbits[j] = live ? slot_bits[sl] : 0u;
                }
                // centre slot of this lane's row in each of its blocks (local to the tile's line)
                int cs_l[PBW];
#pragma unroll
                for (int a = 0; a < PBW; ++a) {
                    const int rl = a < nb_mine ? (wave_m * nblk_w + a) * 32 + (lane & 31) : 0;
                    cs_l[a] = row_cs[r0 + rl] - s0;
                }

                f32x16_t acc[PBW][CB];
#pragma unroll
                for (int a = 0; a < PBW; ++a)
#pragma unroll
                    for (int b = 0; b < CB; ++b)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            acc[a][b][q * 4 + 0] = bias_q[b][q].x;
                            acc[a][b][q * 4 + 1] = bias_q[b][q].y;
                            acc[a][b][q * 4 + 2] = bias_q[b][q].z;
                            acc[a][b][q * 4 + 3] = bias_q[b][q].w;
                        }

                // ---- stage loop, instantiated for the number of blocks this wave multiplies (so
                // that the loads and multiplies of a stage are straight-line code) and for the two
                // line forms: TG = horizontal taps per gathered line ----
                auto run_stages = [&](auto tg_c, auto nbm_c) {
                    constexpr int TG = decltype(tg_c)::value;
                    constexpr int NBM = decltype(nbm_c)::value;
                    int xkh = 0, xcc = 0, xkw = 0, xleft = (TG == 3 ? 3 * cchunks : nstage), xbuf_i = 0; // next line
                    uint32_t ldx_off[XL];
                    auto prep_x = [&]() {
                        const uint32_t sx = (uint32_t)(((xkh * g.dh) * g.w + xkw * g.dw) * g.c_in + xcc * TK) * ES;
                        const int q = TG == 3 ? xkh : xkh * KW + xkw;
                        const bool in_k = xleft > 0 && xcc * TK + xgp * EPP < g.c_in;
                        --xleft;
#pragma unroll
                        for (int j = 0; j < XL; ++j)
                            ldx_off[j] = (in_k && ((hxbits[j] >> (q & 31)) & 1u)) ? hxoff[j] + sx : kOutOfRange;
                    };
                    auto issue_x = [&](int j) {
                        dma_load16(rsrc_x, ldx_off[j],
                                   __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)xbuf_i * XB + (uint32_t)wave * 1024u +
                                                                  (uint32_t)j * (RPP * 128)));
                    };
                    auto advance_x = [&]() {
                        if (TG == 3) {
                            const int wrap = (xcc + 1 == cchunks);
                            xcc = wrap ? 0 : xcc + 1;
                            xkh += wrap;
                        } else {
                            const int last_t = (xkw + 1 == KW);
                            xkw = last_t ? 0 : xkw + 1;
                            const int wc = last_t & (xcc + 1 == cchunks);
                            xcc = last_t ? (wc ? 0 : xcc + 1) : xcc;
                            xkh += wc;
                        }
                        xbuf_i ^= 1;
                    };
                    // first line
                    prep_x();
#pragma unroll
                    for (int j = 0; j < XL; ++j) issue_x(j);
                    advance_x();
                    int cxb = 0, cwb = 0; // line buffer and slab being multiplied
                    const int ngroups = 3 * cchunks; // (kernel row, chunk) pairs
                    for (int gi = 0; gi < ngroups; ++gi) {
#pragma unroll
                        for (int t = 0; t < KW; ++t) {
                            const bool new_line = TG == 1 || t == 0; // this stage multiplies a line of its own
                            // The loads of this stage (the slab NBW - 1 stages ahead and, with a new
                            // line, the next line) are spread over its k-steps.  Issue order: three-tap
                            // lines slab then line, one-tap lines line then slab.  Before that, wait
                            // for this stage's own slab and line: the counts are what may stay in flight.
                            prep_w();
                            if (new_line) prep_x();
                            if (gi == 0 && t == 0) {
                                wait_vmcnt<0>(); // (the first slabs went out before the set-up's own loads)
                            } else {
                                if (TG == 1) wait_vmcnt<WR>();
                                else if (t == 0) wait_vmcnt<(NBW - 2 < 2 ? NBW - 2 : 2) * WR>(); // (behind this group's line: at most two slabs)
                                else wait_vmcnt<(NBW - 2) * WR + XL>();
                            }
                            __syncthreads();
                            const unsigned char *xs = smem_raw + (uint32_t)cxb * XB;
                            const unsigned char *ws = wbuf + (uint32_t)cwb * WB + (wave_n * (CB * 32)) * 128 + frag_row;
                            // LDS addresses of this lane's fragments in the line
                            uint32_t xfa[NBM > 0 ? NBM : 1];
#pragma unroll
                            for (int a = 0; a < NBM; ++a) {
                                const int sl = cs_l[a] + (TG == 3 ? t - 1 : 0);
                                xfa[a] = (uint32_t)sl * 128u + (uint32_t)((lane >> 5) ^ FC_SWZ(sl)) * 16u;
                            }
                            constexpr int NLW = WR;
                            const int nlx = new_line ? XL : 0;
                            const int nld = NLW + nlx;
                            const int lpk = (nld + KK - 1) / KK;
                            Frag<DT> wf[2][CB], xf[2][NBM > 0 ? NBM : 1];
                            if (NBM > 0) {
#pragma unroll
                                for (int b = 0; b < CB; ++b) wf[0][b].load(ws + b * 4096, frag_t16);
#pragma unroll
                                for (int a = 0; a < NBM; ++a) xf[0][a].load(xs, xfa[a]);
                            }
#pragma unroll
                            for (int kk = 0; kk < KK; ++kk) {
                                if (NBM > 0 && kk + 1 < KK) {
                                    const uint32_t o = ((uint32_t)(kk + 1) * KSTEP) ^ frag_t16;
#pragma unroll
                                    for (int b = 0; b < CB; ++b) wf[(kk + 1) & 1][b].load(ws + b * 4096, o);
#pragma unroll
                                    for (int a = 0; a < NBM; ++a)
                                        xf[(kk + 1) & 1][a].load(xs, xfa[a] ^ ((uint32_t)(kk + 1) * KSTEP));
                                }
                                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                                for (int j2 = 0; j2 < WR + XL; ++j2) {
                                    if (j2 >= kk * lpk && j2 < (kk + 1) * lpk && j2 < nld) {
                                        // position j2 of this stage's issue order
                                        const bool is_w = TG == 3 ? j2 < NLW : j2 >= nlx;
                                        if (is_w) issue_w(TG == 3 ? j2 : j2 - nlx);
                                        else issue_x(TG == 3 ? j2 - NLW : j2);
                                    }
                                }
#pragma unroll
                                for (int a = 0; a < NBM; ++a)
#pragma unroll
                                    for (int b = 0; b < CB; ++b) acc[a][b] = mfma32<DT>(wf[kk & 1][b], xf[kk & 1][a], acc[a][b]);
                            }
                            advance_w();
                            if (new_line) advance_x();
                            cwb = (cwb + 1 == NBW) ? 0 : cwb + 1;
                            if (TG == 1) cxb ^= 1;
                        }
                        if (TG == 3) cxb ^= 1;
                    }
                };
                auto run_blocks = [&](auto tg_c) {
                    switch (nb_mine) {
                    case 0: run_stages(tg_c, std::integral_constant<int, 0>{}); break;
                    case 1: run_stages(tg_c, std::integral_constant<int, 1>{}); break;
                    case 2: if constexpr (PBW >= 2) run_stages(tg_c, std::integral_constant<int, 2>{}); break;
                    case 3: if constexpr (PBW >= 3) run_stages(tg_c, std::integral_constant<int, 3>{}); break;
                    case 4: if constexpr (PBW >= 4) run_stages(tg_c, std::integral_constant<int, 4>{}); break;
                    case 5: if constexpr (PBW >= 5) run_stages(tg_c, std::integral_constant<int, 5>{}); break;
                    case 6: if constexpr (PBW >= 6) run_stages(tg_c, std::integral_constant<int, 6>{}); break;
                    case 7: if constexpr (PBW >= 7) run_stages(tg_c, std::integral_constant<int, 7>{}); break;
                    default: if constexpr (PBW >= 8) run_stages(tg_c, std::integral_constant<int, 8>{}); break;
                    }
                };
                static_assert(PBW <= 8, "block counts the stage loop is instantiated for");
                if (use_shared) run_blocks(std::integral_constant<int, 3>{});
                else run_blocks(std::integral_constant<int, 1>{});

                // ---- epilogue ----
                wait_vmcnt<0>();
                __syncthreads();
                // the tile leaves through LDS in pieces of 128 rows: one rounding, ReLU, then every
                // thread stores 16 contiguous bytes of a kept row
                unsigned char *Os = smem_raw;
                constexpr int PPR = TN * (int)sizeof(TO) / 16;
                constexpr int EPT = 16 / (int)sizeof(TO);
                constexpr int RPI = NT / PPR;
                constexpr int NPASS = 128 / RPI;
                static_assert(NT % PPR == 0 && 128 % RPI == 0, "store walk");
                for (int c0 = 0; c0 < nblk * 32; c0 += 128) {
                    {
#pragma unroll
                        for (int a = 0; a < PBW; ++a) {
                            const int blk = wave_m * nblk_w + a;
                            if (a < nb_mine && (blk >> 2) == (c0 >> 7)) {
                                const int r = (blk & 3) * 32 + (lane & 31);
#pragma unroll
                                for (int b = 0; b < CB; ++b)
#pragma unroll
                                    for (int q = 0; q < 4; ++q) {
                                        const int cl = wave_n * (CB * 32) + b * 32 + q * 8 + (lane >> 5) * 4;
                                        float v0 = acc[a][b][q * 4 + 0], v1 = acc[a][b][q * 4 + 1];
                                        float v2 = acc[a][b][q * 4 + 2], v3 = acc[a][b][q * 4 + 3];
                                        if constexpr (sizeof(TO) == 4) {
                                            if (g.flags & FC_RELU) {
                                                v0 = relu_keep_nan(v0); v1 = relu_keep_nan(v1);
                                                v2 = relu_keep_nan(v2); v3 = relu_keep_nan(v3);
                                            }
                                            store4<DT, TO>(reinterpret_cast<TO *>(Os + r * OP) + cl, v0, v1, v2, v3);
                                        } else if constexpr (sizeof(TO) == 1) {
                                            uint32_t pk;
                                            store4<DT, TO>(reinterpret_cast<TO *>(&pk), v0, v1, v2, v3);
                                            if (g.flags & FC_RELU) pk = relu_packed8(pk);
                                            *reinterpret_cast<uint32_t *>(Os + r * OP + cl) = pk;
                                        } else {
                                            uint2 pk;
                                            store4<DT, TO>(reinterpret_cast<TO *>(&pk), v0, v1, v2, v3);
                                            if (g.flags & FC_RELU) {
                                                pk.x = relu_packed16(pk.x);
                                                pk.y = relu_packed16(pk.y);
                                            }
                                            *reinterpret_cast<uint2 *>(Os + r * OP + cl * 2) = pk;
                                        }
                                    }
                            }
                        }
                    }
                    __syncthreads();
                    {
                        const int pc = tid % PPR, rr0 = tid / PPR;
                        const int co = co0 + pc * EPT;
                        int pp[NPASS];
                        u32x4_t pv[NPASS];
#pragma unroll
                        for (int k = 0; k < NPASS; ++k) {
                            const int r = rr0 + k * RPI;
                            const bool live = c0 + r < nblk * 32;
                            pp[k] = live ? row_p[r0 + c0 + r] : -1;
                            pv[k] = *reinterpret_cast<const u32x4_t *>(Os + r * OP + pc * 16);
                        }
#pragma unroll
                        for (int k = 0; k < NPASS; ++k)
                            if (pp[k] >= 0 && co < g.c_out)
                                __builtin_nontemporal_store(
                                    pv[k], reinterpret_cast<u32x4_t *>(out + (int64_t)pp[k] * g.c_out + co));
                    }
                    __syncthreads();
                }
            } // tiles
        }     // macro tiles
    }         // units
    if (zero_fill) {
        __syncthreads(); // the last tile is done with the front of LDS
        int32_t *dropped = reinterpret_cast<int32_t *>(smem_raw) + wave * 64;
        if (zf_pending) clear_rows(zf_first + lane, zf_have ? zf_drop : __ballot(!zf_kept), dropped);
        for (int p0 = zf_first + zf_workers * 64; p0 < g.m; p0 += zf_workers * 64)
            clear_rows(p0 + lane, __ballot(!label_of(p0 + lane)), dropped);
    }
}

// ---------------------------------------------------------------------------

bool conv_line_supported(const Geom &g, int in_dtype, int out_dtype)
{
    if (in_dtype != FC_BF16 && in_dtype != FC_F16) return false;
    if (out_dtype != in_dtype && out_dtype != FC_F32 && out_dtype != FC_FP8) return false;
    if (!(g.kh == 3 && g.kw == 3)) return false;
    if (g.c_in % 8 != 0 || g.c_out % 8 != 0) return false;       // 16-byte gathers, 4-channel stores
    if (out_dtype == FC_FP8 && g.c_out % 16 != 0) return false;   // rows are stored in 16-byte pieces
    if (g.flags & (FC_COMPACT_IN | FC_COMPACT_OUT)) return false;
    // row origins are packed into signed 16-bit halves
    if (g.h > 16384 || g.w > 16384 || g.ph > 8192 || g.pw > 8192) return false;
    if ((uint64_t)g.n * g.h * g.w * g.c_in * 2u >= kBufferLimit) return false;
    if ((uint64_t)g.c_out * g.kh * g.kw * g.c_in * 2u >= kBufferLimit) return false;
    return true;
}

static int line_grid()
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

template <int DT, typename TO, int TN, int WM, int WN, int PBW, int NSUB, int NBW, int MINW>
static hipError_t launch_line(const Geom &g, const void *x, const uint8_t *mask_in, const uint8_t *mask_out,
                              const void *w, const float *bias, const int32_t *idx, const int32_t *count, void *out,
                              hipStream_t s)
{
    auto kern = k_conv_line<DT, TO, TN, WM, WN, PBW, NSUB, NBW, MINW>;
    constexpr int TM = WM * PBW * 32;
    constexpr size_t lds = line_lds_bytes<TM, TN, NSUB, NBW>();
    static_assert(lds <= 160 * 1024, "LDS of a CU");
    LineDivs dv;
    dv.wo = make_fastdiv((uint32_t)g.wo);
    dv.ho = make_fastdiv((uint32_t)g.ho);
    dv.n_nt = (g.c_out + TN - 1) / TN;
    dv.n_rs_max = line_grid() / dv.n_nt < 1 ? 1 : line_grid() / dv.n_nt;
    dv.rs = make_fastdiv((uint32_t)dv.n_rs_max);
    // the dynamic LDS limit is raised once per function and device to the most any layer can ask for
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
    hipLaunchKernelGGL(kern, dim3(line_grid()), dim3(kLineThreads), lds, s, g, dv, (const uint16_t *)x, mask_in, mask_out,
                       (const uint16_t *)w, bias, idx, count, (TO *)out);
    return hipGetLastError();
}

#define FC_LINE_ARGS g, x, mask_in, mask_out, w, bias, idx, count, out, s

// 128 output channels per tile, 2 x 4 waves, tiles of up to 8 blocks, three weight slabs in the ring
template <int DT, typename TO>
static hipError_t launch_line_shape(const Geom &g, const void *x, const uint8_t *mask_in, const uint8_t *mask_out,
                                    const void *w, const float *bias, const int32_t *idx, const int32_t *count,
                                    void *out, hipStream_t s)
{
    return launch_line<DT, TO, 128, 2, 4, 4, 1, 3, 2>(FC_LINE_ARGS);
}

hipError_t launch_conv_line(const Geom &g, int in_dtype, int out_dtype, const void *x,
                            const uint8_t *mask_in, const uint8_t *mask_out, const void *w, const float *bias,
                            const int32_t *idx, const int32_t *count, void *out, hipStream_t s)
{
#define FC_LINE_CALL(DT, TO) launch_line_shape<DT, TO>(g, x, mask_in, mask_out, w, bias, idx, count, out, s)
    if (in_dtype == FC_BF16) {
        if (out_dtype == FC_F32) return FC_LINE_CALL(FC_BF16, float);
        if (out_dtype == FC_FP8) return FC_LINE_CALL(FC_BF16, uint8_t);
        return FC_LINE_CALL(FC_BF16, uint16_t);
    }
    if (out_dtype == FC_F32) return FC_LINE_CALL(FC_F16, float);
    if (out_dtype == FC_FP8) return FC_LINE_CALL(FC_F16, uint8_t);
    return FC_LINE_CALL(FC_F16, uint16_t);
#undef FC_LINE_CALL
}

} // namespace fc
