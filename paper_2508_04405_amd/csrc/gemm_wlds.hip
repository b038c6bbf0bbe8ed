// Tiled i8-MFMA GEMM with BOTH operands through LDS: 256x256 tiles, 256x128 or 128x256.
//
// The 128x256 kernel is limited by power, and what costs power besides the
// MFMAs is every byte a wavefront brings in through the vector-memory path:
// timing probes put the packed-weight loads at about a fifth of its run time
// and the activation DMA at a tenth, while doubling the LDS operand reads
// costs 3 %.  This kernel therefore trades vector-memory bytes for LDS reads:
// one workgroup of eight wavefronts (2 along m x 4 along n, 128 x 32 NT each)
// owns a 256 x (128 NT) tile, and a packed weight tile is brought into LDS ONCE
// per workgroup (by DMA, like the activations) and read from there by the two
// wavefronts that share its columns: 0.875 KB through the vector-memory path
// per 32x32x128 block at NT = 2 instead of 1.25.
//
//   LDS: three weight stages (24 KiB for whole tiles), requested TWO stages ahead (a
//   packed weight panel is read by few workgroups, all at the same time, so its lines
//   come from HBM, well over a microsecond away), and activation stages of 32 KiB: for
//   whole tiles two of them, requested one stage ahead (an activation panel is shared by
//   every column tile of its row and mostly found in L2 or the Infinity Cache; a third
//   stage would not fit beside the weights), for half tiles, whose stages are shorter
//   than the memory latency, three, requested two ahead.  One workgroup per CU, two
//   wavefronts per SIMD.  The hand-over waits until at most the loads for the stage after
//   next are outstanding.
//
//   Where in a stage the requests are made matters as much as how far ahead (each
//   measured against the alternative on one box, alternating): whatever all eight
//   wavefronts do at the same moment -- right after the hand-over's barrier, at the
//   start of a stage -- is a burst that the matrix pipe waits out.  So the work beside
//   the MFMAs is dealt out over the eight steps of a stage (a step: the four MFMAs of one
//   k-step and column block):
//     step 0  activation requests (DMA); LDS reads: activation operands of k-step 1,
//             plane 1 of the stage's packed tiles
//     step 1  plane 2            step 2  activation operands of k-step 2
//     step 3  weight requests (DMA)       step 4  activation operands of k-step 3
//     step 6  hand-over: counted wait, barrier; plane 0 of the next stage's tiles
//     step 7  the next stage's first activation operands
//   Against everything at the stage's start and after the barrier: planes 1 and 2 later
//   +1.4 % (and the shorter register lifetimes end the spilling), weight requests later
//   +1.6 %, first activation operands a step after the barrier +0.9 %, one item per step
//   +1.4 %.  The activation requests stay at the start (a step later: -1.2 %; right after
//   the barrier, which would free their buffer a k-step earlier: -1.5 % to -3 %), and the
//   hand-over before the last k-step (a step earlier: -4.5 %, the requests have less time).
//   Letting the two wavefronts that share a pair of packed tiles expand one tile's fourth
//   k-step each and exchange the operands through LDS (a third fewer vector operations):
//   -1.4 %, the exchange costs more than the expansion.  Not
//   kept either: two weight buffers with a second barrier per stage to make room for a
//   third activation buffer (-3 %); raising one wavefront's priority over its SIMD-mate's,
//   for a k-step in turn or for part of a stage (-1 % to -40 %: a wavefront alone does not
//   keep the pipe busy, the two must interleave).
//
// Per-channel scales only: this is the kernel for large M and N.
//
// A launch is PERSISTENT: at most one workgroup per CU, each taking its items
// (tiles) one after the other, and the operands of the next item's first stages
// are already on their way into LDS while the finished tile is scaled and
// stored, so neither the first loads' latency nor the store burst stands
// between two tiles' MFMAs.  The wavefronts accumulate D^T (channels down the
// registers, one token per lane): a lane's four consecutive registers are four
// consecutive channels of one token, so the epilogue scales and converts in
// registers and sends 8-byte pieces of finished fp16 through a small LDS
// transpose, from which whole 128-byte lines are stored (Section 4.3.2's
// coalesced write-back, Section 4.3.4's fused dequantization).
//
// Launch forms.  Whole tiles.  Half tiles, 256x128: the tiles left over after
// the last whole round of 256, as twice as many items of half the work, so a
// round of up to 128 leftover tiles costs little more than half a round.
// And the cut tail (SK): the leftover tiles cut along K into contiguous runs of
// 128-k stages, one run per workgroup, whose int32 sums (exact, so the order of
// addition does not matter) meet in the workspace.  EVENLY (SK = 2): every tile
// into the same number of pieces, which end together and share the tile's
// reduction -- each piece stores the sums of the slabs it does not own, waits a
// bounded number of polls for the tile's stage count to be complete and
// finishes the slabs it owns; a piece whose wait runs out leaves its slabs to
// the piece that completed the count.  Or into 256 equal runs that begin and
// end inside tiles (SK = 1): the workgroups of a tile add their stage counts
// to the tile's counter, and the one that completes the count adds the others'
// sums to its own registers and runs the epilogue; nobody waits for anybody.
// And low tiles, 128x256, on their own: up to 128 tokens on a layer wide enough
// for them to fill the chip in one round, where the time is the one pass over
// the weights (about 37 GB/s per CU come through the DMA path, here as in the
// whole tiles); on narrower layers, from 65 tokens, each cut evenly along K.
#include "flexq_device.h"
#include "flexq_kernels.h"
#include "gemm_common.h"
#include <type_traits>

namespace {

constexpr int WAVES = 8;
constexpr int SLOT_BYTES = 256 * 256 * 4;      // one workgroup's int32 sums of a 256x256 tile

// The eight wavefronts share a whole tile 2 along m x 4 along n, 128 x 64 each (MT = 4 row
// blocks of 32, NT = 2 column blocks of 32: an expanded weight operand feeds four MFMAs,
// an activation operand two), and a half tile 4 along m x 2 along n, 64 x 64 each.  LDS
// delivers 128 bytes a clock to the CU and a 32x32x32 MFMA occupies a SIMD for 32, so a
// stage reads (MT + 0.75 NT) / (MT NT) KiB per MFMA of at most 1 KiB: 0.69 for the whole
// tile, 0.875 for 64 x 64.  (The whole tile's 128-row layout on half the columns, 128 x 32
// per wavefront, would ask for 1.19; measured, it runs the half tiles at the same speed --
// their stages are not bound by LDS reads -- and the lighter shape was kept.  For whole
// tiles, 1 x 8 wavefronts of 256 x 32 halve the expansion work per MFMA for twice the
// activation reads: measured 2-5 % slower on every layer.)
// TILE names the shape: 2 the whole tile (256 x 256), 1 the half tile (256 x 128), 3 the
// low tile (128 x 256, 2 x 4 wavefronts of 64 x 64: for up to 128 tokens on wide layers)
template <int TILE>
struct Shape {
    static_assert(TILE >= 1 && TILE <= 3, "half, whole or low tiles");
    static constexpr int WN = TILE == 1 ? 2 : 4;
    static constexpr int MT = TILE == 2 ? 4 : 2;
    static constexpr int NT = 2;
    static constexpr int BN = WN * NT * 32;
    static constexpr int BM = WAVES / WN * MT * 32;
    static_assert(BN == 256 || BN == 128, "whole or half width");
    static_assert(BM == 256 || BM == 128, "whole or half height");
    static constexpr int XSTAGE = BM * 128;               // bytes of one activation stage
    static constexpr int XDMA = BM / 8 / WAVES;           // 1 KiB activation DMA loads per wavefront and stage
    static constexpr int WTILES = BN / 32;                        // packed tiles per stage
    static constexpr int WSTAGE = WTILES * FLEXQ_TILE_BYTES;
    static constexpr int XA = TILE == 2 ? 1 : 2;                  // activation stages requested ahead
    static constexpr int XBUFS = XA + 1;
    static constexpr int WBASE = XBUFS * XSTAGE;
    // This wavefront's weight DMA loads per stage: plane p of a stage is fetched by
    // wavefront p % 4.  Wavefronts 0 .. 3 fetch all the weights: the two wavefronts of a SIMD
    // do not advance alike -- the older one (0 .. 3) wins the arbitration, runs ahead and
    // waits at the stage's barrier for the younger one, whose instruction stream sets the
    // pace -- and these loads are work that can move to the wavefronts that have the time
    // (measured A/B: about 1 % at 2048 and 4096 tokens, 3 % on the half tiles; moving the
    // activations' loads as well loses 1.3 %: eight more loads in a row per wavefront).
    static constexpr int WISSUERS = 4;
    static_assert(3 * WTILES % WISSUERS == 0, "equal shares");
    static constexpr int WDMA_LOW = 3 * WTILES / WISSUERS;               // wavefronts below WDMA_SPLIT
    static constexpr int WDMA_HIGH = 0;                                  // the others
    static constexpr int WDMA_SPLIT = WISSUERS;
    // Epilogue staging, 32 rows of fp16 per wavefront: it begins where the THIRD weight
    // stage does.  While a tile is stored, the next item's first stages are landing in
    // the activation stages below XA and in weight stages 0 and 1; weight stage 2 and what
    // lies beyond it are free until the next item's stage 0 asks for the weights of its
    // stage 2, after the barrier that ends the epilogue.
    static constexpr int STG = WBASE + 2 * WSTAGE;
    static constexpr int ESTRIDE = NT * 64 + 16;
    static constexpr int STG_END = STG + WAVES * 32 * ESTRIDE;
    static constexpr int LDS_BYTES = STG_END > WBASE + 3 * WSTAGE ? STG_END : WBASE + 3 * WSTAGE;
    static_assert(LDS_BYTES + 1024 <= 160 * 1024, "LDS of one CU (plus the static part)");
};

// One item of a workgroup's list: stages [ks, ke) of the 256-wide tile `t256`
// (its half `half` when the items are half tiles); `tj` numbers the tile within a cut tail.
struct Item {
    int t256, half, ks, ke, tj;
};

// One phase of a launch: this workgroup's share of `item_count` items that begin at the
// 256-wide tile `item_begin` -- whole tiles (TILE = 2), half tiles (two items per tile),
// or, with SK, the stages of `item_count` tiles cut into `tail_wgs` runs.
template <int TILE, int SK>
__device__ __forceinline__ void run_items(const flexq::LinearArgs &a, uint8_t *lds, int &s_last, int tiles_m,
                                          int tiles_n, int item_begin, int item_count, int tail_wgs)
{
#if defined(__HIP_DEVICE_COMPILE__)  // buffer-resource builtins exist in the device pass only
    using S = Shape<TILE>;
    constexpr int MT = S::MT, NT = S::NT;
    constexpr bool WHOLE = S::BN == 256;
    static_assert(!SK || WHOLE, "the tail is cut in whole-width tiles");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / S::WN, wn = wave % S::WN;
    const int M = a.M, N = a.N, K = a.K;
    const int KT = K / FLEXQ_TILE_K;

    // Workgroups 8 apart share an XCD.  Every XCD takes a contiguous share of the items
    // (or of the tail's runs), so the workgroups of one XCD work on neighbouring tiles
    // and find each other's operand panels in their L2.
    const int G = (int)gridDim.x;
    const int xcd = (int)(blockIdx.x % 8), slot = (int)(blockIdx.x / 8);
    int j_next = 0, j_end = 0;                      // !SK: this workgroup's items j_next, j_next + G/8, ...
    long u0 = 0, u1 = 0;                            // SK: this workgroup's run of stages
    int vt = -1;
    const long U = (long)item_count * KT;           // SK: 128-k stages of the tail
    if (!SK) {
        j_next = (int)((long)xcd * item_count / 8) + slot;
        j_end = (int)((long)(xcd + 1) * item_count / 8);
    } else {
        const int per = tail_wgs / 8, rem = tail_wgs % 8;
        if (slot < per + (xcd < rem ? 1 : 0)) vt = xcd * per + min(xcd, rem) + slot;
        if (vt >= 0) {
            u0 = (long)vt * U / tail_wgs;
            u1 = (long)(vt + 1) * U / tail_wgs;
        }
    }
    const long run_begin = u0;
    // the next item of this workgroup, if any (all values wavefront-uniform)
    auto take = [&](Item &it) -> bool {
        if (!SK) {
            if (j_next >= j_end) return false;
            const int j = j_next;
            j_next += G / 8;
            it.t256 = item_begin + (WHOLE ? j : j >> 1);
            it.half = WHOLE ? 0 : (j & 1);
            it.ks = 0;
            it.ke = KT;
            it.tj = 0;
            return true;
        } else {
            if (u0 >= u1) return false;
            it.tj = (int)(u0 / KT);
            it.ks = (int)(u0 - (long)it.tj * KT);
            it.ke = (int)min((long)KT, it.ks + (u1 - u0));
            it.t256 = item_begin + it.tj;
            it.half = 0;
            u0 += it.ke - it.ks;
            return true;
        }
    };

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)a.xq, 0, (unsigned)((long)M * K), 0x00020000);
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)a.packed, 0, (unsigned)((long)N * K / 4 * 3), 0x00020000);

    // ---- where an item's operands are, and the DMA loads of one stage -----------
    // The 32 tiles an XCD works on at a time share operand panels in its L2: a block of
    // 4 tiles along m x 8 along n fetches the fewest bytes (4 activation panels of 2 MB
    // per 8192 of K + 8 weight panels of 1.5 MB).
    struct Where {
        int bm0, bn0;
        unsigned xoff[S::XDMA];
    };
    auto locate = [&](const Item &it, Where &w) {
        int lane_l = lane;        // (opaque: recomputed per item rather than kept live, see the epilogue)
        asm volatile("" : "+v"(lane_l));
        constexpr int SUP_M = 4;  // super-block: 4 tiles along m, then next n
        const int bid = it.t256;
        const int sup = bid / (SUP_M * tiles_n);
        const int first_m = sup * SUP_M;
        const int span_m = min(SUP_M, tiles_m - first_m);
        const int in_sup = bid - sup * SUP_M * tiles_n;
        w.bm0 = (first_m + in_sup % span_m) * S::BM;
        w.bn0 = (in_sup / span_m) * 256 + it.half * S::BN;
#pragma unroll
        for (int i = 0; i < S::XDMA; ++i) {
            const int q = wave * S::XDMA + i;
            const int row = 8 * q + (lane_l >> 3);
            const int c = (lane_l & 7) ^ ((row >> 1) & 7);
            w.xoff[i] = (unsigned)(w.bm0 + row) * (unsigned)K + 16u * c;
        }
    };
    // activations: global -> LDS by DMA; rows beyond M read as zero (stage numbers count from ks)
    auto dma_x = [&](const Where &w, int ks, int kb, int buf) {
#pragma unroll
        for (int i = 0; i < S::XDMA; ++i) {
            uint8_t *dst = lds + buf * S::XSTAGE + (wave * S::XDMA + i) * 1024;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                xrsrc, (void __attribute__((address_space(3))) *)dst, 16, w.xoff[i],
                (ks + kb) * FLEXQ_TILE_K, 0, 0);
        }
    };
    // packed weights: the stage's WTILES tiles of three 1 KiB planes go into LDS exactly as
    // they lie in memory; plane p of the stage is fetched by wavefront p % 4.  The SGPR
    // offset is not range-checked: tiles past the last row block re-read the last one and
    // are never stored.
    const unsigned wlane = (unsigned)lane * 16u;
    auto dma_w = [&](const Where &w, int ks, int kb, int buf) {
#pragma unroll
        for (int p0 = 0; p0 < 3 * S::WTILES; p0 += S::WISSUERS) {
            const int p = p0 + wave;
            if (wave < S::WISSUERS) {
                const int t = p / 3, plane = p - 3 * t;
                const int wtile = min(w.bn0 / 32 + t, N / 32 - 1);
                uint8_t *dst = lds + S::WBASE + buf * S::WSTAGE + p * 1024;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    wrsrc, (void __attribute__((address_space(3))) *)dst, 16, wlane,
                    (unsigned)(wtile * KT + ks + kb) * FLEXQ_TILE_BYTES + 1024u * plane, 0, 0);
            }
        }
    };
    // weights and activations of an item's stage 0, weights (and, where activations run
    // two stages ahead, activations) of its stage 1
    auto issue_prologue = [&](const Item &it, const Where &w) {
        dma_w(w, it.ks, 0, 0);
        dma_x(w, it.ks, 0, 0);
        if (it.ke - it.ks > 1) {
            dma_w(w, it.ks, 1, 1);
            if (S::XA == 2) dma_x(w, it.ks, 1, 1);
        }
    };

    const int arow = (wm * MT) * 32 + (lane & 31);
    const int ahalf = lane >> 5;
    const int wfrag = S::WBASE + (wn * NT) * FLEXQ_TILE_BYTES + lane * 16;   // this lane's piece of tile nt = 0

    Item cur;
    Where at;
    if (!take(cur)) return;
    locate(cur, at);
    issue_prologue(cur, at);
    wait_vmcnt<0>();
    lds_barrier();

    for (;;) {
        const int ks = cur.ks, KN = cur.ke - cur.ks;

        v16i acc[MT][NT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0;

        // operands that live across stages: the stage's packed tiles, the activation
        // operands of two consecutive k-steps, the first weight operand of a stage
        PackedTile wreg[NT];
        v4i af[2][MT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const v4i *t = reinterpret_cast<const v4i *>(lds + wfrag + nt * FLEXQ_TILE_BYTES);
            wreg[nt].q0 = t[0];          // the other two planes follow at the start of the stage
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            af[0][mt] = *reinterpret_cast<const v4i *>(lds + lds_off(arow + 32 * mt, ahalf));
        v4i bf_first = unpack_kstep(wreg[0], 0);

        // One 128-k stage.  CUR = kb % XBUFS names the activation buffer (a constant, so that
        // the operand reads use immediate offsets), wcur = kb % 3 the weight buffer.
        // The MFMA takes the WEIGHT fragment as its row operand: the accumulators hold D^T.
        int wcur = 0;
        auto stage = [&](int kb, auto cur_tag) {
            constexpr int CUR = decltype(cur_tag)::value;
            const bool more1 = kb + 1 < KN, more2 = kb + 2 < KN;
            const int wnext = wcur == 2 ? 0 : wcur + 1, wnext2 = wcur == 0 ? 2 : wcur - 1;
            // First what the hand-over waits for (with everything older, the weights of
            // stage kb + 1 among it): the activations of stage kb + 1, where they run one
            // stage ahead.  Then, during step 3, what may stay in flight across it: the
            // loads for stage kb + 2.  All targets are free: an activation buffer was
            // last read before the previous stage's barrier, and the weight buffer is that
            // of stage kb - 1, whose last plane went to registers during that stage's first
            // k-step, before its barrier.
            if (S::XA == 1 && more1) dma_x(at, ks, kb + 1, (CUR + 1) % S::XBUFS);
            if (S::XA == 2 && more2) dma_x(at, ks, kb + 2, (CUR + 2) % S::XBUFS);

            const uint8_t *xs = lds + CUR * S::XSTAGE;
            const uint8_t *xn = lds + ((CUR + 1) % S::XBUFS) * S::XSTAGE;
            const uint8_t *wcb = lds + wfrag + wcur * S::WSTAGE;
            const uint8_t *wnb = lds + wfrag + wnext * S::WSTAGE;
            wcur = wnext;
            // The packed planes of this stage's tiles not yet in registers: only plane 0 (the
            // first k-step) is fetched after the hand-over, plane 1 during step 0 and plane 2
            // during step 1, well before the steps that expand them.
            auto rest_of_tiles = [&](int plane) {
#pragma unroll
                for (int n2 = 0; n2 < NT; ++n2) {
                    const v4i *t = reinterpret_cast<const v4i *>(wcb + n2 * FLEXQ_TILE_BYTES);
                    if (plane == 1) wreg[n2].q1 = t[64];
                    if (plane == 2) wreg[n2].q2 = t[128];
                }
            };
            // At the hand-over stage kb + 1 (weights and activations, every wavefront's
            // share) must have landed; the loads for stage kb + 2 may be in flight.
            auto hand_over = [&] {
                constexpr int XFLY = S::XA == 2 ? S::XDMA : 0;
                if (!more2)
                    wait_vmcnt<0>();
                else if (wave < S::WDMA_SPLIT)
                    wait_vmcnt<XFLY + S::WDMA_LOW>();
                else
                    wait_vmcnt<XFLY + S::WDMA_HIGH>();
                lds_barrier();
                if (more1) {
#pragma unroll
                    for (int n2 = 0; n2 < NT; ++n2) {
                        const v4i *t = reinterpret_cast<const v4i *>(wnb + n2 * FLEXQ_TILE_BYTES);
                        wreg[n2].q0 = t[0];
                    }
                }
            };
            static_assert((MT == 4 || MT == 2) && NT == 2, "the step tables below are written for these blockings");
            if constexpr (MT == 2) {
                // 64 x 64 per wavefront: eight steps of two MFMAs, two dwords of the next
                // step's operand expanded per MFMA; the dearer operands of the fourth k-step
                // (steps 6 and 7) are spread over steps 2..5, one dword per MFMA
                v4i bfc = bf_first, bf6 = {0, 0, 0, 0}, bf7 = {0, 0, 0, 0};
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const int j = s >> 1, nt = s & 1;
                    if (nt == 0) {
                        if (j < 3) {
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
                                af[(j + 1) & 1][mt] = *reinterpret_cast<const v4i *>(
                                    xs + lds_off(arow + 32 * mt, 2 * (j + 1) + ahalf));
                            if (j == 0) rest_of_tiles(1);
                        } else {
                            hand_over();
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (s == 1) {
                        rest_of_tiles(2);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (s == 3 && more2) {
                        dma_w(at, ks, kb + 2, wnext2);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (s == 7 && more1) {   // the next stage's first activation operands
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
                            af[0][mt] = *reinterpret_cast<const v4i *>(xn + lds_off(arow + 32 * mt, ahalf));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    const v4i cur_b = s == 6 ? bf6 : s == 7 ? bf7 : bfc;
                    v4i nxt = bfc;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        acc[mt][nt] = mfma_i8(cur_b, af[j & 1][mt], acc[mt][nt]);
#pragma unroll
                        for (int d = 2 * mt; d < 2 * mt + 2; ++d) {
                            if (s < 5) nxt[d] = unpack_kstep_dword(wreg[(s + 1) & 1], (s + 1) >> 1, d);
                            if (s == 7) nxt[d] = unpack_kstep_dword(wreg[0], 0, d);   // the next stage's first
                        }
                        if (s == 2) bf6[mt] = unpack_kstep_dword(wreg[0], 3, mt);
                        if (s == 3) bf6[2 + mt] = unpack_kstep_dword(wreg[0], 3, 2 + mt);
                        if (s == 4) bf7[mt] = unpack_kstep_dword(wreg[1], 3, mt);
                        if (s == 5) bf7[2 + mt] = unpack_kstep_dword(wreg[1], 3, 2 + mt);
                        {
                            int p0 = nxt[2 * mt], p1 = nxt[2 * mt + 1], p2 = bf6[(s & 1) * 2 + mt],
                                p3 = bf7[(s & 1) * 2 + mt];
                            asm volatile("" : "+v"(p0), "+v"(p1), "+v"(p2), "+v"(p3));   // pins the expansion here
                            nxt[2 * mt] = p0;
                            nxt[2 * mt + 1] = p1;
                            bf6[(s & 1) * 2 + mt] = p2;
                            bf7[(s & 1) * 2 + mt] = p3;
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    bfc = nxt;
                }
                bf_first = bfc;
            } else {
                v4i bfc = bf_first, bf6, bf7;
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const int j = s >> 1, nt = s & 1;
                    if (nt == 0) {
                        if (j < 3) {
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
                                af[(j + 1) & 1][mt] = *reinterpret_cast<const v4i *>(
                                    xs + lds_off(arow + 32 * mt, 2 * (j + 1) + ahalf));
                            if (j == 0) rest_of_tiles(1);
                        } else {
                            hand_over();
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (s == 1) {
                        rest_of_tiles(2);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (s == 3 && more2) {
                        dma_w(at, ks, kb + 2, wnext2);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (s == 7 && more1) {   // the next stage's first activation operands
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
                            af[0][mt] = *reinterpret_cast<const v4i *>(xn + lds_off(arow + 32 * mt, ahalf));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    const v4i cur_b = s == 6 ? bf6 : s == 7 ? bf7 : bfc;
                    v4i nxt = bfc;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        acc[mt][nt] = mfma_i8(cur_b, af[j & 1][mt], acc[mt][nt]);
                        // shadow work of this MFMA: one dword of an operand that is due later
                        if (s < 5) nxt[mt] = unpack_kstep_dword(wreg[(s + 1) & 1], (s + 1) >> 1, mt);
                        if (s == 3) bf6[mt] = unpack_kstep_dword(wreg[0], 3, mt);
                        if (s == 4) bf7[mt] = unpack_kstep_dword(wreg[1], 3, mt);
                        if (s == 7) nxt[mt] = unpack_kstep_dword(wreg[0], 0, mt);   // the next stage's first
                        {
                            int p0 = nxt[mt], p1 = bf6[mt], p2 = bf7[mt];
                            asm volatile("" : "+v"(p0), "+v"(p1), "+v"(p2));   // pins the expansion here
                            nxt[mt] = p0;
                            bf6[mt] = p1;
                            bf7[mt] = p2;
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    bfc = nxt;
                }
                bf_first = bfc;
            }
        };

        int kb = 0;
        for (; kb + S::XBUFS <= KN; kb += S::XBUFS) {
            stage(kb, std::integral_constant<int, 0>{});
            stage(kb + 1, std::integral_constant<int, 1>{});
            if constexpr (S::XBUFS == 3) stage(kb + 2, std::integral_constant<int, 2>{});
        }
        if (kb < KN) stage(kb, std::integral_constant<int, 0>{});
        if (S::XBUFS == 3 && kb + 1 < KN) stage(kb + 1, std::integral_constant<int, 1>{});
        // (every wavefront has passed the last stage's barrier with its LDS reads done: the
        // stage buffers are free)

        // ---- a run that is not a whole tile: leave the sums, or collect the others' ----
        bool finish = true;                              // this workgroup stores the tile
        unsigned fin_slabs = ~0u;                        // ... these 32-row slabs of each wavefront's part
        const int pieces = SK == 2 ? tail_wgs / item_count : 1;
        if (SK == 2 && KN != KT) {
            // EVEN CUT: every tile is cut into the same number of pieces, one per workgroup,
            // which therefore reach the end of their runs together.  The reduction is shared:
            // slab (wavefront w, row block mt) of the tile belongs to piece (w MT + mt) %
            // pieces.  A piece stores the sums of the slabs it does not own, adds its
            // stage count to the tile's counter, waits -- a bounded number of polls -- until
            // the count is complete, adds the other pieces' sums to the slabs it owns and
            // stores those.  No workgroup ever waits without a bound: a piece whose wait runs
            // out (its partners are not resident: a busy or smaller device) stores its own
            // slabs' sums as well, sets its bit in the tile's flag word and leaves; the piece
            // that completed the count closes the tile after its own slabs (one atomic OR)
            // and finishes the slabs of every piece whose bit it finds.  A piece that finds
            // the tile closed when it sets its bit finishes its slabs itself (all sums are
            // there by then).  Each piece ends with one add to the flag word's leave count;
            // the last to leave clears counter and flags for the next call.
            constexpr int kScopeAgent = 16;
            constexpr unsigned kClosed = 1u << 16, kLeave = 1u << 20;
            constexpr int PIECE_BYTES = S::BM * 256 * 4;      // one piece's int32 sums: slot `vt` of the area
            const __amdgpu_buffer_rsrc_t prsrc = __builtin_amdgcn_make_buffer_rsrc(
                a.partial, 0, (unsigned)tail_wgs * (unsigned)PIECE_BYTES, 0x00020000);
            // (the lane number passes through an opaque statement so that nothing derived
            // from it here is computed ahead of the main loop and kept in registers across it)
            int lane_m = lane;
            asm volatile("" : "+v"(lane_m));
            const unsigned in_slot = (unsigned)(wave * (PIECE_BYTES / WAVES) + lane_m * 16);
            const int tj = cur.tj;
            const int me = vt - tj * pieces;
            unsigned *flags = a.counters + 2048;
            auto owner = [&](int mt) { return (wave * MT + mt) % pieces; };      // uniform
            auto store_slab = [&](int mt) {
                const unsigned mine = (unsigned)vt * PIECE_BYTES + in_slot;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const v4u piece = {(unsigned)acc[mt][nt][4 * q], (unsigned)acc[mt][nt][4 * q + 1],
                                           (unsigned)acc[mt][nt][4 * q + 2], (unsigned)acc[mt][nt][4 * q + 3]};
                        __builtin_amdgcn_raw_buffer_store_b128(
                            piece, prsrc, mine + (unsigned)(((mt * NT + nt) * 4 + q) * 1024), 0, kScopeAgent);
                    }
            };
            auto load_slab = [&](v4u (&got)[NT * 4], int mt, int from) {
                const unsigned theirs = (unsigned)(tj * pieces + from) * PIECE_BYTES + in_slot;
#pragma unroll
                for (int i = 0; i < NT * 4; ++i)
                    got[i] = __builtin_amdgcn_raw_buffer_load_b128(
                        prsrc, theirs + (unsigned)((mt * NT * 4 + i) * 1024), 0, kScopeAgent);
            };
            auto sum_slab = [&](const v4u (&got)[NT * 4], int mt) {
#pragma unroll
                for (int i = 0; i < NT * 4; ++i)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[mt][i >> 2][4 * (i & 3) + c] += (int)got[i][c];
            };
            // every other piece's sums of slab mt, the next piece's loads in flight while one
            // piece's sums are added (one round trip in all instead of one per piece)
            auto gather_slab = [&](int mt) {
                auto following = [&](int from) {
                    const int n = from + 1;
                    return n == me ? n + 1 : n;
                };
                v4u got_a[NT * 4], got_b[NT * 4];
                int from = following(-1);
                load_slab(got_a, mt, from);
                for (;;) {
                    int nxt = following(from);
                    if (nxt < pieces) load_slab(got_b, mt, nxt);
                    sum_slab(got_a, mt);
                    if (nxt >= pieces) break;
                    from = following(nxt);
                    if (from < pieces) load_slab(got_a, mt, from);
                    sum_slab(got_b, mt);
                    if (from >= pieces) break;
                }
            };
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                if (owner(mt) != me) store_slab(mt);
            wait_vmcnt<0>();
            lds_barrier();
            if (tid == 0) {
                const unsigned prev = __hip_atomic_fetch_add(&a.counters[tj], (unsigned)KN, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_AGENT);
                bool all = prev + (unsigned)KN == (unsigned)KT;
                const int completed = all ? 1 : 0;
                for (int poll = 0; !all && poll < a.spin; ++poll) {
                    __builtin_amdgcn_s_sleep(8);
                    all = __hip_atomic_load(&a.counters[tj], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                          (unsigned)KT;
                }
                s_last = all ? 1 + completed : 0;
            }
            lds_barrier();
            int state = __builtin_amdgcn_readfirstlane(s_last);   // 0 gave up, 1 all sums there, 2 and this piece completed the count
            lds_barrier();                                        // (read by all before it is written again)
            if (state == 0) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    if (owner(mt) == me) store_slab(mt);
                wait_vmcnt<0>();
                lds_barrier();
                if (tid == 0) {
                    const unsigned old = __hip_atomic_fetch_or(&flags[tj], 1u << me, __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_AGENT);
                    s_last = (old & kClosed) ? 1 : 0;
                }
                lds_barrier();
                state = __builtin_amdgcn_readfirstlane(s_last);
                lds_barrier();
            }
            fin_slabs = 0;
            if (state != 0) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    if (owner(mt) == me) {
                        gather_slab(mt);
                        fin_slabs |= 1u << mt;
                    }
                if (state == 2) {
                    if (tid == 0) {
                        const unsigned old = __hip_atomic_fetch_or(&flags[tj], kClosed, __ATOMIC_RELAXED,
                                                                   __HIP_MEMORY_SCOPE_AGENT);
                        s_last = (int)(old & 0xffffu);
                    }
                    lds_barrier();
                    const unsigned gone = (unsigned)__builtin_amdgcn_readfirstlane(s_last);
                    lds_barrier();
                    if (gone != 0) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
                            if ((gone >> owner(mt)) & 1u) {
                                gather_slab(mt);
                                fin_slabs |= 1u << mt;
                            }
                    }
                }
            }
            if (tid == 0) {
                const unsigned old = __hip_atomic_fetch_add(&flags[tj], kLeave, __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT);
                if ((int)(old >> 20) + 1 == pieces) {
                    __hip_atomic_store(&a.counters[tj], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(&flags[tj], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            finish = fin_slabs != 0;
        } else if (SK == 1 && KN != KT) {
            // [slot][wavefront][block mt, nt][quarter][lane] 16-byte pieces: every store and
            // load below is one contiguous KiB per wavefront.  Cache policy bit 4 = sc1 =
            // device scope: the access goes to memory all XCDs share.
            constexpr int kScopeAgent = 16;
            const __amdgpu_buffer_rsrc_t prsrc = __builtin_amdgcn_make_buffer_rsrc(
                a.partial, 0, (unsigned)(2 * tail_wgs) * (unsigned)SLOT_BYTES, 0x00020000);
            const unsigned in_slot = (unsigned)(wave * (SLOT_BYTES / WAVES) + lane * 16);
            const int tj = cur.tj;
            const long tile_begin = (long)tj * KT;
            // a run leaves at most two partial tiles: slot 2 vt for the one it begins in,
            // 2 vt + 1 for the one it ends in
            const unsigned mine = (unsigned)(2 * vt + (run_begin < tile_begin ? 1 : 0)) * SLOT_BYTES + in_slot;
            // The tile a run ends in is begun by this workgroup and finished by its successor,
            // which reached it first thing: by now it has most likely arrived, and so has
            // everybody else.  One look at the counter tells (it only ever grows until the
            // last arrival; a workgroup adds to it after its stores are acknowledged): then
            // this workgroup is the last without storing its own sums first.
            int early = 0;
            if (run_begin < tile_begin) {
                if (tid == 0) {
                    const unsigned seen = __hip_atomic_load(&a.counters[tj], __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT);
                    s_last = (seen + (unsigned)KN == (unsigned)KT);
                    if (s_last)
                        __hip_atomic_store(&a.counters[tj], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                lds_barrier();
                early = __builtin_amdgcn_readfirstlane(s_last);
            }
            if (!early) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const v4u piece = {(unsigned)acc[mt][nt][4 * q], (unsigned)acc[mt][nt][4 * q + 1],
                                               (unsigned)acc[mt][nt][4 * q + 2], (unsigned)acc[mt][nt][4 * q + 3]};
                            __builtin_amdgcn_raw_buffer_store_b128(
                                piece, prsrc, mine + (unsigned)(((mt * NT + nt) * 4 + q) * 1024), 0, kScopeAgent);
                        }
                // Once the stores are acknowledged (vmcnt 0) they are visible device-wide; the
                // barrier plus one relaxed device-scope add to the tile's stage count publishes
                // them.  Whoever brings the count to KT is the last and resets it.
                wait_vmcnt<0>();
                lds_barrier();
                if (tid == 0) {
                    const unsigned prev = __hip_atomic_fetch_add(&a.counters[tj], (unsigned)KN, __ATOMIC_RELAXED,
                                                                 __HIP_MEMORY_SCOPE_AGENT);
                    s_last = (prev + (unsigned)KN == (unsigned)KT);
                    if (s_last)
                        __hip_atomic_store(&a.counters[tj], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                lds_barrier();
                finish = __builtin_amdgcn_readfirstlane(s_last) != 0;   // wavefront-uniform
            }
            if (finish) {
                // the runs that meet this tile: the one holding its first stage through the one
                // holding its last (run w is [w U / W, (w + 1) U / W))
                const long W = tail_wgs;
                const int va = (int)(((tile_begin + 1) * W + U - 1) / U) - 1;
                const int vb = (int)(((tile_begin + KT) * W + U - 1) / U) - 1;
                for (int w2 = va; w2 <= vb; ++w2) {
                    if (w2 == vt) continue;
                    const long begin2 = (long)w2 * U / W;
                    const unsigned theirs =
                        (unsigned)(2 * w2 + (begin2 < tile_begin ? 1 : 0)) * SLOT_BYTES + in_slot;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        v4u got[NT * 4];
#pragma unroll
                        for (int i = 0; i < NT * 4; ++i)
                            got[i] = __builtin_amdgcn_raw_buffer_load_b128(
                                prsrc, theirs + (unsigned)((mt * NT * 4 + i) * 1024), 0, kScopeAgent);
#pragma unroll
                        for (int i = 0; i < NT * 4; ++i)
#pragma unroll
                            for (int c = 0; c < 4; ++c) acc[mt][i >> 2][4 * (i & 3) + c] += (int)got[i][c];
                    }
                }
            }
        }

        // ---- the next item's first stages set out now, before this tile is stored ----
        Item nxt_item;
        Where nxt_at;
        const bool has_next = take(nxt_item);
        if (has_next) {
            locate(nxt_item, nxt_at);
            issue_prologue(nxt_item, nxt_at);
        }

        // ---- epilogue --------------------------------------------------------------
        // Register r of block (mt, nt) at lane l is token 32 mt' + (l & 31), channel
        // 32 nt' + 8 (r / 4) + 4 (l >> 5) + r % 4: four consecutive channels per register
        // quarter.  Scale (sx[m] * sw[n] in fp32, exact; the 1/4 of the 4x weights folded
        // into sx, a power of two) and convert in registers, pass 8-byte pieces of fp16
        // through this wavefront's own LDS rows (stride NT * 64 + 16 bytes), read 16-byte
        // pieces back so that the lanes of a row hold consecutive pieces, and store whole
        // lines.  Rows beyond M and column blocks beyond N are never stored.
        if (finish) {
            const int bm0 = at.bm0, bn0 = at.bn0;
            // (the lane number passes through an opaque statement: what the epilogue derives
            // from it is recomputed per tile, a handful of operations, instead of being kept
            // in registers -- or spilled -- across the main loop)
            int lane_e = lane;
            asm volatile("" : "+v"(lane_e));
            const int ml = lane_e & 31, hh = lane_e >> 5;
            const int n_wave = bn0 + wn * NT * 32;
            // (kept as packed fp16 and converted where used: sixteen registers, not thirty-two)
            uint2 sw4[NT][4];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const bool cvalid = n_wave + nt * 32 < N;                 // uniform; N is a multiple of 32
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n_wave + nt * 32 + 8 * q + 4 * hh;
                    sw4[nt][q] = cvalid ? *reinterpret_cast<const uint2 *>(a.scales + n) : make_uint2(0u, 0u);
                }
            }
            float sxq[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = bm0 + (wm * MT + mt) * 32 + ml;
                sxq[mt] = m < M ? 0.25f * h2f(a.sx[m]) : 0.0f;
            }
            uint8_t *stg = lds + S::STG + wave * (32 * S::ESTRIDE);
            constexpr int LPR = NT * 4;                 // lanes per staged row, 16 bytes (8 channels) each
            constexpr int RPI = 64 / LPR;               // rows per read instruction
            const int erow = lane_e / LPR, echunk = lane_e % LPR;
            const bool ecvalid = n_wave + echunk * 8 < N;
            // the output as a buffer from this wavefront's corner: a lane's offset is fixed,
            // the row offset is an SGPR
            const long corner = (long)(bm0 + wm * MT * 32) * N + n_wave;
            const __amdgpu_buffer_rsrc_t yrsrc = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(a.y + corner), 0, (unsigned)(((long)(MT * 32 - 1) * N + NT * 32) * 2), 0x00020000);
            const unsigned yoff = (unsigned)((erow * N + echunk * 8) * 2);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m_slab = bm0 + (wm * MT + mt) * 32;
                if (m_slab >= M) break;                          // uniform: nothing below is stored
                if (SK == 2 && !((fin_slabs >> mt) & 1u)) continue;   // uniform: another piece stores this slab
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const unsigned swp[2] = {sw4[nt][q].x, sw4[nt][q].y};
                        uint16_t h[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const float swc = h2f((uint16_t)(swp[c >> 1] >> (16 * (c & 1))));
                            h[c] = f2h((float)acc[mt][nt][4 * q + c] * (sxq[mt] * swc));
                        }
                        uint2 out2;
                        out2.x = (unsigned)h[0] | ((unsigned)h[1] << 16);
                        out2.y = (unsigned)h[2] | ((unsigned)h[3] << 16);
                        *reinterpret_cast<uint2 *>(stg + ml * S::ESTRIDE + (nt * 32 + 8 * q + 4 * hh) * 2) = out2;
                    }
                if (a.acc_out) {     // the exact int32 sums, straight from the registers
                    const int m = m_slab + ml;
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int n = n_wave + nt * 32 + 8 * q + 4 * hh;
                            if (m < M && n < N) {
                                const v4i four = {acc[mt][nt][4 * q] >> 2, acc[mt][nt][4 * q + 1] >> 2,
                                                  acc[mt][nt][4 * q + 2] >> 2, acc[mt][nt][4 * q + 3] >> 2};
                                *reinterpret_cast<v4i *>(a.acc_out + (long)m * N + n) = four;
                            }
                        }
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // own region only: no barrier
#pragma unroll
                for (int i = 0; i < 32 / RPI; ++i) {
                    const int row = i * RPI + erow;
                    const v4u piece = *reinterpret_cast<const v4u *>(stg + row * S::ESTRIDE + echunk * 16);
                    if (m_slab + row < M && ecvalid)
                        __builtin_amdgcn_raw_buffer_store_b128(piece, yrsrc, yoff,
                                                               (unsigned)((mt * 32 + i * RPI) * N * 2), 0);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the next slab overwrites
            }
        }
        if (!has_next) break;
        // the next item's first stages (every wavefront's share) have landed
        wait_vmcnt<0>();
        lds_barrier();
        cur = nxt_item;
        at = nxt_at;
    }
#endif
}

// FORM 3: `full_count` low tiles (tiles_m counts 128-row tiles) and nothing else.  FORM 5:
// `tail_count` low tiles, each cut along K into tail_wgs / tail_count pieces.
// FORM 0: `full_count` whole tiles.  FORM 1: then the `tail_count` tiles that follow them as
// 2 * tail_count half tiles.  FORM 2: then those tiles cut along K into `tail_wgs` runs
// across tile borders.  FORM 4: then those tiles each cut into tail_wgs / tail_count pieces.
// One launch: a second launch for the tail would cost the first one's drain and the
// end-of-kernel cache write-back in between (about 20 us, measured).
template <int FORM>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gemm_wlds_kernel(flexq::LinearArgs a, int tiles_m, int tiles_n, int full_count, int tail_count,
                      int tail_wgs)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    __shared__ int s_last;
    if (FORM == 3) {   // every item a low tile (128 x 256)
        run_items<3, 0>(a, lds, s_last, tiles_m, tiles_n, 0, full_count, 0);
        return;
    }
    if (FORM == 5) {   // every low tile cut evenly along K
        run_items<3, 2>(a, lds, s_last, tiles_m, tiles_n, 0, tail_count, tail_wgs);
        return;
    }
    if (full_count > 0) run_items<2, 0>(a, lds, s_last, tiles_m, tiles_n, 0, full_count, 0);
#if defined(__HIP_DEVICE_COMPILE__)
    // The two phases lay LDS out differently: every wavefront must be through with its last
    // epilogue's staging rows before anyone's first loads of the next phase land on them.
    if (FORM != 0) lds_barrier();
#endif
    if (FORM == 1) run_items<1, 0>(a, lds, s_last, tiles_m, tiles_n, full_count, 2 * tail_count, 0);
    if (FORM == 2) run_items<2, 1>(a, lds, s_last, tiles_m, tiles_n, full_count, tail_count, tail_wgs);
    if (FORM == 4) run_items<2, 2>(a, lds, s_last, tiles_m, tiles_n, full_count, tail_count, tail_wgs);
}

}  // namespace

namespace flexq {

size_t low_cut_bytes(int pieces_in_all) { return (size_t)pieces_in_all * (128 * 256 * 4); }

// 65 to 128 tokens on a layer too narrow to fill the chip with 128x256 tiles: every tile
// cut along K into this many pieces (0: the form does not apply).  Measured on the
// LLaMA-2-7B and 70B layers at 96 and 128 tokens: fastest with 130 to 190 pieces in all
// (beyond that the partial sums of all pieces, which cross the memory system at the same
// moment, cost more than the shorter runs save) and runs of at least 13 stages; 5-22 %
// faster than 128x128 tiles with K splits in 11 cells of 12.
int low_cut_pieces(int M, int N, int K)
{
    if (M <= 64 || M > 128) return 0;
    const int tiles = (N + 255) / 256, KT = K / FLEXQ_TILE_K;
    int pieces = 176 / tiles;
    if (pieces > KT / 13) pieces = KT / 13;
    if (pieces > 8) pieces = 8;
    return pieces >= 2 ? pieces : 0;
}

StreamKPlan streamk_plan(int M, int N, int K)
{
    StreamKPlan p;
    p.tiles = ((M + 256 - 1) / 256) * ((N + 255) / 256);
    p.full_tiles = p.tiles / kStreamKGrid * kStreamKGrid;
    p.tail_tiles = p.tiles - p.full_tiles;
    // two slots per run; a run is at least one 128-k stage, and there are at most 256 runs
    const long stages = (long)p.tail_tiles * (K / FLEXQ_TILE_K);
    p.partial_bytes = (size_t)2 * (size_t)(stages < kStreamKGrid ? stages : kStreamKGrid) * SLOT_BYTES;
    return p;
}

// Estimated run time in microseconds of the fastest launch form, from measured constants
// of the MI355X.  A 128-k stage of a whole tile takes 1.50 us when every CU has a tile and
// 1.20 us when at most two thirds of them have (the chip is power-limited: idle CUs let
// the others clock higher), a half tile's stage 0.93 / 0.75 us; a tile costs 4 us more for
// its first loads and its epilogue.  Meeting in the workspace costs 7 to 27 us when every
// tile is cut into the same number of pieces (one partial tile per workgroup, the pieces of
// a tile share its reduction); about 45 us when the tail is simply cut into 256 equal
// runs, which then begin and end inside tiles (two partial tiles per workgroup, the last
// to arrive at a tile reads the others').
WldsChoice gemm_wlds_choose(int M, int N, int K, bool may_cut)
{
    const StreamKPlan p = streamk_plan(M, N, K);
    const int KT = K / FLEXQ_TILE_K;
    auto busy = [](double frac) { return frac <= 0.65 ? 0.0 : (frac - 0.65) / 0.35; };
    auto whole_us = [&](int tiles) { return (1.20 + 0.30 * busy(tiles / 256.0)) * KT + 4.0; };
    auto half_us = [&](int halves) { return (0.75 + 0.18 * busy(halves / 256.0)) * KT + 4.0; };
    const double rounds = (double)(p.full_tiles / kStreamKGrid) * whole_us(kStreamKGrid);
    WldsChoice best{rounds + (p.tail_tiles ? whole_us(p.tail_tiles) : 0.0), 0, 0};
    if (p.tail_tiles == 0) return best;
    {   // the tail as half tiles: one half round, or two
        const int halves = 2 * p.tail_tiles;
        const double t = rounds + (halves <= kStreamKGrid ? half_us(halves)
                                                          : half_us(kStreamKGrid) + half_us(halves - kStreamKGrid));
        if (t < best.us) best = WldsChoice{t, 1, halves};
    }
    if (!may_cut) return best;
    const double stage_us = 1.50;
    // every tile cut into S pieces that share its reduction: meeting costs by the pieces
    // per tile (a piece adds S - 1 others' sums) and by their number in all (the partial sums
    // of all pieces cross the memory system at the same moment); measured on the 8192- and
    // 28672-deep layers at 256 .. 3072 tokens, 2 .. 8 pieces per tile, 64 .. 256 in all
    for (int S = 2; S <= 16 && p.tail_tiles * S <= kStreamKGrid && S <= KT; ++S) {
        const int wgs = p.tail_tiles * S;
        const double meet = 1.0 + 2.0 * S + 0.03 * wgs + (wgs > 192 ? 0.03 * (wgs - 192) : 0.0);
        const double t = rounds + (1.15 + 0.35 * busy(wgs / 256.0)) * ((KT + S - 1) / S) + 4.0 + meet;
        if (t < best.us) best = WldsChoice{t, 2, wgs};
    }
    if ((long)p.tail_tiles * KT >= 2L * kStreamKGrid) {
        const double t = rounds + stage_us * KT * p.tail_tiles / kStreamKGrid + 4.0 + 45.0;
        if (t < best.us) best = WldsChoice{t, 2, kStreamKGrid};
    }
    return best;
}

namespace {

constexpr int kLdsMax(int a, int b) { return a > b ? a : b; }
constexpr int kLdsBytes = kLdsMax(Shape<2>::LDS_BYTES, kLdsMax(Shape<1>::LDS_BYTES, Shape<3>::LDS_BYTES));

template <int FORM>
hipError_t launch_form(const LinearArgs &a, int tiles_m, int tiles_n, int full_count, int tail_count,
                       int tail_wgs, int grid, hipStream_t st)
{
    auto kern = gemm_wlds_kernel<FORM>;
    static std::atomic<unsigned long long> lds_allowed{0};
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), kLdsBytes, lds_allowed);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * WAVES), kLdsBytes, st, a, tiles_m, tiles_n,
                       full_count, tail_count, tail_wgs);
    return hipGetLastError();
}

// workgroups for `items` items: a multiple of 8 (one share per XCD), at most one per CU
// on the 256-CU device the persistent forms are laid out for, else one per item
int grid_for(int items)
{
    const int g = (items + 7) / 8 * 8;
    return device_cu_count() == kStreamKGrid && g > kStreamKGrid ? kStreamKGrid : g;
}

}  // namespace

hipError_t launch_gemm_wlds(const LinearArgs &a, int tail_form, int tail_wgs, hipStream_t st)
{
    if (a.group != 0 || a.split_k > 1 || a.sxg) return hipErrorInvalidValue;
    if (tail_form == 3) {   // low tiles throughout
        const int low_m = (a.M + 127) / 128, cols = (a.N + 255) / 256;
        return launch_form<3>(a, low_m, cols, low_m * cols, 0, 0, grid_for(low_m * cols), st);
    }
    if (tail_form == 5) {   // low tiles, each cut into tail_wgs / tiles pieces
        const int low_m = (a.M + 127) / 128, cols = (a.N + 255) / 256, tiles = low_m * cols;
        const int pieces = tail_wgs / tiles;
        if (tail_wgs % tiles != 0 || pieces < 2 || pieces > 16 || pieces > a.K / FLEXQ_TILE_K ||
            tail_wgs > kStreamKGrid || a.partial_bytes < low_cut_bytes(tail_wgs) ||
            device_cu_count() != kStreamKGrid)
            return hipErrorInvalidValue;
        return launch_form<5>(a, low_m, cols, 0, tiles, tail_wgs, (tail_wgs + 7) / 8 * 8, st);
    }
    const int tiles_m = (a.M + 256 - 1) / 256, tiles_n = (a.N + 255) / 256;
    const StreamKPlan p = streamk_plan(a.M, a.N, a.K);
    // without room for the partial sums, or on a device that is not 256 CUs wide, a tail
    // that was to be cut runs as whole tiles
    if (tail_form == 2 && (tail_wgs <= 0 || a.partial_bytes < p.partial_bytes ||
                           device_cu_count() != kStreamKGrid))
        tail_form = 0;
    if (tail_form == 0 || p.tail_tiles == 0)      // every tile whole
        return launch_form<0>(a, tiles_m, tiles_n, p.tiles, 0, 0, grid_for(p.tiles), st);
    // the whole rounds first, then the tiles of the last, partial round in their own form
    const int g_full = p.full_tiles ? grid_for(p.full_tiles) : 0;
    if (tail_form == 1) {
        const int g = grid_for(2 * p.tail_tiles);
        return launch_form<1>(a, tiles_m, tiles_n, p.full_tiles, p.tail_tiles, 0, g > g_full ? g : g_full, st);
    }
    // a run is at least one stage, and the tail has at most 256 runs
    const long stages = (long)p.tail_tiles * (a.K / FLEXQ_TILE_K);
    if (tail_wgs > kStreamKGrid) tail_wgs = kStreamKGrid;
    if (tail_wgs > stages) tail_wgs = (int)stages;
    const int g = (tail_wgs + 7) / 8 * 8;
    // every tile cut into the same number of pieces (each at least one stage): the pieces
    // of a tile end together and share its reduction
    const int pieces = tail_wgs / p.tail_tiles;
    if (tail_wgs % p.tail_tiles == 0 && pieces >= 2 && pieces <= 16 && pieces <= a.K / FLEXQ_TILE_K)
        return launch_form<4>(a, tiles_m, tiles_n, p.full_tiles, p.tail_tiles, tail_wgs, g > g_full ? g : g_full, st);
    return launch_form<2>(a, tiles_m, tiles_n, p.full_tiles, p.tail_tiles, tail_wgs, g > g_full ? g : g_full, st);
}

}  // namespace flexq
