// Tiled i8-MFMA GEMM for prefill-sized M.
//
// Large M makes the layer a dense contraction, so the matrix pipe is the
// roofline (the paper measures no batch above 8; Section 4.3.6 describes its
// pipeline, which this kernel re-creates for CDNA4 in its own way):
//   - activations (int8) go global -> LDS by DMA (buffer loads with the lds
//     bit: no registers in between), three stage buffers of 128 k, two stages
//     ahead, in an XOR-swizzled row layout so that the 16-byte MFMA-operand
//     reads are bank-conflict free;
//   - packed weights never touch LDS: each wavefront loads the 3 KiB tiles of
//     its own columns straight into registers two stages ahead and expands them
//     to int8 (nine VALU operations per 16 weights) in the shadow of the MFMAs;
//     an expanded operand is reused by MT MFMAs, which is what keeps the VALU
//     work hidden;
//   - stages are handed over with counted s_waitcnt vmcnt and a raw s_barrier;
//   - the epilogue shifts the 4x accumulators back, transposes them through
//     LDS, applies sx[m]*sw[n] in fp32 and stores whole lines of fp16 (Section
//     4.3.4, fused dequantization; Section 4.3.2, coalesced write-back);
//   - for mid-size M, K can be split over several workgroups per output tile;
//     the last one to finish adds the partial sums (exact for int32).
// The default shape is a 128x256 tile per workgroup of four wavefronts, two
// workgroups per CU: what one workgroup loses at its barrier, prologue and
// epilogue the other fills with MFMAs.  Workgroup ids are remapped so that the
// workgroups an XCD runs at one time form a compact block of output tiles and
// share operand panels in that XCD's L2.
#include "flexq_device.h"
#include "flexq_kernels.h"
#include "gemm_common.h"
#include <type_traits>

namespace {

template <int WM, int WN, int MT, int NT, int GROUP, int WPE>
__global__ __launch_bounds__(64 * WM * WN) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void gemm_kernel(flexq::LinearArgs a, int tiles_m, int tiles_n)
{
#if defined(__HIP_DEVICE_COMPILE__)  // buffer-resource builtins exist in the device pass only
    constexpr int WAVES = WM * WN;
    constexpr int BM = WM * MT * 32;
    constexpr int BN = WN * NT * 32;
    constexpr int XSTAGE = BM * 128;            // bytes of one activation stage in LDS
    constexpr int XDMA = BM / 8 / WAVES;        // 1 KiB LDS-DMA loads per wavefront per stage
    constexpr int WLOADS = 3 * NT;              // 16-byte register loads per lane per stage
    static_assert(BM % (8 * WAVES) == 0, "tile / wavefront mismatch");
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];  // 3 * XSTAGE

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int M = a.M, N = a.N, K = a.K;
    const int KT = K / FLEXQ_TILE_K;

    // ---- XCD-aware tile choice: blocks 8 apart share an XCD ---------------
    // K splits of one output tile are adjacent block ids
    const int KS = a.split_k;
    const int ksplit = blockIdx.x % KS;
    const int kb0 = (int)((long)ksplit * KT / KS);              // first 128-k stage of this block
    const int KN = (int)((long)(ksplit + 1) * KT / KS) - kb0;   // and how many
    const int nblk = tiles_m * tiles_n;
    int bid = blockIdx.x / KS;
    const int tile_id = bid;
    {
        const int per = nblk / 8, rem = nblk % 8;
        const int xcd = bid % 8, slot = bid / 8;
        // blocks of XCD x occupy a contiguous range of logical ids
        bid = xcd * per + (xcd < rem ? xcd : rem) + slot;
    }
    constexpr int SUP_M = 8;  // super-block: 8 tiles along m, then next n
    const int sup = bid / (SUP_M * tiles_n);
    const int first_m = sup * SUP_M;
    const int span_m = min(SUP_M, tiles_m - first_m);
    const int in_sup = bid - sup * SUP_M * tiles_n;
    const int tile_m = first_m + in_sup % span_m;
    const int tile_n = in_sup / span_m;
    const int bm0 = tile_m * BM, bn0 = tile_n * BN;

    // ---- activations: global -> LDS by DMA, no registers in between --------
    // DMA load q of a stage fills LDS bytes [1024q, 1024q + 1024) = rows 8q..8q+7;
    // lane i lands at 16-byte slot i, i.e. row 8q + i/8, position i%8, and must
    // therefore FETCH the chunk the swizzle keeps at that position.
    // Buffer addressing keeps the per-stage address arithmetic on the scalar
    // unit: a lane's offset is fixed for the whole kernel, the k offset is an
    // SGPR, and rows beyond M fall outside the buffer and read as zero.
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)a.xq, 0, (unsigned)((long)M * K), 0x00020000);
    unsigned xoff[XDMA];
#pragma unroll
    for (int i = 0; i < XDMA; ++i) {
        const int q = wave * XDMA + i;
        const int row = 8 * q + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        xoff[i] = (unsigned)(bm0 + row) * (unsigned)K + 16u * c;
    }
    auto dma_x = [&](int kb, int buf) {
#pragma unroll
        for (int i = 0; i < XDMA; ++i) {
            uint8_t *dst = lds + buf * XSTAGE + (wave * XDMA + i) * 1024;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                xrsrc, (void __attribute__((address_space(3))) *)dst, 16, xoff[i],
                (kb0 + kb) * FLEXQ_TILE_K, 0, 0);
        }
    };

    // ---- per-wave packed tiles: SGPR tile offset + lane * 16 -----------------
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)a.packed, 0, (unsigned)((long)N * K / 4 * 3), 0x00020000);
    bool wvalid[NT];
    int wnb[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        wnb[nt] = bn0 / 32 + wn * NT + nt;
        wvalid[nt] = wnb[nt] < N / 32;
        // the SGPR offset is not range-checked: tiles past the last row block
        // re-read the last one and are never stored
        if (!wvalid[nt]) wnb[nt] = N / 32 - 1;
    }
    const unsigned wlane = (unsigned)lane * 16u;

    // ---- GROUP == 2: the tile's token scales of one group, 2 bytes each, follow the
    // activations into LDS (one 4-byte DMA load per lane covers the 128 rows).  A ring of
    // four slots: a stage's scales are still read at the start of the next stage (the
    // scaling runs one block behind the MFMAs), so its slot is reused three stages later,
    // with a stage barrier in between.  Every wavefront issues the same load (the bytes
    // land identically), which keeps the per-wavefront load count uniform.
    static_assert(GROUP != 2 || (BM == 128 && WM == 1), "one 4-byte DMA load per lane covers the tile's rows");
    constexpr int XSRING = 3 * XSTAGE;          // byte offset of the ring in LDS
    constexpr int XSSLOT = BM * 2;
    const __amdgpu_buffer_rsrc_t xsrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(GROUP == 2 ? a.sxg : a.scales), 0,
        GROUP == 2 ? (unsigned)((long)KT * a.sxg_stride * 2) : 0u, 0x00020000);
    // lanes whose two rows lie beyond M fetch nothing (an offset past the buffer reads as zero)
    const unsigned xsoff = bm0 + 2 * lane < M ? (unsigned)(bm0 + 2 * lane) * 2u : 0x80000000u;
    auto dma_xs = [&](int kb) {
        if constexpr (GROUP == 2) {
            uint8_t *dst = lds + XSRING + (kb & 3) * XSSLOT;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                xsrsrc, (void __attribute__((address_space(3))) *)dst, 4, xsoff,
                (unsigned)(kb0 + kb) * (unsigned)a.sxg_stride * 2u, 0, 0);
        }
    };
    const int xslane = 8 * (lane >> 5);         // register r of a block: row 8 (r / 4) + 4 (lane / 32) + r % 4
    auto xs_ptr = [&](int kb, int mt, int q) {  // the four scales of quarter q of row block mt, stage kb
        return reinterpret_cast<const uint2 *>(lds + XSRING + (kb & 3) * XSSLOT + 64 * mt + 16 * q + xslane);
    };

    v16i acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0;
    static_assert(!GROUP || MT * NT >= 2, "group mode scales up to two blocks behind");
    v16f facc[GROUP ? MT : 1][GROUP ? NT : 1];
    v16i gpart[3];             // group mode: int32 sums of the block in flight and the two before
    float gs_prev[NT];         // scales of the stage before, for the blocks it leaves unscaled
    uint2 xsq = make_uint2(0u, 0u);   // GROUP == 2: the four token scales of the quarter due next
    if (GROUP) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) gs_prev[nt] = 0.0f;
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) gpart[i][r] = 0;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) facc[GROUP ? mt : 0][GROUP ? nt : 0][r] = 0.0f;
    }

    PackedTile wreg[3][NT];
    uint16_t gsreg[3][NT];
    auto load_w = [&](int kb, auto buf_tag) {
        constexpr int B = decltype(buf_tag)::value;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const unsigned soff = (unsigned)(wnb[nt] * KT + kb0 + kb) * FLEXQ_TILE_BYTES;
            wreg[B][nt].q0 = (v4i)__builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane, soff, 0);
            wreg[B][nt].q1 = (v4i)__builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane, soff + 1024, 0);
            wreg[B][nt].q2 = (v4i)__builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane, soff + 2048, 0);
            if (GROUP) gsreg[B][nt] = a.scales[((long)wnb[nt] * KT + kb0 + kb) * 32 + (lane & 31)];
        }
    };

    // prologue: stages 0 and 1 in flight, stage 0 landed
    dma_x(0, 0);
    load_w(0, std::integral_constant<int, 0>{});
    dma_xs(0);
    if (KN > 1) {
        dma_x(1, 1);
        load_w(1, std::integral_constant<int, 1>{});
        dma_xs(1);
    }
    if constexpr (GROUP == 2)   // "the stage before the first": its scales are read (times zero sums)
        *reinterpret_cast<unsigned *>(lds + XSRING + 3 * XSSLOT + 4 * lane) = 0u;
    wait_vmcnt<0>();
    v4i bf_first = unpack_kstep(wreg[0][0], 0);   // weight operand of a stage's first step
    lds_barrier();

    const int arow = (wm * MT) * 32 + (lane & 31);
    const int ahalf = lane >> 5;

    // One 128-k stage.  CUR = kb % 3 names the LDS buffer and register set it reads.
    auto stage = [&](int kb, auto cur_tag) {
        constexpr int CUR = decltype(cur_tag)::value;
        constexpr int NXT2 = (CUR + 2) % 3;
        const bool more2 = kb + 2 < KN;
        if (more2) {  // two stages ahead: that buffer was last read in stage kb - 1
            dma_x(kb + 2, NXT2);
            load_w(kb + 2, std::integral_constant<int, NXT2>{});
            dma_xs(kb + 2);
        }
        const uint8_t *xs = lds + CUR * XSTAGE;
        if constexpr (GROUP) {
            // Group-128 scales: the int32 sum of one 128-k stage is exact, and is
            // folded into the fp32 accumulator as facc += float(sum) * sw[n][g]
            // (Eq. 7 with the factor 2^(s+t) restored).  That is two vector
            // operations per accumulator and stage, as many cycles as the MFMAs
            // themselves, so they are issued in the MFMAs' shadow.  A block's four
            // MFMAs (one per k-step, chained through the same registers) are
            // slots 4b .. 4b+3; quarter q of block c is scaled in slot 4c + q + 5,
            // one block and one slot later, when its last MFMA has surely
            // finished.  Three block buffers rotate so that the block two back,
            // whose last quarter is still being read, is not the one overwritten.
            // Activation operands: all of the stage's up front, or (mode 2, which has
            // no registers to spare) one row block ahead of its MFMAs.
            constexpr bool AF_AHEAD = GROUP == 2;
            static_assert(!AF_AHEAD || (MT * NT) % 2 == 0, "two operand sets alternate by block");
            v4i af[AF_AHEAD ? 2 : MT][4];
#pragma unroll
            for (int mt = 0; mt < (AF_AHEAD ? 1 : MT); ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    af[mt][j] = *reinterpret_cast<const v4i *>(
                        xs + lds_off(arow + 32 * mt, 2 * j + ahalf));
            float gsv[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) gsv[nt] = h2f(gsreg[CUR][nt]);
            const v16i vzero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            constexpr int NB = MT * NT;          // blocks per stage, b = nt * MT + mt
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                v4i bf[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) bf[j] = unpack_kstep(wreg[CUR][nt], j);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int b = nt * MT + mt;
                    const int buf = (CUR * NB + b) % 3;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        gpart[buf] = mfma_i8(af[AF_AHEAD ? (b & 1) : mt][j], bf[j],
                                             j == 0 ? vzero : gpart[buf]);
                        if constexpr (AF_AHEAD) {
                            if (b + 1 < NB)
                                af[(b + 1) & 1][j] = *reinterpret_cast<const v4i *>(
                                    xs + lds_off(arow + 32 * ((b + 1) % MT), 2 * j + ahalf));
                        }
                        // the quarter that is due: block b - 1 (quarter j - 1), or the last
                        // quarter of block b - 2; blocks before this stage's first belong to
                        // the previous stage and carry its scale
                        const int c = j == 0 ? b - 2 : b - 1;
                        const int q = j == 0 ? 3 : j - 1;
                        const int cw = (c + NB) % NB;                   // block within its stage
                        const int cmt = cw % MT, cnt = cw / MT;
                        const int cbuf = (CUR * NB + b + (c - b) + 3) % 3;
                        const float cgs = c >= 0 ? gsv[cnt] : gs_prev[cnt];
                        float t[4];
                        if constexpr (GROUP == 2) {
                            // token scales of this quarter were fetched during the slot
                            // before; fetch the next slot's now
                            const uint2 mine = xsq;
                            {
                                const int b2 = j < 3 ? b : b + 1, j2 = j < 3 ? j + 1 : 0;
                                const int c2 = j2 == 0 ? b2 - 2 : b2 - 1, q2 = j2 == 0 ? 3 : j2 - 1;
                                // past this stage's last slot: the next stage's first unit,
                                // which is this stage's block NB - 2
                                const int kb2 = b2 == NB ? kb : (c2 >= 0 ? kb : kb - 1);
                                const int cw2 = b2 == NB ? NB - 2 : (c2 + NB) % NB;
                                xsq = *xs_ptr(kb2, cw2 % MT, q2);
                            }
                            const unsigned sh[2] = {mine.x, mine.y};
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const float xs = h2f((uint16_t)(sh[r >> 1] >> (16 * (r & 1))));
                                t[r] = __builtin_fmaf((float)gpart[cbuf][4 * q + r] * cgs, xs,
                                                      facc[cmt][cnt][4 * q + r]);
                            }
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                t[r] = __builtin_fmaf((float)gpart[cbuf][4 * q + r], cgs,
                                                      facc[cmt][cnt][4 * q + r]);
                        }
                        // an empty volatile statement that "uses" the four results: code
                        // motion cannot sink the scaling out of the MFMAs' shadow
                        asm volatile("" : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]));
#pragma unroll
                        for (int r = 0; r < 4; ++r) facc[cmt][cnt][4 * q + r] = t[r];
                        // keep this order: the scheduler would otherwise gather the
                        // MFMAs and leave the vector work with nothing to hide behind
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) gs_prev[nt] = gsv[nt];
        } else {
            // One flat software pipeline over the stage's 4 * NT (k-step, column tile)
            // steps.  Activation operands are read from LDS a k-step ahead of their
            // MFMAs, and the weight operand of step s + 1 is expanded one dword per
            // MFMA of step s, i.e. in the shadow of the MFMA just issued.  The
            // scheduling barriers keep that order (left alone, the scheduler sinks the
            // LDS reads next to their first use and gathers the MFMAs).
            static_assert(MT == 2 || MT >= 4, "one dword of the next operand per MFMA, or two");
            constexpr int DPM = MT >= 4 ? 1 : 4 / MT;   // dwords of the next operand per MFMA
            v4i af[2][MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                af[0][mt] = *reinterpret_cast<const v4i *>(xs + lds_off(arow + 32 * mt, ahalf));
            v4i bfc = bf_first;
#pragma unroll
            for (int s = 0; s < 4 * NT; ++s) {
                const int j = s / NT, nt = s % NT;
                if (nt == 0 && j < 3) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        af[(j + 1) & 1][mt] = *reinterpret_cast<const v4i *>(
                            xs + lds_off(arow + 32 * mt, 2 * (j + 1) + ahalf));
                    __builtin_amdgcn_sched_barrier(0);
                }
                v4i bfn = bfc;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    acc[mt][nt] = mfma_i8(af[j & 1][mt], bfc, acc[mt][nt]);
                    if (mt * DPM < 4 && s + 1 < 4 * NT) {
#pragma unroll
                        for (int d = mt * DPM; d < (mt + 1) * DPM; ++d)
                            bfn[d] = unpack_kstep_dword(wreg[CUR][(s + 1) % NT], (s + 1) / NT, d);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                bfc = bfn;
            }
        }
        // stage kb + 1 must have landed in LDS (every wavefront's share) before
        // anyone reads it; the loads of stage kb + 2 may stay in flight
        if (more2)
            wait_vmcnt<XDMA + WLOADS + (GROUP ? NT : 0) + (GROUP == 2 ? 1 : 0)>();
        else
            wait_vmcnt<0>();
        if constexpr (!GROUP) bf_first = unpack_kstep(wreg[(CUR + 1) % 3][0], 0);   // has landed
        lds_barrier();
    };

    int kb = 0;
    for (; kb + 2 < KN; kb += 3) {
        stage(kb, std::integral_constant<int, 0>{});
        stage(kb + 1, std::integral_constant<int, 1>{});
        stage(kb + 2, std::integral_constant<int, 2>{});
    }
    if (kb < KN) stage(kb, std::integral_constant<int, 0>{});
    if (kb + 1 < KN) stage(kb + 1, std::integral_constant<int, 1>{});
    if constexpr (GROUP) {
        // still unscaled: the last block of the last stage, and the last quarter of
        // the block before it
        constexpr int NB = MT * NT;
        const int last = (KN * NB - 1) % 3, before = (KN * NB - 2) % 3;
        auto fold = [&](int buf, int c, int r0) {
            const int cmt = c % MT, cnt = c / MT;
#pragma unroll
            for (int i = 0; i < 3; ++i)
                if (i == buf) {
#pragma unroll
                    for (int r = r0; r < 16; ++r) {
                        if constexpr (GROUP == 2) {
                            const uint2 four = *xs_ptr(KN - 1, cmt, r >> 2);
                            const unsigned half = (r & 2) ? four.y : four.x;
                            const float xs = h2f((uint16_t)(half >> (16 * (r & 1))));
                            facc[cmt][cnt][r] = __builtin_fmaf((float)gpart[i][r] * gs_prev[cnt], xs,
                                                               facc[cmt][cnt][r]);
                        } else {
                            facc[cmt][cnt][r] = __builtin_fmaf((float)gpart[i][r], gs_prev[cnt],
                                                               facc[cmt][cnt][r]);
                        }
                    }
                }
        };
        fold(before, NB - 2, 12);
        fold(last, NB - 1, 0);
    }

    // ---- epilogue -----------------------------------------------------------
    // The accumulators leave through LDS so that global stores are whole lines:
    // each wavefront transposes one 32-row slab of its tile at a time in its own
    // LDS region (row stride NT*32 + 8 dwords: the two half-waves of a write and
    // the sixteen lanes of a 16-byte read each cover all banks once), then every
    // lane owns four consecutive columns of one row, applies sx[m] * sw[n] in
    // fp32, and the lanes of a row store whole 64- or 128-byte runs of fp16.
    constexpr int ESTRIDE = (NT * 32 + 8) * 4;          // bytes per staged row
    static_assert(3 * XSTAGE >= WAVES * 32 * ESTRIDE, "epilogue staging must fit the stage buffers");
    constexpr int LPR = NT * 8;                          // lanes per staged row (4 columns each)
    constexpr int RPI = 64 / LPR;                        // rows per read instruction
    static_assert(64 % LPR == 0, "a read instruction covers whole rows");
    uint8_t *stg = lds + wave * (32 * ESTRIDE);
    const int ecol = (lane % LPR) * 4;                  // first of this lane's 4 columns
    const int erow = lane / LPR;
    const int n_wave = bn0 + wn * NT * 32;
    const int n_lane = n_wave + ecol;
    const bool cvalid = n_lane < N;
    float swv[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) swv[c] = GROUP ? 0.25f : h2f(a.scales[cvalid ? n_lane + c : 0]);
    // scale and store four columns of row m (q: exact int32 sums, or fp32 group sums)
    auto finish = [&](const v4i &q, int m, float sxm) {
        uint16_t h[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            h[c] = GROUP ? f2h(__int_as_float(q[c]) * swv[c] * sxm) : f2h((float)q[c] * (sxm * swv[c]));
        uint2 out2;
        out2.x = (unsigned)h[0] | ((unsigned)h[1] << 16);
        out2.y = (unsigned)h[2] | ((unsigned)h[3] << 16);
        *reinterpret_cast<uint2 *>(a.y + (long)m * N + n_lane) = out2;
        if (!GROUP && a.acc_out) *reinterpret_cast<v4i *>(a.acc_out + (long)m * N + n_lane) = q;
    };
    // split-K partial sums [split][M][N] int32, addressed as a buffer; cache policy
    // bit 4 = sc1 = device scope: the access goes to memory all XCDs share
    constexpr int kScopeAgent = 16;
    const __amdgpu_buffer_rsrc_t prsrc = __builtin_amdgcn_make_buffer_rsrc(
        a.partial, 0, (unsigned)((long)KS * M * N * 4), 0x00020000);
    // every token scale this wavefront will need, fetched in one go ahead of the stores: a
    // load per row, or per slab, inside the loop would wait a memory round trip each time
    // (the compiler cannot move it above the stores, which might alias)
    float sxall[MT][32 / RPI];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int m = bm0 + (wm * MT + mt) * 32 + i * RPI + erow;
            // (mode 2 is scaled per group already; K splits scale after they have met)
            sxall[mt][i] = (GROUP != 2 && KS == 1 && m < M) ? h2f(a.sx[m]) : 1.0f;
        }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m_slab = bm0 + (wm * MT + mt) * 32;
        if (m_slab >= M) break;                          // uniform: nothing below is stored
        const float *sxv = sxall[mt];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int v = GROUP ? __float_as_int(facc[GROUP ? mt : 0][GROUP ? nt : 0][r])
                                    : (acc[mt][nt][r] >> 2);
                *reinterpret_cast<int *>(stg + mfma_row(r, lane) * ESTRIDE +
                                         (nt * 32 + (lane & 31)) * 4) = v;
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // own region only: no barrier
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int row = i * RPI + erow;
            const v4i q = *reinterpret_cast<const v4i *>(stg + row * ESTRIDE + ecol * 4);
            const int m = m_slab + row;
            if (m < M && cvalid) {
                if (KS == 1) {
                    finish(q, m, sxv[i]);
                } else {
                    // device-scope (sc1) 16-byte store: see the hand-off below
                    const unsigned off = (unsigned)((((long)ksplit * M + m) * N + n_lane) * 4);
                    __builtin_amdgcn_raw_buffer_store_b128((v4u)q, prsrc, off, 0, kScopeAgent);
                }
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the next slab overwrites
    }
    if (KS == 1) return;

    // ---- K splits meet: the last block of this tile to arrive adds the partial
    // sums in split order and stores the tile.  Partial sums were written with
    // device-scope stores; once they are acknowledged (vmcnt 0) the barrier plus
    // one relaxed device-scope counter increment publishes them, and the reader
    // uses device-scope loads -- no L2 write-back / invalidate is needed.
    __shared__ int s_last;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
    if (tid == 0) {
        const unsigned prev = __hip_atomic_fetch_add(&a.counters[tile_id], 1u, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == (unsigned)(KS - 1));
        if (s_last) __hip_atomic_store(&a.counters[tile_id], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    lds_barrier();
    if (!s_last) return;
    // A row of the tile per step: its four columns of every split are loaded, added in
    // split order and stored.  The loads of the NEXT row (its first four splits and its
    // token scale) are issued before this row is finished -- in program order the
    // compiler may not lift a load above the stores of `finish`, and each row would then
    // cost a full memory round trip of its own.
    constexpr int ROWS_PER_SLAB = 32 / RPI, NROW = MT * ROWS_PER_SLAB;
    auto row_of = [&](int it) {
        return bm0 + (wm * MT + it / ROWS_PER_SLAB) * 32 + (it % ROWS_PER_SLAB) * RPI + erow;
    };
    auto issue4 = [&](int m, int k0, v4i (&v)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = k0 + u < KS ? k0 + u : KS - 1;
            const unsigned off = (unsigned)((((long)k * M + m) * N + n_lane) * 4);
            v[u] = (v4i)__builtin_amdgcn_raw_buffer_load_b128(prsrc, off, 0, kScopeAgent);
        }
    };
    v4i ahead[4];
    uint16_t sx_ahead = 0;
    if (row_of(0) < M && cvalid) {
        issue4(row_of(0), 0, ahead);
        if (GROUP != 2) sx_ahead = a.sx[row_of(0)];
    }
#pragma unroll
    for (int it = 0; it < NROW; ++it) {
        const int m = row_of(it);
        const bool valid = m < M && cvalid;
        v4i v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = ahead[u];
        const float sxm = GROUP == 2 ? 1.0f : h2f(sx_ahead);
        if (it + 1 < NROW) {
            const int m2 = row_of(it + 1);
            if (m2 < M && cvalid) {
                issue4(m2, 0, ahead);
                if (GROUP != 2) sx_ahead = a.sx[m2];
            }
        }
        if (valid) {
            v4i q = {0, 0, 0, 0};
            float f[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            for (int k0 = 0; k0 < KS; k0 += 4) {       // four independent loads in flight
                if (k0) issue4(m, k0, v);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (k0 + u < KS) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            if (GROUP)
                                f[c] += __int_as_float(v[u][c]);
                            else
                                q[c] += v[u][c];
                        }
                    }
                }
            }
            if (GROUP) {
#pragma unroll
                for (int c = 0; c < 4; ++c) q[c] = __float_as_int(f[c]);
            }
            finish(q, m, sxm);
        }
    }
#endif
}

template <int WM, int WN, int MT, int NT, int GROUP, int WPE>
hipError_t launch_cfg(const flexq::LinearArgs &a, hipStream_t st)
{
    constexpr int BM = WM * MT * 32, BN = WN * NT * 32;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const size_t lds_bytes = 3 * BM * 128 + (GROUP == 2 ? 4 * BM * 2 : 0);
    auto kern = gemm_kernel<WM, WN, MT, NT, GROUP, WPE>;
    static std::atomic<unsigned long long> lds_allowed{0};
    if (hipError_t e = flexq::allow_dynamic_lds(reinterpret_cast<const void *>(kern), (int)lds_bytes, lds_allowed);
        e != hipSuccess)
        return e;
    if (a.split_k > 1 && tiles_m * tiles_n > 4096) return hipErrorInvalidValue;  // one counter per tile
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n * a.split_k)), dim3(64 * WM * WN),
                       lds_bytes, st, a, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

namespace flexq {

hipError_t launch_gemm(const LinearArgs &a, int cfg, hipStream_t st, int *chosen, int *tail_runs)
{
    int unused_cfg, unused_runs;
    if (!chosen) chosen = &unused_cfg;
    if (!tail_runs) tail_runs = &unused_runs;
    *tail_runs = 0;
    *chosen = 8;   // the group modes run 128x128 tiles
    // Group-128 scales cost two vector operations per accumulator and group (int -> float,
    // multiply-add), as many cycles as the MFMAs: that mode is bound by the vector unit.
    // 128x128 tiles with two workgroups per CU keep the int32 sums out of the AGPR half
    // of the register file (which vector instructions cannot read directly).
    if (a.group != 0) {
        if (a.sxg) return launch_cfg<1, 4, 4, 1, 2, 2>(a, st);          // scales per group on both operands
#ifdef FLEXQ_DEV
        if (cfg == 21) {
            *chosen = 21;
            return launch_cfg<1, 4, 4, 2, 1, 1>(a, st);      // 128x256, 1 wave/SIMD
        }
#endif
        return launch_cfg<1, 4, 4, 1, 1, 2>(a, st);
    }
    if (cfg == 0) {
        // The candidates beyond 128 tokens: 128x256 tiles (two workgroups per CU), 128x128 (three per CU;
        // the only shape with K splits), 256x256 with both operands through LDS (one per
        // CU, the fewest bytes per MFMA through the vector-memory path), and the
        // persistent form of the latter that cuts the tiles beyond the last whole round
        // of 256 along K.  Which is fastest depends mostly on how evenly the work fills
        // the 256 CUs, so the time of the busiest CU is estimated for each: its
        // ceil(tiles / 256) tiles run `slots` at a time at the measured relative
        // throughput of that many co-resident workgroups, a remainder at the throughput
        // of fewer.  Fitted on the LLaMA-2-70B layers at 256..4096 tokens.
        auto busiest_cu = [](long tiles, double area, int slots, const double *throughput) {
            const long per_cu = (tiles + 255) / 256;
            const long full = per_cu / slots, rest = per_cu % slots;
            double t = (double)full * slots * area / throughput[slots - 1];
            if (rest) t += (double)rest * area / throughput[rest - 1];
            return t;
        };
        static const double thr7[2] = {0.70, 1.00}, thr8_busy[3] = {0.40, 0.75, 0.85};
        // with at most one 128x128 workgroup per CU on the whole chip the clock is higher
        static const double thr8_sparse[3] = {0.58, 0.75, 0.85};
        const long m128 = (a.M + 127) / 128, n128 = (a.N + 127) / 128, n256 = (a.N + 255) / 256;
        // microseconds per unit of tile area: a whole 256x256 tile (relative throughput
        // 1.03) takes 1.556 us per 128-k stage plus 7 us
        const double unit = (1.556 * (a.K / 128) + 7.0) * 1.03 / 65536.0;
        double t_best;
        // Up to 128 tokens on a layer so wide that 128 x 256 tiles alone fill most of the chip
        // in one round (LLaMA-2-70B's 57344-wide gate+up: 224 tiles): the 128-row form of the
        // kernel with both operands through LDS, one tile per workgroup, no K split --
        // measured 66 / 68 / 73 / 80 us at 33 / 64 / 96 / 128 tokens against 68 / 72 / 85 / 94
        // for the tiles below.
        if (a.M > 32 && a.M <= 128 && n256 >= 160 && n256 <= kStreamKGrid &&
            (long)a.N * a.K / 4 * 3 < (1L << 32)) {
            LinearArgs b = a;
            b.split_k = 1;
            *chosen = 15;
            return launch_gemm_wlds(b, 3, 0, st);
        }
        if (const int pieces = low_cut_pieces(a.M, a.N, a.K); pieces != 0) {
            // 65 to 128 tokens on a narrower layer: the same tiles, each cut along K
            const int tail_wgs = (int)n256 * pieces;
            if (a.partial_bytes >= low_cut_bytes(tail_wgs) && device_cu_count() == kStreamKGrid &&
                (long)a.N * a.K / 4 * 3 < (1L << 32)) {
                LinearArgs b = a;
                b.split_k = 1;
                *chosen = 16;
                *tail_runs = tail_wgs;
                return launch_gemm_wlds(b, 5, tail_wgs, st);
            }
        }
        if (a.M <= 64) {
            // every token fits a 64-row tile: half the MFMAs and half the activation bytes
            // of the 128x128 tile, same columns and K splits (5-10 % faster, measured)
            *chosen = 5;
            return launch_cfg<1, 4, 2, 1, 0, 4>(a, st);
        }
        if (a.split_k > 1) {   // K splits were chosen for 128x128 tiles; meeting costs about 16 us
            cfg = 8;
            const double *thr8 = m128 * n128 * a.split_k <= 256 ? thr8_sparse : thr8_busy;
            t_best = busiest_cu(m128 * n128 * a.split_k, 128.0 * 128 / a.split_k, 3, thr8) * unit + 16.0;
        } else {
            const double t7 = busiest_cu(m128 * n256, 128.0 * 256, 2, thr7) * unit;
            const double *thr8 = m128 * n128 <= 256 ? thr8_sparse : thr8_busy;
            const double t8 = busiest_cu(m128 * n128, 128.0 * 128, 3, thr8) * unit;
            cfg = t8 < t7 ? 8 : 7;
            t_best = t8 < t7 ? t8 : t7;
        }
        if (a.M > 128) {
            const bool may_cut = a.partial_bytes >= streamk_plan(a.M, a.N, a.K).partial_bytes &&
                                 device_cu_count() == kStreamKGrid;
            WldsChoice c = gemm_wlds_choose(a.M, a.N, a.K, may_cut);
            // a cut tail must promise 5 % (it adds workspace traffic the estimate is unsure
            // of); else the best form that leaves the workspace alone
            if (c.tail_form == 2 && c.us >= 0.95 * t_best) c = gemm_wlds_choose(a.M, a.N, a.K, false);
            if (c.us < t_best) {
                LinearArgs b = a;
                b.split_k = 1;
                *chosen = 12 + (c.tail_form == 2 ? 1 : c.tail_form == 1 ? 2 : 0);
                *tail_runs = c.tail_wgs;
                return launch_gemm_wlds(b, c.tail_form, c.tail_wgs, st);
            }
        }
    }
    *chosen = cfg;
    if (cfg == 12 && a.split_k == 1) return launch_gemm_wlds(a, 0, 0, st);
    if (cfg == 13) {
        // forced: cut the tail also where another form is estimated to be faster; a forced
        // number of K splits is the number of pieces per tile
        const WldsChoice c = gemm_wlds_choose(a.M, a.N, a.K, true);
        int tail_wgs = c.tail_form == 2 ? c.tail_wgs : kStreamKGrid;
        if (a.split_k > 1) {
            tail_wgs = streamk_plan(a.M, a.N, a.K).tail_tiles * a.split_k;
            if (tail_wgs > kStreamKGrid || a.split_k > a.K / FLEXQ_TILE_K) return hipErrorInvalidValue;
        }
        LinearArgs b = a;
        b.split_k = 1;
        *tail_runs = tail_wgs;
        return launch_gemm_wlds(b, 2, tail_wgs, st);
    }
    if (cfg == 17 && a.split_k == 1) {
        // the tail cut into 256 equal runs that begin and end inside tiles (never a whole
        // number of runs per tile: that would be the even cut)
        const StreamKPlan p = streamk_plan(a.M, a.N, a.K);
        const long stages = (long)p.tail_tiles * (a.K / FLEXQ_TILE_K);
        int tail_wgs = stages < kStreamKGrid ? (int)stages : kStreamKGrid;
        if (p.tail_tiles > 1 && tail_wgs % p.tail_tiles == 0 && tail_wgs > p.tail_tiles) tail_wgs -= 1;
        *tail_runs = tail_wgs;
        return launch_gemm_wlds(a, 2, tail_wgs, st);
    }
    if (cfg == 15 && a.split_k == 1) return launch_gemm_wlds(a, 3, 0, st);
    if (cfg == 16) {   // 128x256 tiles, each cut into split_k pieces
        const int tail_wgs = (int)(((a.M + 127) / 128) * ((a.N + 255) / 256)) * a.split_k;
        LinearArgs b = a;
        b.split_k = 1;
        *tail_runs = tail_wgs;
        return launch_gemm_wlds(b, 5, tail_wgs, st);
    }
    if (cfg == 14 && a.split_k == 1) {
        *tail_runs = 2 * streamk_plan(a.M, a.N, a.K).tail_tiles;
        return launch_gemm_wlds(a, 1, 0, st);
    }
    switch (cfg) {
#ifdef FLEXQ_DEV   // shapes the dispatch never picks: kept selectable for comparisons
    case 1: return launch_cfg<2, 2, 4, 4, 0, 1>(a, st);   // 256x256, 4 waves, 1 wave/SIMD
    case 2: return launch_cfg<2, 4, 4, 2, 0, 2>(a, st);   // 256x256, 8 waves (128x64 each)
    case 6: return launch_cfg<1, 4, 8, 2, 0, 1>(a, st);   // 256x256, 4 waves side by side (256x64 each)
#endif
    case 7: return launch_cfg<1, 4, 4, 2, 0, 2>(a, st);   // 128x256, 4 waves side by side, 2 workgroups/CU
    case 8: return launch_cfg<1, 4, 4, 1, 0, 3>(a, st);   // 128x128, 4 waves side by side, 3 workgroups/CU
    case 5: return launch_cfg<1, 4, 2, 1, 0, 4>(a, st);   // 64x128, 4 waves side by side, 4 workgroups/CU
    default: *chosen = 7; return launch_cfg<1, 4, 4, 2, 0, 2>(a, st);
    }
}

}  // namespace flexq
