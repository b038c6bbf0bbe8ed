// Tiled i8-MFMA GEMM, 256x256 tile, BOTH operands through LDS.
//
// The 128x256 kernel is limited by power, and what costs power besides the
// MFMAs is every byte a wavefront brings in through the vector-memory path:
// timing probes put the packed-weight loads at about a fifth of its run time
// and the activation DMA at a tenth, while doubling the LDS operand reads
// costs 3 %.  This kernel therefore trades vector-memory bytes for LDS reads:
// one workgroup of eight wavefronts (2 along m x 4 along n, 128x64 each) owns a
// 256x256 tile, and a packed weight tile is brought into LDS ONCE per
// workgroup (by DMA, like the activations) and read from there by the two
// wavefronts that share its columns: 0.875 KB through the vector-memory path
// per 32x32x128 block instead of 1.25.
//
//   LDS: three activation stages of 32 KiB (two stages ahead) and two weight
//   stages of 24 KiB (one stage ahead: a weight stage is consumed -- copied to
//   registers -- right at the start of its stage, so its buffer is free for the
//   stage after next as soon as every wavefront has passed the next barrier);
//   144 KiB, one workgroup per CU, two wavefronts per SIMD.
//   Per stage and wavefront: 3 weight DMA loads, then 4 activation DMA loads;
//   the hand-over waits until at most the 4 youngest are outstanding.
//
// Per-channel scales only: this is the kernel for large M and N.  Inner loop and
// epilogue follow the 128x256 kernel.
//
// Two launch forms.  One workgroup per tile, when the tiles come in whole rounds
// of the 256 CUs.  Otherwise a persistent form (SK) of 256 workgroups: each takes
// its share of the whole rounds tile by tile, and the tiles of the last, partial
// round are cut along K into equal contiguous runs of 128-k stages, one run per
// workgroup, so that every CU is busy to the end.  A run that is not a whole tile
// leaves its int32 sums in the workspace (exact, so the order of addition does
// not matter); the workgroups of a tile add their stage counts to the tile's
// counter, and the one that completes the count adds the others' sums to its own
// registers and runs the epilogue.  Nobody waits for anybody.
#include "flexq_device.h"
#include "flexq_kernels.h"
#include "gemm_common.h"
#include <type_traits>

namespace {

constexpr int BM = 256, BN = 256, WAVES = 8, MT = 4, NT = 2;
constexpr int XSTAGE = BM * 128;               // bytes of one activation stage
constexpr int WSTAGE = (BN / 32) * FLEXQ_TILE_BYTES;
constexpr int WBASE = 3 * XSTAGE;
constexpr int LDS_BYTES = WBASE + 2 * WSTAGE;
constexpr int XDMA = BM / 8 / WAVES;           // 1 KiB activation DMA loads per wavefront and stage
constexpr int WDMA = 3;                        // each wavefront fetches one weight tile (3 planes)
static_assert(BN / 32 == WAVES, "one weight tile per wavefront");

constexpr int SLOT_BYTES = BM * BN * 4;         // one workgroup's int32 sums of a tile

template <bool SK>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gemm_wlds_kernel(flexq::LinearArgs a, int tiles_m, int tiles_n, int full_tiles, int tail_tiles,
                      int tail_wgs)
{
#if defined(__HIP_DEVICE_COMPILE__)  // buffer-resource builtins exist in the device pass only
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int M = a.M, N = a.N, K = a.K;
    const int KT = K / FLEXQ_TILE_K;
    const int nblk = tiles_m * tiles_n;

    // SK: workgroups 8 apart share an XCD; v numbers them XCD by XCD, so that the
    // workgroups of one XCD work on neighbouring tiles (and neighbouring runs of the tail)
    const int G = (int)gridDim.x;
    const int v = SK ? (int)(blockIdx.x % 8) * (G / 8) + (int)(blockIdx.x / 8) : 0;
    const int rounds = SK ? full_tiles / G : 0;
    const long U = (long)tail_tiles * KT;           // 128-k stages of the tail
    // the tail's runs are numbered so that every XCD takes a contiguous share of them,
    // also when there are fewer runs than workgroups
    int vt = -1;
    if (SK) {
        const int x = (int)(blockIdx.x % 8), slot = (int)(blockIdx.x / 8);
        const int per = tail_wgs / 8, rem = tail_wgs % 8;
        if (slot < per + (x < rem ? 1 : 0)) vt = x * per + min(x, rem) + slot;
    }
    long u0 = 0, u1 = 0;                            // this workgroup's run of stages
    if (vt >= 0) {
        u0 = (long)vt * U / tail_wgs;
        u1 = (long)(vt + 1) * U / tail_wgs;
    }
    const long run_begin = u0;

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)a.xq, 0, (unsigned)((long)M * K), 0x00020000);
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)a.packed, 0, (unsigned)((long)N * K / 4 * 3), 0x00020000);

    for (int it = 0;; ++it) {
        // ---- which tile, which stages [ks, ke) of it ---------------------------
        int bid, ks = 0, ke = KT, tj = 0;
        if (!SK) {
            if (it) break;
            // XCD-aware tile choice: blocks 8 apart share an XCD
            bid = blockIdx.x;
            const int per = nblk / 8, rem = nblk % 8;
            const int xcd = bid % 8, slot = bid / 8;
            bid = xcd * per + (xcd < rem ? xcd : rem) + slot;
        } else if (it < rounds) {
            bid = (v / (G / 8)) * (full_tiles / 8) + it * (G / 8) + v % (G / 8);
        } else {
            if (u0 >= u1) break;
            tj = (int)(u0 / KT);
            ks = (int)(u0 - (long)tj * KT);
            ke = (int)min((long)KT, ks + (u1 - u0));
            bid = full_tiles + tj;
            u0 += ke - ks;
        }
        const int KN = ke - ks;
        // The 32 tiles an XCD works on at a time share operand panels in its L2: a block of
        // 4 tiles along m x 8 along n fetches the fewest bytes (4 activation panels of 2 MB
        // per 8192 of K + 8 weight panels of 1.5 MB).
        constexpr int SUP_M = 4;  // super-block: 4 tiles along m, then next n
        const int sup = bid / (SUP_M * tiles_n);
        const int first_m = sup * SUP_M;
        const int span_m = min(SUP_M, tiles_m - first_m);
        const int in_sup = bid - sup * SUP_M * tiles_n;
        const int tile_m = first_m + in_sup % span_m;
        const int tile_n = in_sup / span_m;
        const int bm0 = tile_m * BM, bn0 = tile_n * BN;

        // ---- activations: global -> LDS by DMA; rows beyond M read as zero -----
        // (stage numbers below count from ks)
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
                    (ks + kb) * FLEXQ_TILE_K, 0, 0);
            }
        };

        // ---- packed weights: wavefront w brings tile w of the workgroup's eight
        // column tiles into LDS, plane by plane, exactly as it lies in memory ------
        // the SGPR offset is not range-checked: tiles past the last row block
        // re-read the last one and are never stored
        const int wtile = min(bn0 / 32 + wave, N / 32 - 1);
        const unsigned wlane = (unsigned)lane * 16u;
        auto dma_w = [&](int kb, int buf) {
#pragma unroll
            for (int p = 0; p < WDMA; ++p) {
                uint8_t *dst = lds + WBASE + buf * WSTAGE + wave * FLEXQ_TILE_BYTES + p * 1024;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    wrsrc, (void __attribute__((address_space(3))) *)dst, 16, wlane,
                    (unsigned)(wtile * KT + ks + kb) * FLEXQ_TILE_BYTES + 1024u * p, 0, 0);
            }
        };

        v16i acc[MT][NT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0;

        // prologue: weights and activations of stage 0, activations of stage 1
        dma_w(0, 0);
        dma_x(0, 0);
        if (KN > 1) dma_x(1, 1);
        wait_vmcnt<0>();
        lds_barrier();

        const int arow = (wm * MT) * 32 + (lane & 31);
        const int ahalf = lane >> 5;
        const int wfrag = WBASE + (wn * NT) * FLEXQ_TILE_BYTES + lane * 16;   // this lane's piece of tile nt = 0

        // operands that live across stages: the stage's packed tiles, the activation
        // operands of two consecutive k-steps, the first weight operand of a stage
        PackedTile wreg[NT];
        v4i af[2][MT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const v4i *t = reinterpret_cast<const v4i *>(lds + wfrag + nt * FLEXQ_TILE_BYTES);
            wreg[nt].q0 = t[0];
            wreg[nt].q1 = t[64];
            wreg[nt].q2 = t[128];
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            af[0][mt] = *reinterpret_cast<const v4i *>(lds + lds_off(arow + 32 * mt, ahalf));
        v4i bf_first = unpack_kstep(wreg[0], 0);

        // One 128-k stage.  CUR = kb % 3 names the activation buffer; kb & 1 the weight buffer.
        auto stage = [&](int kb, auto cur_tag) {
            constexpr int CUR = decltype(cur_tag)::value;
            constexpr int NXT2 = (CUR + 2) % 3;
            const bool more1 = kb + 1 < KN, more2 = kb + 2 < KN;
            // weights first: the hand-over waits for them and for everything older,
            // while the activation loads issued after them may stay in flight
            if (more1) dma_w(kb + 1, (kb + 1) & 1);
            if (more2) dma_x(kb + 2, NXT2);

            const uint8_t *xs = lds + CUR * XSTAGE;
            const uint8_t *xn = lds + ((CUR + 1) % 3) * XSTAGE;
            const uint8_t *wnb = lds + wfrag + ((kb + 1) & 1) * WSTAGE;
            // Flat software pipeline over the 4 * NT (k-step, column tile) steps: LDS
            // operand reads a k-step ahead, weight operands expanded one dword per MFMA in
            // the shadow of the MFMA just issued.  The two wavefronts of a SIMD belong to
            // the same workgroup and reach the stage boundary together, so nothing would
            // cover the operand fetch of a new stage: the hand-over therefore sits BEFORE
            // the last k-step.  By then this wavefront has read all it needs of stage kb
            // (the operands of k-step 3 are in registers: activations were read during
            // k-step 2, the weight operands expanded during steps 3 and 4), so after the
            // barrier the packed tiles and first activation operands of stage kb + 1 are
            // fetched from LDS while k-step 3's MFMAs run.
            static_assert(NT == 2 && MT == 4, "the step table below is written for 4 x 2 blocks");
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
                    } else {
                        // stage kb + 1 (weights and activations, every wavefront's share) must
                        // have landed; the activations of stage kb + 2 may be in flight
                        if (more2)
                            wait_vmcnt<XDMA>();
                        else
                            wait_vmcnt<0>();
                        lds_barrier();
                        if (more1) {
#pragma unroll
                            for (int n2 = 0; n2 < NT; ++n2) {
                                const v4i *t = reinterpret_cast<const v4i *>(wnb + n2 * FLEXQ_TILE_BYTES);
                                wreg[n2].q0 = t[0];
                                wreg[n2].q1 = t[64];
                                wreg[n2].q2 = t[128];
                            }
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
                                af[0][mt] = *reinterpret_cast<const v4i *>(xn + lds_off(arow + 32 * mt, ahalf));
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                const v4i cur = s == 6 ? bf6 : s == 7 ? bf7 : bfc;
                v4i nxt = bfc;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    acc[mt][nt] = mfma_i8(af[j & 1][mt], cur, acc[mt][nt]);
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
        };

        int kb = 0;
        for (; kb + 2 < KN; kb += 3) {
            stage(kb, std::integral_constant<int, 0>{});
            stage(kb + 1, std::integral_constant<int, 1>{});
            stage(kb + 2, std::integral_constant<int, 2>{});
        }
        if (kb < KN) stage(kb, std::integral_constant<int, 0>{});
        if (kb + 1 < KN) stage(kb + 1, std::integral_constant<int, 1>{});

        // ---- a run that is not a whole tile: leave the sums, or collect the others' ----
        if (SK && KN != KT) {
            // [slot][wavefront][block mt, nt][quarter][lane] 16-byte pieces: every store and
            // load below is one contiguous KiB per wavefront.  Cache policy bit 4 = sc1 =
            // device scope: the access goes to memory all XCDs share.
            constexpr int kScopeAgent = 16;
            const __amdgpu_buffer_rsrc_t prsrc = __builtin_amdgcn_make_buffer_rsrc(
                a.partial, 0, (unsigned)(2 * tail_wgs) * (unsigned)SLOT_BYTES, 0x00020000);
            const unsigned in_slot = (unsigned)(wave * (SLOT_BYTES / WAVES) + lane * 16);
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
                if (!__builtin_amdgcn_readfirstlane(s_last)) continue;   // scalar branch: barriers follow
            }
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

        // ---- epilogue: as in the 128x256 kernel -----------------------------------
        // After the last barrier nobody reads the stage buffers again, so each
        // wavefront transposes its 32-row slabs through a region of its own (row
        // stride NT*32 + 8 dwords), then every lane owns four consecutive columns of
        // one row, applies sx[m] * sw[n] in fp32, and the lanes of a row store whole
        // 128-byte runs of fp16.
        constexpr int ESTRIDE = (NT * 32 + 8) * 4;
        static_assert(3 * XSTAGE >= WAVES * 32 * ESTRIDE, "epilogue staging must fit the stage buffers");
        constexpr int LPR = NT * 8;
        constexpr int RPI = 64 / LPR;
        uint8_t *stg = lds + wave * (32 * ESTRIDE);
        const int ecol = (lane % LPR) * 4;
        const int erow = lane / LPR;
        const int n_lane = bn0 + wn * NT * 32 + ecol;
        const bool cvalid = n_lane < N;
        float swv[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) swv[c] = h2f(a.scales[cvalid ? n_lane + c : 0]);
        // Whole slabs (every row below M, every column below N, no int32 copy wanted) take a
        // path without per-row branches or 64-bit address arithmetic: the output is addressed
        // as a buffer from this wavefront's corner, a lane's offset is fixed, the row offset is
        // an SGPR; and the accumulators are staged as they are (4x the sum), the factor 1/4
        // folded into the weight scale (a power of two: the rounded result is identical).
        const bool cols_whole = bn0 + (wn + 1) * NT * 32 <= N;
        const long corner = (long)(bm0 + wm * MT * 32) * N + bn0 + wn * NT * 32;
        const __amdgpu_buffer_rsrc_t yrsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(a.y + corner), 0, (unsigned)(((long)(MT * 32 - 1) * N + NT * 32) * 2), 0x00020000);
        const unsigned yoff = (unsigned)((erow * N + ecol) * 2);
        float swq[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) swq[c] = 0.25f * swv[c];
        // every token scale this wavefront will need, fetched in one go: a load per row
        // inside the store loop would wait a memory round trip each time (the compiler cannot
        // move it above the stores, which might alias), a batch per slab once per slab
        float sxall[MT][32 / RPI];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 32 / RPI; ++i) {
                const int m = bm0 + (wm * MT + mt) * 32 + i * RPI + erow;
                sxall[mt][i] = m < M ? h2f(a.sx[m]) : 0.0f;
            }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m_slab = bm0 + (wm * MT + mt) * 32;
            if (m_slab >= M) break;                          // uniform: nothing below is stored
            const bool whole = cols_whole && m_slab + 32 <= M && !a.acc_out;   // uniform
            const float *sxv = sxall[mt];
            if (whole) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        *reinterpret_cast<int *>(stg + mfma_row(r, lane) * ESTRIDE +
                                                 (nt * 32 + (lane & 31)) * 4) = acc[mt][nt][r];
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // own region only: no barrier
#pragma unroll
                for (int i = 0; i < 32 / RPI; ++i) {
                    const v4i q = *reinterpret_cast<const v4i *>(stg + (i * RPI + erow) * ESTRIDE + ecol * 4);
                    uint16_t h[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) h[c] = f2h((float)q[c] * (sxv[i] * swq[c]));
                    typedef unsigned v2u __attribute__((ext_vector_type(2)));
                    v2u out2;
                    out2.x = (unsigned)h[0] | ((unsigned)h[1] << 16);
                    out2.y = (unsigned)h[2] | ((unsigned)h[3] << 16);
                    __builtin_amdgcn_raw_buffer_store_b64(out2, yrsrc, yoff,
                                                          (unsigned)((mt * 32 + i * RPI) * N * 2), 0);
                }
            } else {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        *reinterpret_cast<int *>(stg + mfma_row(r, lane) * ESTRIDE +
                                                 (nt * 32 + (lane & 31)) * 4) = acc[mt][nt][r] >> 2;
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
                for (int i = 0; i < 32 / RPI; ++i) {
                    const int row = i * RPI + erow;
                    const v4i q = *reinterpret_cast<const v4i *>(stg + row * ESTRIDE + ecol * 4);
                    const int m = m_slab + row;
                    if (m < M && cvalid) {
                        const float sxm = sxv[i];
                        uint16_t h[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) h[c] = f2h((float)q[c] * (sxm * swv[c]));
                        uint2 out2;
                        out2.x = (unsigned)h[0] | ((unsigned)h[1] << 16);
                        out2.y = (unsigned)h[2] | ((unsigned)h[3] << 16);
                        *reinterpret_cast<uint2 *>(a.y + (long)m * N + n_lane) = out2;
                        if (a.acc_out) *reinterpret_cast<v4i *>(a.acc_out + (long)m * N + n_lane) = q;
                    }
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the next slab overwrites
        }
        if (!SK) break;
        lds_barrier();   // every wavefront is done with its staging region before the next run's DMA
    }
#endif
}

}  // namespace

namespace flexq {

StreamKPlan streamk_plan(int M, int N, int K)
{
    StreamKPlan p;
    p.tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    p.full_tiles = p.tiles / kStreamKGrid * kStreamKGrid;
    p.tail_tiles = p.tiles - p.full_tiles;
    // two slots per run; a run is at least one 128-k stage, and there are at most 256 runs
    const long stages = (long)p.tail_tiles * (K / FLEXQ_TILE_K);
    p.partial_bytes = (size_t)2 * (size_t)(stages < kStreamKGrid ? stages : kStreamKGrid) * SLOT_BYTES;
    return p;
}

// Estimated run time in microseconds, measured constants of the MI355X: a 128-k
// stage of a 256x256 tile takes 1.56 us at the clock this load sustains, prologue plus
// epilogue 7 us per tile.  Meeting in the workspace costs 14 us plus 2 us per
// workgroup of a tile when every tile is cut into the same number S of runs (one
// partial tile per workgroup: 256 KiB written, the last to arrive reads the others');
// about 45 us when the tail is simply cut into 256 equal runs, which then begin and
// end inside tiles (two partial tiles per workgroup).
double gemm_wlds_estimate_us(int M, int N, int K, bool may_cut, int *tail_wgs)
{
    const StreamKPlan p = streamk_plan(M, N, K);
    const int KT = K / FLEXQ_TILE_K;
    const double stage_us = 1.556, tile_us = stage_us * KT + 7.0;
    const double whole_rounds = (double)(p.full_tiles / kStreamKGrid) * tile_us;
    // every tail tile whole: one more round
    double best = whole_rounds + (p.tail_tiles ? tile_us : 0.0);
    *tail_wgs = 0;
    if (p.tail_tiles == 0 || !may_cut) return best;
    for (int S = 2; S <= 8 && p.tail_tiles * S <= kStreamKGrid && S <= KT; ++S) {
        const double t = whole_rounds + stage_us * ((KT + S - 1) / S) + 7.0 + 14.0 + 2.0 * S;
        if (t < best) {
            best = t;
            *tail_wgs = p.tail_tiles * S;
        }
    }
    if ((long)p.tail_tiles * KT >= 2L * kStreamKGrid) {
        const double t = whole_rounds + stage_us * KT * p.tail_tiles / kStreamKGrid + 7.0 + 45.0;
        if (t < best) {
            best = t;
            *tail_wgs = kStreamKGrid;
        }
    }
    return best;
}

hipError_t launch_gemm_wlds(const LinearArgs &a, int tail_wgs, hipStream_t st)
{
    if (a.group != 0 || a.split_k > 1 || a.sxg) return hipErrorInvalidValue;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    static std::atomic<unsigned long long> lds_allowed[2];
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(gemm_wlds_kernel<false>), LDS_BYTES,
                                     lds_allowed[0]);
    if (e == hipSuccess)
        e = allow_dynamic_lds(reinterpret_cast<const void *>(gemm_wlds_kernel<true>), LDS_BYTES, lds_allowed[1]);
    if (e != hipSuccess) return e;
    const StreamKPlan p = streamk_plan(a.M, a.N, a.K);
    // (without room for the partial sums, or on a device that is not 256 CUs wide, the
    // tail tiles simply run whole)
    if (tail_wgs <= 0 || p.tail_tiles == 0 || a.partial_bytes < p.partial_bytes ||
        device_cu_count() != kStreamKGrid) {
        hipLaunchKernelGGL(gemm_wlds_kernel<false>, dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WAVES),
                           LDS_BYTES, st, a, tiles_m, tiles_n, 0, 0, 0);
        return hipGetLastError();
    }
    // a run is at least one stage, and the tail has at most 256 runs
    const long stages = (long)p.tail_tiles * (a.K / FLEXQ_TILE_K);
    if (tail_wgs > kStreamKGrid) tail_wgs = kStreamKGrid;
    if (tail_wgs > stages) tail_wgs = (int)stages;
    hipLaunchKernelGGL(gemm_wlds_kernel<true>, dim3(kStreamKGrid), dim3(64 * WAVES), LDS_BYTES, st, a,
                       tiles_m, tiles_n, p.full_tiles, p.tail_tiles, tail_wgs);
    return hipGetLastError();
}

}  // namespace flexq
