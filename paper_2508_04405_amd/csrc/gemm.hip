// Tiled i8-MFMA GEMM for prefill-sized M.
//
// Large M makes the layer a dense contraction, so the matrix pipe is the
// roofline (the paper measures no batch above 8; Section 4.3.6 describes its
// pipeline, which this kernel re-creates for CDNA4 in its own way):
//   - activations (int8) go global -> registers -> LDS, double buffered, one
//     128-k stage ahead, in an XOR-swizzled row layout so that both the 16-byte
//     writes and the 16-byte MFMA-operand reads are bank-conflict free;
//   - packed weights never touch LDS: each wavefront loads the 3 KiB tiles of
//     its own columns straight into registers one stage ahead and expands them
//     to int8 (nine VALU operations per 16 weights) in the shadow of the MFMAs;
//     an expanded operand is reused by MT MFMAs, which is what keeps the VALU
//     work hidden;
//   - the epilogue shifts the 4x accumulators back, applies sx[m]*sw[n] in
//     fp32 and stores fp16 (Section 4.3.4, fused dequantization).
// Workgroup ids are remapped so that the workgroups an XCD runs at one time
// form a compact block of output tiles and share operand panels in that XCD's
// L2.
#include "flexq_device.h"
#include "flexq_kernels.h"
#include <type_traits>

namespace {

// swizzled byte offset of 16-byte chunk c (0..7) of row `row` in a stage
__device__ __forceinline__ int lds_off(int row, int c)
{
    return row * 128 + ((c ^ ((row >> 1) & 7)) << 4);
}

// s_waitcnt vmcnt(N): at most N of this wavefront's vector-memory loads (in
// issue order, LDS-DMA loads included) are still outstanding afterwards.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() (and any
// fence the compiler knows about) also waits for every outstanding global load
// -- LDS-DMA loads share the counter -- which would drain the prefetch pipeline
// at the end of each stage.  Here every wavefront has already waited, by count,
// for exactly the loads that must have landed; its own LDS reads are complete
// once lgkmcnt is zero.  The asm is opaque to the compiler, so no memory access
// moves across it.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int WM, int WN, int MT, int NT, bool GROUP, int WPE>
__global__ __launch_bounds__(64 * WM * WN) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void gemm_kernel(flexq::LinearArgs a, int tiles_m, int tiles_n)
{
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
    const int nblk = tiles_m * tiles_n;
    int bid = blockIdx.x;
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
    const int8_t *xsrc[XDMA];
#pragma unroll
    for (int i = 0; i < XDMA; ++i) {
        const int q = wave * XDMA + i;
        const int row = 8 * q + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        int m = bm0 + row;
        m = m < M ? m : M - 1;
        xsrc[i] = a.xq + (long)m * K + 16 * c;
    }
    auto dma_x = [&](int kb, int buf) {
#pragma unroll
        for (int i = 0; i < XDMA; ++i) {
            uint8_t *dst = lds + buf * XSTAGE + (wave * XDMA + i) * 1024;
            __builtin_amdgcn_global_load_lds(
                (const void __attribute__((address_space(1))) *)(xsrc[i] + (long)kb * FLEXQ_TILE_K),
                (void __attribute__((address_space(3))) *)dst, 16, 0, 0);
        }
    };

    // ---- per-wave packed tiles ---------------------------------------------
    const v4i *wsrc[NT];
    bool wvalid[NT];
    int wnb[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        int nb = bn0 / 32 + wn * NT + nt;
        wvalid[nt] = nb < N / 32;
        nb = wvalid[nt] ? nb : N / 32 - 1;
        wnb[nt] = nb;
        wsrc[nt] = reinterpret_cast<const v4i *>(a.packed) + (long)nb * KT * (FLEXQ_TILE_BYTES / 16);
    }

    v16i acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0;
    v16f facc[GROUP ? MT : 1][GROUP ? NT : 1];
    if (GROUP) {
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
            wreg[B][nt] = load_packed_tile_cached(wsrc[nt] + (long)kb * (FLEXQ_TILE_BYTES / 16), lane);
            if (GROUP) gsreg[B][nt] = a.scales[((long)wnb[nt] * KT + kb) * 32 + (lane & 31)];
        }
    };

    // prologue: stages 0 and 1 in flight, stage 0 landed
    dma_x(0, 0);
    load_w(0, std::integral_constant<int, 0>{});
    if (KT > 1) {
        dma_x(1, 1);
        load_w(1, std::integral_constant<int, 1>{});
    }
    wait_vmcnt<0>();
    lds_barrier();

    const int arow = (wm * MT) * 32 + (lane & 31);
    const int ahalf = lane >> 5;

    // One 128-k stage.  CUR = kb % 3 names the LDS buffer and register set it reads.
    auto stage = [&](int kb, auto cur_tag) {
        constexpr int CUR = decltype(cur_tag)::value;
        constexpr int NXT2 = (CUR + 2) % 3;
        const bool more2 = kb + 2 < KT;
        if (more2) {  // two stages ahead: that buffer was last read in stage kb - 1
            dma_x(kb + 2, NXT2);
            load_w(kb + 2, std::integral_constant<int, NXT2>{});
        }
        const uint8_t *xs = lds + CUR * XSTAGE;
        v16i part[GROUP ? MT : 1][GROUP ? NT : 1];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v4i af[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                af[mt] = *reinterpret_cast<const v4i *>(xs + lds_off(arow + 32 * mt, 2 * j + ahalf));
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const v4i bf = unpack_kstep(wreg[CUR][nt], j);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    if (GROUP) {
                        if (j == 0) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) part[GROUP ? mt : 0][GROUP ? nt : 0][r] = 0;
                        }
                        part[GROUP ? mt : 0][GROUP ? nt : 0] =
                            mfma_i8(af[mt], bf, part[GROUP ? mt : 0][GROUP ? nt : 0]);
                    } else {
                        acc[mt][nt] = mfma_i8(af[mt], bf, acc[mt][nt]);
                    }
                }
            }
        }
        if (GROUP) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const float gs = h2f(gsreg[CUR][nt]);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        facc[GROUP ? mt : 0][GROUP ? nt : 0][r] +=
                            (float)part[GROUP ? mt : 0][GROUP ? nt : 0][r] * gs;
            }
        }
        // stage kb + 1 must have landed in LDS (every wavefront's share) before
        // anyone reads it; the loads of stage kb + 2 may stay in flight
        if (more2)
            wait_vmcnt<XDMA + WLOADS + (GROUP ? NT : 0)>();
        else
            wait_vmcnt<0>();
        lds_barrier();
    };

    int kb = 0;
    for (; kb + 2 < KT; kb += 3) {
        stage(kb, std::integral_constant<int, 0>{});
        stage(kb + 1, std::integral_constant<int, 1>{});
        stage(kb + 2, std::integral_constant<int, 2>{});
    }
    if (kb < KT) stage(kb, std::integral_constant<int, 0>{});
    if (kb + 1 < KT) stage(kb + 1, std::integral_constant<int, 1>{});

    // ---- epilogue -----------------------------------------------------------
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        if (!wvalid[nt]) continue;
        const int n = bn0 + (wn * NT + nt) * 32 + (lane & 31);
        const float swn = GROUP ? 0.25f : h2f(a.scales[n]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = bm0 + (wm * MT + mt) * 32 + mfma_row(r, lane);
                if (m < M) {
                    const float sxm = h2f(a.sx[m]);
                    if (GROUP) {
                        a.y[(long)m * N + n] = f2h(facc[GROUP ? mt : 0][GROUP ? nt : 0][r] * swn * sxm);
                    } else {
                        const int q = acc[mt][nt][r] >> 2;
                        if (a.acc_out) a.acc_out[(long)m * N + n] = q;
                        a.y[(long)m * N + n] = f2h((float)q * (sxm * swn));
                    }
                }
            }
        }
    }
}

template <int WM, int WN, int MT, int NT, bool GROUP, int WPE>
hipError_t launch_cfg(const flexq::LinearArgs &a, hipStream_t st)
{
    constexpr int BM = WM * MT * 32, BN = WN * NT * 32;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const size_t lds_bytes = 3 * BM * 128;
    auto kern = gemm_kernel<WM, WN, MT, NT, GROUP, WPE>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WM * WN), lds_bytes, st, a,
                       tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

namespace flexq {

hipError_t launch_gemm(const LinearArgs &a, int cfg, hipStream_t st)
{
    if (a.group != 0) return launch_cfg<2, 2, 2, 2, true, 1>(a, st);
    switch (cfg) {
    case 1: return launch_cfg<2, 2, 4, 4, false, 1>(a, st);   // 256x256, 4 waves, 1 wave/SIMD
    case 2: return launch_cfg<2, 4, 4, 2, false, 2>(a, st);   // 256x256, 8 waves (128x64 each)
    case 3: return launch_cfg<4, 2, 2, 4, false, 2>(a, st);   // 256x256, 8 waves (64x128 each)
    case 4: return launch_cfg<2, 2, 2, 4, false, 2>(a, st);   // 128x256, 4 waves, 2 workgroups/CU
    case 5: return launch_cfg<2, 2, 4, 2, false, 2>(a, st);   // 256x128, 4 waves, 2 workgroups/CU
    case 6: return launch_cfg<1, 4, 8, 2, false, 1>(a, st);   // 256x256, 4 waves side by side (256x64 each)
    default: return launch_cfg<2, 4, 4, 2, false, 2>(a, st);
    }
}

}  // namespace flexq
