// Streaming ("skinny") kernel for decode and small batches, M <= 128.
//
// The time of a small-M linear layer is the one pass over the packed weights
// from HBM (paper Section 3.1: the token-generation phase is memory bound;
// Section 4.3.2: each weight is used once per call).  Every wavefront streams
// whole 3 KiB tiles straight from global memory into registers (three 1 KiB
// contiguous loads, non-temporal so the stream does not displace the
// activations in L2 -- the role the paper gives its evict-first hint), expands
// them to int8 with nine VALU operations per 16 weights, and feeds the 32x32x32
// i8 MFMA with the tokens as the row operand.  Rows beyond M are padding that
// costs nothing: the matrix pipe is a few percent busy at HBM speed.
//
// What decides the speed is how many bytes each CU keeps in flight and how few
// dependent round trips to HBM a wavefront makes (the paper's Section 4.3.6
// pipeline, in CDNA terms): a workgroup of W wavefronts owns one 32-row block
// of W and one K range, the wavefronts interleave over its tiles with P tiles
// (3 KiB each) in flight per wavefront, and the small activation slice the
// workgroup needs is staged once in LDS (padded rows, conflict-free 16-byte
// reads) when it fits.
//
// Where the slice does not fit (more than eight tokens of an 8192-deep layer) each lane
// loads its token's operands per tile: from row-major activations that is four loads of
// 32 scattered lines each, which is what slows batches of 16 to 32 tokens down; from
// activations in TILE ORDER (XT: the quantizer writes tiles of 32 tokens x 128 k whose
// planes give a lane its 16 bytes per k-step contiguously -- int8, or 6 bits packed exactly
// like the weights and expanded the same way, Section 4.3.1) it is three or four
// coalesced 1 KiB loads.  Packed 6-bit operands are 4x on both sides: the sums are 16x.
//
// Partial sums of the wavefronts meet in LDS (the counterpart of the paper's
// Section 4.3.5 reduction: exact integer sums, in any order).  With more than
// one K split the workgroups leave partial sums in the workspace and the last
// one to arrive at the block's counter adds them in split order and runs the
// epilogue; it resets the counter so the workspace is ready for the next call.
#include "flexq_device.h"
#include "flexq_kernels.h"

namespace {

constexpr int kXldsBytes = 64 * 1024;  // activation slice staged in LDS up to this size

template <int MT, bool XLDS>
struct Stage {
    PackedTile w;
    v4i a[XLDS ? 1 : MT][XLDS ? 1 : 4];
    uint16_t gs;      // group scale of this lane's column (group modes)
    uint16_t xs[MT];  // group mode 2: this tile's scale of token 32 mt + (lane & 31)
};

// GROUP: 0 = one scale per output channel and per token; 1 = weight scales per 128-k
// group (Section 4.1.1), one scale per token; 2 = both operands scaled per group (Eq. 7).
template <int MT, int GROUP, bool XLDS, bool NTW, int XT>
__device__ __forceinline__ void load_stage(Stage<MT, XLDS> &s, const v4i *packed,
                                           const uint16_t *scales, const int8_t *const (&xrow)[MT],
                                           const bool (&xact)[MT], long tile_index, int t, int lane,
                                           const uint16_t *sxg, int sxg_stride, int KT)
{
    // NTW: non-temporal loads, so that the weight stream (used once) does not displace
    // the activations in L2; the cached form exists for the ablation only
    s.w = NTW ? load_packed_tile(packed + tile_index * (FLEXQ_TILE_BYTES / 16), lane)
              : load_packed_tile_cached(packed + tile_index * (FLEXQ_TILE_BYTES / 16), lane);
    if (XT != 0) {
        // tile (mt, t) of the activations: plane j gives this lane its 16 bytes of k-step j
        // (8 bits), or the three planes of a packed 6-bit tile; padding rows hold anything
        static_assert(XT == 0 || !XLDS, "tile-ordered activations are read straight from memory");
        constexpr int TB = XT == 6 ? FLEXQ_TILE_BYTES : 4096;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const v4i *tile = reinterpret_cast<const v4i *>(
                reinterpret_cast<const uint8_t *>(xrow[0]) + ((long)mt * KT + t) * TB);
#pragma unroll
            for (int j = 0; j < (XT == 6 ? 3 : 4); ++j) s.a[XLDS ? 0 : mt][XLDS ? 0 : j] = tile[64 * j];
        }
    } else if (!XLDS) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (xact[mt]) {  // lanes of padding rows load nothing
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    s.a[XLDS ? 0 : mt][XLDS ? 0 : j] = *reinterpret_cast<const v4i *>(
                        xrow[mt] + (long)t * FLEXQ_TILE_K + 32 * j);
            }
        }
    }
    if (GROUP) s.gs = scales[tile_index * 32 + (lane & 31)];
    if (GROUP == 2) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            s.xs[mt] = xact[mt] ? sxg[(long)t * sxg_stride + 32 * mt + (lane & 31)] : (uint16_t)0;
    }
}

// Quantizer arithmetic of the fused prologue: the same operations, in the same
// order, as the stand-alone activation quantizer (scale = fp16(absmax / qmax),
// 1.0 if zero; code = clamp(rne(v / scale))), so both give identical codes.
__device__ __forceinline__ void prologue_scale(float amax, float qmax, float &sf)
{
    const float s32 = amax / qmax;
    sf = h2f(f2h(s32));
    if (amax == 0.0f || sf == 0.0f) sf = 1.0f;
}

__device__ __forceinline__ unsigned prologue_code(uint16_t hbits, float sf, float qmin, float qmax)
{
    float q = __builtin_rintf(h2f(hbits) / sf);
    q = fminf(fmaxf(q, qmin), qmax);
    return (unsigned)((int)q & 0xff);
}

template <int MT, int GROUP, bool XLDS, bool FUSEQ, int P, int W, int WPE, bool NTW = true, int XT = 0>
__global__ __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void skinny_kernel(flexq::LinearArgs a)
{
    static_assert(!FUSEQ || (XLDS && MT == 1), "the fused quantizer fills the LDS slice");
    static_assert(XT == 0 || ((XT == 6 || XT == 8) && !XLDS && !FUSEQ && GROUP != 2), "tile-ordered activations");
    // packed 6-bit activations enter the MFMA as 4x, like the weights: the sums are 16 x
    constexpr int SUM_SHIFT = XT == 6 ? 4 : 2;
    constexpr float SUM_SCALE = XT == 6 ? 0.0625f : 0.25f;
    static_assert(!FUSEQ || GROUP != 2, "the fused quantizer makes one scale per token");
    __shared__ int red[W][4][64];
    __shared__ int s_last;
    __shared__ float s_sx[32];      // FUSEQ: per-token scales made in this kernel
    extern __shared__ __attribute__((aligned(16))) uint8_t xlds[];  // XLDS: M rows of (span + 16) bytes

    constexpr int THREADS = 64 * W;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int KS = a.split_k;
    const int nb = blockIdx.x / KS;
    const int s = blockIdx.x % KS;
    const int KT = a.K / FLEXQ_TILE_K;
    const int t0 = (int)((long)s * KT / KS);
    const int t1 = (int)((long)(s + 1) * KT / KS);
    const int M = a.M, N = a.N;

    const v4i *packed = reinterpret_cast<const v4i *>(a.packed);
    const long tile_base = (long)nb * KT;

    // ---- activations: this lane's token row, k-half ------------------------
    const int8_t *xrow[MT];
    bool xact[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int row = 32 * mt + (lane & 31);
        xact[mt] = row < M;
        if (XT != 0)   // the lane's 16 bytes of plane 0 of tile (0, 0)
            xrow[mt] = a.xq + 16 * lane;
        else
            xrow[mt] = a.xq + (long)(xact[mt] ? row : 0) * a.K + 16 * (lane >> 5);
    }
    const int span = (t1 - t0) * FLEXQ_TILE_K;  // bytes of k per token in this K range
    const int xstride = span + 16;              // padded LDS row

    v4i xstage[XLDS ? 4 : 1];
    if (XLDS && !FUSEQ) {
        // issue the slice's global loads first so they complete ahead of the weight stream
        const int chunks_per_row = span >> 4;
        const int total = M * chunks_per_row;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * THREADS;
            if (c < total) {
                const int row = c / chunks_per_row, kc = c - row * chunks_per_row;
                xstage[XLDS ? i : 0] = *reinterpret_cast<const v4i *>(
                    a.xq + (long)row * a.K + (long)t0 * FLEXQ_TILE_K + 16 * kc);
            }
        }
    }

    // FUSEQ, small slices: this thread's share of the fp16 rows, loaded ahead of the
    // weight stream so that the absmax does not queue behind it (loads return in order)
    constexpr int XH = 8;
    uint4 xh[FUSEQ ? XH : 1];
    const int row_chunks = a.K >> 3;                     // 16-byte chunks of 8 fp16 per row
    const bool xh_fits = FUSEQ && M * row_chunks <= XH * THREADS;
    if (FUSEQ && xh_fits) {
#pragma unroll
        for (int i = 0; i < XH; ++i) {
            const int idx = tid + i * THREADS;
            if (idx < M * row_chunks)
                xh[FUSEQ ? i : 0] = reinterpret_cast<const uint4 *>(a.x_fp16)[idx];
        }
    }

    Stage<MT, XLDS> st[P];
    const int tw = t0 + wave;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int t = tw + W * p;
        if (t < t1)
            load_stage<MT, GROUP, XLDS, NTW, XT>(st[p], packed, a.scales, xrow, xact, tile_base + t, t, lane,
                                            a.sxg, a.sxg_stride, KT);
    }

    if (FUSEQ) {
        // The weight tiles above are already in flight; meanwhile quantize the
        // activations here instead of in a separate launch.  Every workgroup
        // scans the whole fp16 row (it is L2-resident) for the token's absmax,
        // then quantizes only its own K range into the LDS slice.
        const float qmax = a.qmax, qmin = -a.qmax - 1.0f;
        auto scan = [](const uint4 &v, unsigned best) {
            const unsigned w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                best = max(best, w4[i] & 0x7fffu);     // fp16 magnitudes order like their bits
                best = max(best, (w4[i] >> 16) & 0x7fffu);
            }
            return best;
        };
        auto emit = [&](const uint4 &v, int m, int c) {    // chunk c of the K range of token m
            const float sf = s_sx[m];
            const unsigned w4[4] = {v.x, v.y, v.z, v.w};
            unsigned out[2] = {0u, 0u};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned lo = prologue_code((uint16_t)(w4[i] & 0xffffu), sf, qmin, qmax);
                const unsigned hi = prologue_code((uint16_t)(w4[i] >> 16), sf, qmin, qmax);
                out[i >> 1] |= (lo | (hi << 8)) << (16 * (i & 1));
            }
            *reinterpret_cast<uint2 *>(xlds + m * xstride + 8 * c) = make_uint2(out[0], out[1]);
        };
        // LDS-only barrier: __syncthreads() would also wait for the weight tiles
        auto lds_sync = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
        for (int m = 0; m < M; ++m) {
            unsigned best = 0;
            if (xh_fits) {
#pragma unroll
                for (int i = 0; i < XH; ++i) {
                    const int idx = tid + i * THREADS;
                    if (idx >= m * row_chunks && idx < (m + 1) * row_chunks)
                        best = scan(xh[FUSEQ ? i : 0], best);
                }
            } else {
                const uint4 *src = reinterpret_cast<const uint4 *>(a.x_fp16 + (long)m * a.K);
                for (int c = tid; c < row_chunks; c += THREADS) best = scan(src[c], best);
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1)
                best = max(best, (unsigned)__shfl_xor((int)best, off, 64));
            if (lane == 0) red[wave][0][m & 3] = (int)best;
            if ((m & 3) == 3 || m == M - 1) {
                lds_sync();
                if (tid <= (m & 3)) {
                    const int mm = (m & ~3) + tid;
                    unsigned b = 0;
                    for (int w = 0; w < W; ++w) b = max(b, (unsigned)red[w][0][tid]);
                    float sf;
                    prologue_scale(h2f((uint16_t)b), qmax, sf);
                    s_sx[mm] = sf;
                }
                lds_sync();
            }
        }
        const int c0 = t0 * 16, c1 = t1 * 16;            // this K range in 8-element chunks
        if (xh_fits) {
#pragma unroll
            for (int i = 0; i < XH; ++i) {
                const int idx = tid + i * THREADS;
                if (idx < M * row_chunks) {
                    const int m = idx / row_chunks, c = idx - m * row_chunks;
                    if (c >= c0 && c < c1) emit(xh[FUSEQ ? i : 0], m, c - c0);
                }
            }
        } else {
            const int span_chunks = c1 - c0;
            for (int idx = tid; idx < M * span_chunks; idx += THREADS) {
                const int m = idx / span_chunks, c = idx - m * span_chunks;
                emit(*reinterpret_cast<const uint4 *>(a.x_fp16 + (long)m * a.K + 8L * (c0 + c)), m, c);
            }
        }
        lds_sync();
    } else if (XLDS) {
        const int chunks_per_row = span >> 4;
        const int total = M * chunks_per_row;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * THREADS;
            if (c < total) {
                const int row = c / chunks_per_row, kc = c - row * chunks_per_row;
                *reinterpret_cast<v4i *>(xlds + row * xstride + 16 * kc) = xstage[XLDS ? i : 0];
            }
        }
        // slices larger than 4 chunks per thread: the rest, synchronously
        for (int c = tid + 4 * THREADS; c < total; c += THREADS) {
            const int row = c / chunks_per_row, kc = c - row * chunks_per_row;
            *reinterpret_cast<v4i *>(xlds + row * xstride + 16 * kc) = *reinterpret_cast<const v4i *>(
                a.xq + (long)row * a.K + (long)t0 * FLEXQ_TILE_K + 16 * kc);
        }
        __syncthreads();
    }
    const uint8_t *xl = xlds + (xact[0] ? (lane & 31) : 0) * xstride + 16 * (lane >> 5);

    v16i acc[MT];
    v16f facc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc[mt][r] = 0;
            facc[mt][r] = 0.0f;
        }

    for (int t = tw; t < t1;) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (t < t1) {
                v4i b[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) b[j] = unpack_kstep(st[p].w, j);
                v4i af[MT][4];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (XLDS) {
                            af[mt][j] = *reinterpret_cast<const v4i *>(
                                xl + (t - t0) * FLEXQ_TILE_K + 32 * j);
                        } else if (XT == 6) {
                            const PackedTile xa = {st[p].a[XLDS ? 0 : mt][0], st[p].a[XLDS ? 0 : mt][XLDS ? 0 : 1],
                                                   st[p].a[XLDS ? 0 : mt][XLDS ? 0 : 2]};
                            af[mt][j] = unpack_kstep(xa, j);
                        } else {
                            af[mt][j] = st[p].a[XLDS ? 0 : mt][XLDS ? 0 : j];
                        }
                    }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    if (GROUP) {
                        v16i part;
#pragma unroll
                        for (int r = 0; r < 16; ++r) part[r] = 0;
#pragma unroll
                        for (int j = 0; j < 4; ++j) part = mfma_i8(af[mt][j], b[j], part);
                        const float gs = h2f(st[p].gs);
                        // registers 4q .. 4q+3 hold token rows 8q .. 8q+7 of this row block:
                        // quarters wholly beyond M are padding and are skipped (uniform)
                        const int live = (M - 32 * mt + 7) >> 3;
                        const int mine = GROUP == 2 ? st[p].xs[mt] : 0;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            if (q < live) {
#pragma unroll
                                for (int r = 4 * q; r < 4 * q + 4; ++r) {
                                    if (GROUP == 2) {
                                        // the scale of token 8q + 4 (lane / 32) + r % 4 for this
                                        // tile sits in the lane of that number
                                        const int src = 8 * q + 4 * (lane >> 5) + (r & 3);
                                        const float xs = h2f(
                                            (uint16_t)__builtin_amdgcn_ds_bpermute(4 * src, mine));
                                        facc[mt][r] =
                                            __builtin_fmaf((float)part[r] * gs, xs, facc[mt][r]);
                                    } else {
                                        facc[mt][r] = __builtin_fmaf((float)part[r], gs, facc[mt][r]);
                                    }
                                }
                            }
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[mt] = mfma_i8(af[mt][j], b[j], acc[mt]);
                    }
                }
                const int tn = t + W * P;
                if (tn < t1)
                    load_stage<MT, GROUP, XLDS, NTW, XT>(st[p], packed, a.scales, xrow, xact, tile_base + tn,
                                                    tn, lane, a.sxg, a.sxg_stride, KT);
                t += W;
            }
        }
    }

    // ---- meet in LDS: 8 token rows (4 accumulator registers) at a time ------
    int *partial_i = reinterpret_cast<int *>(a.partial);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (32 * mt + 8 * g >= M) break;  // these rows are padding (uniform)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                red[wave][q][lane] = GROUP ? __float_as_int(facc[mt][4 * g + q]) : acc[mt][4 * g + q];
            __syncthreads();
            if (tid < 256) {
                const int q = tid >> 6, ln = tid & 63;
                const int m = 32 * mt + mfma_row(4 * g + q, ln);
                const int n = 32 * nb + (ln & 31);
                if (m < M) {
                    int v;
                    if (GROUP) {
                        float f = 0.0f;
#pragma unroll
                        for (int w = 0; w < W; ++w) f += __int_as_float(red[w][q][ln]);
                        v = __float_as_int(f);
                    } else {
                        v = 0;
#pragma unroll
                        for (int w = 0; w < W; ++w) v += red[w][q][ln];
                    }
                    if (KS == 1) {
                        if (GROUP) {
                            a.y[(long)m * N + n] = f2h(__int_as_float(v) * SUM_SCALE *
                                                       (GROUP == 2 ? 1.0f : FUSEQ ? s_sx[m] : h2f(a.sx[m])));
                        } else {
                            const int qv = v >> SUM_SHIFT;
                            if (a.acc_out) a.acc_out[(long)m * N + n] = qv;
                            a.y[(long)m * N + n] =
                                f2h((float)qv * ((FUSEQ ? s_sx[m] : h2f(a.sx[m])) * h2f(a.scales[n])));
                        }
                    } else {
                        // device-coherent write-through store: nothing stays dirty in
                        // this XCD's L2, so publishing needs no cache write-back
                        __hip_atomic_store(&partial_i[((long)s * M + m) * N + n], v, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
            __syncthreads();
        }
    }
    if (KS == 1) return;

    // ---- last workgroup of this row block adds the K splits ---------------
    // Every partial sum was written with a device-scope store; once this
    // thread's stores are acknowledged (vmcnt 0) they are visible to every
    // XCD, so the barrier plus one relaxed device-scope counter increment
    // publishes them.  The reader uses device-scope loads, which never hit
    // stale lines.  A full release/acquire fence would write back and
    // invalidate the whole L2 for every workgroup -- far dearer than the GEMV.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        unsigned prev = __hip_atomic_fetch_add(&a.counters[nb], 1u, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == (unsigned)(KS - 1));
    }
    __syncthreads();
    if (!s_last) return;
    if (tid == 0)
        __hip_atomic_store(&a.counters[nb], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int n = 32 * nb + (tid & 31);
    for (int m = tid >> 5; m < M; m += THREADS / 32) {
        if (GROUP) {
            float f = 0.0f;
            for (int k = 0; k < KS; ++k)
                f += __int_as_float(__hip_atomic_load(&partial_i[((long)k * M + m) * N + n],
                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            a.y[(long)m * N + n] = f2h(f * SUM_SCALE * (GROUP == 2 ? 1.0f : FUSEQ ? s_sx[m] : h2f(a.sx[m])));
        } else {
            int v = 0;
            for (int k = 0; k < KS; ++k)
                v += __hip_atomic_load(&partial_i[((long)k * M + m) * N + n], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            const int q = v >> SUM_SHIFT;
            if (a.acc_out) a.acc_out[(long)m * N + n] = q;
            a.y[(long)m * N + n] = f2h((float)q * ((FUSEQ ? s_sx[m] : h2f(a.sx[m])) * h2f(a.scales[n])));
        }
    }
}

template <int MT, int GROUP, bool XLDS, bool FUSEQ, int P, int W, int WPE, bool NTW = true, int XT = 0>
hipError_t launch_one(const flexq::LinearArgs &a, hipStream_t st)
{
    const unsigned blocks = (unsigned)(a.N / 32) * (unsigned)a.split_k;
    auto kern = skinny_kernel<MT, GROUP, XLDS, FUSEQ, P, W, WPE, NTW, XT>;
    size_t dyn = 0;
    if (XLDS) {
        const int KT = a.K / 128;
        const int max_tiles = (KT + a.split_k - 1) / a.split_k;
        dyn = (size_t)a.M * (max_tiles * 128 + 16);
        static std::atomic<unsigned long long> lds_allowed{0};
        if (hipError_t e = flexq::allow_dynamic_lds(reinterpret_cast<const void *>(kern),
                                                    kXldsBytes + 32 * 16, lds_allowed);
            e != hipSuccess)
            return e;
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(64 * W), dyn, st, a);
    return hipGetLastError();
}

template <int GROUP>
hipError_t pick(const flexq::LinearArgs &a, int waves, hipStream_t st)
{
    const int KT = a.K / 128;
    const int max_tiles = (KT + a.split_k - 1) / a.split_k;
    const bool xlds = a.M <= 32 && (long)a.M * max_tiles * 128 <= kXldsBytes;
    if (a.xt != 0) {  // activations in tile order: one token block, per-token scales
        if (a.M > 32 || GROUP == 2 || a.x_fp16 || a.ablate != 0) return hipErrorInvalidValue;
        constexpr int G = GROUP == 2 ? 1 : GROUP;     // never instantiated for mode 2
        if (a.xt == 6) {
            if (waves >= 8) return launch_one<1, G, false, false, 2, 8, 4, true, 6>(a, st);
            return launch_one<1, G, false, false, 2, 4, 4, true, 6>(a, st);
        }
        if (a.xt == 8) {
            if (waves >= 8) return launch_one<1, G, false, false, 2, 8, 4, true, 8>(a, st);
            return launch_one<1, G, false, false, 2, 4, 4, true, 8>(a, st);
        }
        return hipErrorInvalidValue;
    }
    if (a.x_fp16) {  // fused quantize prologue: the caller checked skinny_can_fuse()
        if (!xlds || GROUP == 2) return hipErrorInvalidValue;
        constexpr int G = GROUP == 2 ? 1 : GROUP;     // never instantiated for mode 2
        if (waves == 16) return launch_one<1, G, true, true, 4, 16, 4>(a, st);
        if (waves == 8) return launch_one<1, G, true, true, 4, 8, 4>(a, st);
        return launch_one<1, G, true, true, 4, 4, 4>(a, st);
    }
    // Ablation variants (development build, measurement only): one design choice of the
    // decode kernel undone.
#ifndef FLEXQ_DEV
    if (a.ablate != 0) return hipErrorInvalidValue;
#else
    if (a.ablate != 0) {
        if (GROUP != 0 || a.M > 32 || a.x_fp16 || waves != 8) return hipErrorInvalidValue;
        constexpr int G = 0;
        if (a.ablate == 4) return launch_one<1, G, false, false, 4, 8, 4>(a, st);   // no LDS staging
        if (!xlds) return hipErrorInvalidValue;
        if (a.ablate == 1) return launch_one<1, G, true, false, 4, 8, 4, false>(a, st);   // cached loads
        if (a.ablate == 2) return launch_one<1, G, true, false, 1, 8, 4>(a, st);   // one tile in flight
        if (a.ablate == 3) return launch_one<1, G, true, false, 2, 8, 4>(a, st);   // two tiles in flight
        return hipErrorInvalidValue;
    }
#endif
    if (a.M <= 32) {
        if (xlds) {
            if (waves == 16) return launch_one<1, GROUP, true, false, 4, 16, 4>(a, st);
            if (waves == 8) return launch_one<1, GROUP, true, false, 4, 8, 4>(a, st);
            return launch_one<1, GROUP, true, false, 4, 4, 4>(a, st);
        }
        if (waves == 16) return launch_one<1, GROUP, false, false, 2, 16, 4>(a, st);
        if (waves == 8) return launch_one<1, GROUP, false, false, 2, 8, 4>(a, st);
        return launch_one<1, GROUP, false, false, 2, 4, 4>(a, st);
    }
    if (a.M <= 64) {
        if (waves >= 8) return launch_one<2, GROUP, false, false, 2, 8, 2>(a, st);
        return launch_one<2, GROUP, false, false, 2, 4, 2>(a, st);
    }
    if (waves >= 8) return launch_one<4, GROUP, false, false, 1, 8, 2>(a, st);
    return launch_one<4, GROUP, false, false, 1, 4, 2>(a, st);
}

}  // namespace

namespace flexq {

bool skinny_slice_fits(int M, int K, int split_k)
{
    const int KT = K / 128;
    const int max_tiles = (KT + split_k - 1) / split_k;
    return M <= 32 && (long)M * max_tiles * 128 <= kXldsBytes;
}

bool skinny_can_fuse(int M, int K, int split_k)
{
    const int KT = K / 128;
    const int max_tiles = (KT + split_k - 1) / split_k;
    return M <= 8 && (long)M * max_tiles * 128 <= kXldsBytes;
}

hipError_t launch_skinny(const LinearArgs &a, int waves, hipStream_t st)
{
    if (a.sxg) return a.group == 128 ? pick<2>(a, waves, st) : hipErrorInvalidValue;
    return a.group != 0 ? pick<1>(a, waves, st) : pick<0>(a, waves, st);
}

}  // namespace flexq
