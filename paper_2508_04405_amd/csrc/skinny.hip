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
// Work split: one workgroup per (32-row block of W, K split); its four
// wavefronts interleave over the tiles of that K range, and their partial
// sums meet in LDS (the counterpart of the paper's Section 4.3.5 reduction:
// exact integer sums, in any order).  With more than one K split the
// workgroups leave partial sums in the workspace and the last one to arrive
// at the block's counter adds them and runs the epilogue; it resets the
// counter so the workspace is ready for the next call.
#include "flexq_device.h"
#include "flexq_kernels.h"

namespace {

template <int MT>
struct Stage {
    PackedTile w;
    v4i a[MT][4];
    uint16_t gs;  // group scale of this lane's column (group mode)
};

template <int MT, bool GROUP>
__device__ __forceinline__ void load_stage(Stage<MT> &s, const v4i *packed, const uint16_t *scales,
                                           const int8_t *const (&xrow)[MT], long tile_index, int t,
                                           int lane)
{
    s.w = load_packed_tile(packed + tile_index * (FLEXQ_TILE_BYTES / 16), lane);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            s.a[mt][j] = *reinterpret_cast<const v4i *>(xrow[mt] + (long)t * FLEXQ_TILE_K + 32 * j);
    if (GROUP) s.gs = scales[tile_index * 32 + (lane & 31)];
}

template <int MT, bool GROUP, int P, int WAVES_PER_EU>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WAVES_PER_EU, WAVES_PER_EU)))
void skinny_kernel(flexq::LinearArgs a)
{
    __shared__ int red[4][16][64];
    __shared__ int s_last;

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

    const int8_t *xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int row = 32 * mt + (lane & 31);
        row = row < M ? row : M - 1;
        xrow[mt] = a.xq + (long)row * a.K + 16 * (lane >> 5);
    }

    v16i acc[MT];
    v16f facc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc[mt][r] = 0;
            facc[mt][r] = 0.0f;
        }

    Stage<MT> st[P];
    const int tw = t0 + wave;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int t = tw + 4 * p;
        if (t < t1) load_stage<MT, GROUP>(st[p], packed, a.scales, xrow, tile_base + t, t, lane);
    }

    for (int t = tw; t < t1;) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (t < t1) {
                v4i b[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) b[j] = unpack_kstep(st[p].w, j);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    if (GROUP) {
                        v16i part;
#pragma unroll
                        for (int r = 0; r < 16; ++r) part[r] = 0;
#pragma unroll
                        for (int j = 0; j < 4; ++j) part = mfma_i8(st[p].a[mt][j], b[j], part);
                        const float gs = h2f(st[p].gs);
#pragma unroll
                        for (int r = 0; r < 16; ++r) facc[mt][r] += (float)part[r] * gs;
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[mt] = mfma_i8(st[p].a[mt][j], b[j], acc[mt]);
                    }
                }
                const int tn = t + 4 * P;
                if (tn < t1)
                    load_stage<MT, GROUP>(st[p], packed, a.scales, xrow, tile_base + tn, tn, lane);
                t += 4;
            }
        }
    }

    // ---- meet in LDS, one 32-token slab at a time -------------------------
    int *partial_i = reinterpret_cast<int *>(a.partial);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            red[wave][r][lane] = GROUP ? __float_as_int(facc[mt][r]) : acc[mt][r];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i;
            const int r = idx >> 6, ln = idx & 63;
            const int m = 32 * mt + mfma_row(r, ln);
            const int n = 32 * nb + (ln & 31);
            if (m < M) {
                int v;
                if (GROUP) {
                    float f = __int_as_float(red[0][r][ln]) + __int_as_float(red[1][r][ln]) +
                              __int_as_float(red[2][r][ln]) + __int_as_float(red[3][r][ln]);
                    v = __float_as_int(f);
                } else {
                    v = red[0][r][ln] + red[1][r][ln] + red[2][r][ln] + red[3][r][ln];
                }
                if (KS == 1) {
                    if (GROUP) {
                        a.y[(long)m * N + n] = f2h(__int_as_float(v) * 0.25f * h2f(a.sx[m]));
                    } else {
                        const int q = v >> 2;
                        if (a.acc_out) a.acc_out[(long)m * N + n] = q;
                        a.y[(long)m * N + n] = f2h((float)q * (h2f(a.sx[m]) * h2f(a.scales[n])));
                    }
                } else {
                    partial_i[((long)s * M + m) * N + n] = v;
                }
            }
        }
        __syncthreads();
    }
    if (KS == 1) return;

    // ---- last workgroup of this row block adds the K splits ---------------
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        unsigned prev = __hip_atomic_fetch_add(&a.counters[nb], 1u, __ATOMIC_ACQ_REL,
                                               __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == (unsigned)(KS - 1));
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    if (tid == 0)
        __hip_atomic_store(&a.counters[nb], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int n = 32 * nb + (tid & 31);
    for (int m = tid >> 5; m < M; m += 8) {
        if (GROUP) {
            float f = 0.0f;
            for (int k = 0; k < KS; ++k)
                f += __int_as_float(__builtin_nontemporal_load(&partial_i[((long)k * M + m) * N + n]));
            a.y[(long)m * N + n] = f2h(f * 0.25f * h2f(a.sx[m]));
        } else {
            int v = 0;
            for (int k = 0; k < KS; ++k)
                v += __builtin_nontemporal_load(&partial_i[((long)k * M + m) * N + n]);
            const int q = v >> 2;
            if (a.acc_out) a.acc_out[(long)m * N + n] = q;
            a.y[(long)m * N + n] = f2h((float)q * (h2f(a.sx[m]) * h2f(a.scales[n])));
        }
    }
}

template <int MT, bool GROUP, int P, int WPE>
hipError_t launch_one(const flexq::LinearArgs &a, hipStream_t st)
{
    const unsigned blocks = (unsigned)(a.N / 32) * (unsigned)a.split_k;
    hipLaunchKernelGGL((skinny_kernel<MT, GROUP, P, WPE>), dim3(blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace

namespace flexq {

hipError_t launch_skinny(const LinearArgs &a, hipStream_t st)
{
    const bool g = a.group != 0;
    if (a.M <= 32) return g ? launch_one<1, true, 2, 4>(a, st) : launch_one<1, false, 2, 4>(a, st);
    if (a.M <= 64) return g ? launch_one<2, true, 2, 2>(a, st) : launch_one<2, false, 2, 2>(a, st);
    return g ? launch_one<4, true, 1, 2>(a, st) : launch_one<4, false, 1, 2>(a, st);
}

}  // namespace flexq
