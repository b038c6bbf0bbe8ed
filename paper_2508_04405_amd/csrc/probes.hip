// Measurement helpers: the two ceilings the kernels are compared with on the
// box they run on -- how fast a kernel that does nothing but read can stream a
// buffer from HBM, and how fast the matrix pipe runs the i8 MFMA on operands
// with the bit statistics of the real workload (the chip lowers its clock with
// switching activity, so this is well under the published peak).  No part of
// the linear layer's arithmetic; built into the development library only.
#include "../../include/flexq_dev.h"
#include "flexq_device.h"
#include <type_traits>

namespace {

// Every wavefront reads 12 consecutive KiB (all loads in flight at once).
__global__ __launch_bounds__(256) void read_probe_kernel(const v4i *__restrict__ src, long chunks,
                                                         int *sink)
{
    const int lane = threadIdx.x & 63;
    const long wave = ((long)blockIdx.x * 256 + threadIdx.x) >> 6;
    v4i acc = {0, 0, 0, 0};
#pragma unroll
    for (int u = 0; u < 12; ++u) {
        const long c = wave * 12 + u;               // one chunk = 64 lanes x 16 bytes
        if (c < chunks) acc ^= __builtin_nontemporal_load(src + c * 64 + lane);
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x5a5a1234) sink[0] = 1;   // keeps the loads alive
}

// 16 independent 32x32 accumulators, operands fixed in registers: MFMA only.
__global__ __launch_bounds__(256) void mfma_probe_kernel(const v4i *__restrict__ a_src,
                                                         const v4i *__restrict__ b_src, int iters,
                                                         int *sink)
{
    v4i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = a_src[i * 256 + threadIdx.x];
        b[i] = b_src[i * 256 + threadIdx.x] & (int)0xFCFCFCFC;   // as expanded weights: 4*w
    }
    v16i c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) c[i * 4 + j] = mfma_i8(a[i], b[j], c[i * 4 + j]);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[i][r];
    if (s == 0x7fffffff) sink[0] = s;
}

// The matrix pipe beside the other work of a GEMM wavefront, in the GEMM kernels' operand
// pattern: steps of eight MFMAs on four activation operands and two weight operands (each
// weight operand held for four MFMAs), the next step's weight operands being rebuilt
// meanwhile by V vector operations per MFMA (mask operations on packed bytes held in
// registers, as the weight expansion does), and L 16-byte LDS reads per step fetching the
// next step's activation operands.  Nothing else: no global loads, no barriers.
template <int V, int L>
__global__ __launch_bounds__(512) void mfma_mix_kernel(const v4i *__restrict__ a_src,
                                                       const v4i *__restrict__ b_src, int iters, int *sink)
{
    __shared__ __attribute__((aligned(16))) char lds[65536];
    const int tid = threadIdx.x;
    v4i a[4], an[4], p[4], bs[2][2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = a_src[(i * 64 + (tid & 63)) & 1023];
        an[i] = a_src[((i + 4) * 64 + (tid & 63)) & 1023];
        p[i] = b_src[(i * 64 + (tid & 63)) & 1023];
        bs[i >> 1][i & 1] = p[i] & (int)0xFCFCFCFC;
    }
    for (int i = tid; i < 65536 / 16; i += blockDim.x) reinterpret_cast<v4i *>(lds)[i] = a_src[i & 1023];
    __syncthreads();
    v16i c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[i][r] = 0;
    const char *lp = lds + (tid & 63) * 16 + (tid >> 6) * 4096;
    auto step = [&](int it, auto parity, v4i(&cur)[4], v4i(&nxt)[4]) {
        constexpr int PAR = decltype(parity)::value;
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            if (L > 0 && m == 0) {
#pragma unroll
                for (int q = 0; q < L; ++q)
                    nxt[q & 3] = *reinterpret_cast<const v4i *>(lp + ((q + it) & 15) * 1024);
                __builtin_amdgcn_sched_barrier(0);
            }
            c[m] = mfma_i8(bs[PAR][m >> 2], cur[m & 3], c[m]);
#pragma unroll
            for (int v = 0; v < V; ++v) {   // rebuild a dword of the other step's weight operands
                const int k = m * V + v, nt = (k >> 2) & 1, d = k & 3;
                int x;
                asm volatile("v_and_b32 %0, %1, %2" : "=v"(x) : "s"(0xfcfcfcfc), "v"(p[2 * (1 - PAR) + nt][d]));
                bs[1 - PAR][nt][d] = x;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    for (int it = 0; it < iters; it += 2) {
        step(it, std::integral_constant<int, 0>{}, a, an);
        step(it + 1, std::integral_constant<int, 1>{}, an, a);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[i][r];
    if (s == 0x7fffffff) sink[0] = s;
}

template <int V, int L>
void launch_mix(const v4i *a, const v4i *b, int iters, int workgroups, int waves, int *sink, hipStream_t st)
{
    hipLaunchKernelGGL((mfma_mix_kernel<V, L>), dim3((unsigned)workgroups), dim3(64 * waves), 0, st, a, b, iters,
                       sink);
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

flexq_status flexq_dev_probe_hbm_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink || bytes < 1024) return FLEXQ_EINVAL;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) != 0) return FLEXQ_EALIGN;
    const long chunks = (long)(bytes / 1024);
    const long waves = (chunks + 11) / 12;
    const unsigned blocks = (unsigned)((waves + 3) / 4);
    hipLaunchKernelGGL(read_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       (const v4i *)src, chunks, (int *)sink);
    return hipGetLastError() == hipSuccess ? FLEXQ_OK : FLEXQ_EHIP;
}

flexq_status flexq_dev_probe_mfma_i8(const void *a_operands, const void *b_operands, int iters,
                                 int workgroups, void *sink, void *stream)
{
    if (!a_operands || !b_operands || !sink || iters < 1 || workgroups < 1) return FLEXQ_EINVAL;
    if (((reinterpret_cast<uintptr_t>(a_operands) | reinterpret_cast<uintptr_t>(b_operands)) & 15u) != 0)
        return FLEXQ_EALIGN;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0,
                       (hipStream_t)stream, (const v4i *)a_operands, (const v4i *)b_operands, iters,
                       (int *)sink);
    return hipGetLastError() == hipSuccess ? FLEXQ_OK : FLEXQ_EHIP;
}

flexq_status flexq_dev_probe_mfma_mix(const void *a_operands, const void *b_operands, int valu_per_mfma,
                                      int lds_reads_per_8, int iters, int workgroups, int waves, void *sink,
                                      void *stream)
{
    if (!a_operands || !b_operands || !sink || iters < 2 || iters % 2 != 0 || workgroups < 1) return FLEXQ_EINVAL;
    if (waves != 4 && waves != 8) return FLEXQ_EINVAL;
    if (((reinterpret_cast<uintptr_t>(a_operands) | reinterpret_cast<uintptr_t>(b_operands)) & 15u) != 0)
        return FLEXQ_EALIGN;
    const v4i *a = (const v4i *)a_operands, *b = (const v4i *)b_operands;
    int *sk = (int *)sink;
    hipStream_t st = (hipStream_t)stream;
    const int key = valu_per_mfma * 10 + lds_reads_per_8;
    switch (key) {
    case 0: launch_mix<0, 0>(a, b, iters, workgroups, waves, sk, st); break;
    case 20: launch_mix<2, 0>(a, b, iters, workgroups, waves, sk, st); break;
    case 30: launch_mix<3, 0>(a, b, iters, workgroups, waves, sk, st); break;
    case 40: launch_mix<4, 0>(a, b, iters, workgroups, waves, sk, st); break;
    case 60: launch_mix<6, 0>(a, b, iters, workgroups, waves, sk, st); break;
    case 80: launch_mix<8, 0>(a, b, iters, workgroups, waves, sk, st); break;
    case 4: launch_mix<0, 4>(a, b, iters, workgroups, waves, sk, st); break;
    case 34: launch_mix<3, 4>(a, b, iters, workgroups, waves, sk, st); break;
    case 38: launch_mix<3, 8>(a, b, iters, workgroups, waves, sk, st); break;
    default: return FLEXQ_EINVAL;
    }
    return hipGetLastError() == hipSuccess ? FLEXQ_OK : FLEXQ_EHIP;
}

}  // extern "C"
#pragma GCC visibility pop
