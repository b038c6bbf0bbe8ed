// Weight quantizer and the 6-bit packer (gfx950); the activation quantizer
// lives with the activation producers.
//
// Quantization is the symmetric, zero-point-free scheme of the paper's Section
// 2.1 with one scale per group of consecutive elements (Section 4.1.1); a whole
// row as one group is the per-channel / per-token case.  The scale is rounded
// to fp16 first and the SAME fp16 value divides the inputs, so quantize and
// dequantize agree; the division is the correctly rounded fp32 one and the
// rounding to an integer is v_rndne_f32 (half to even).
#include "flexq_device.h"
#include "flexq_kernels.h"

namespace {

__device__ __forceinline__ float block_max(float v, float *red)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        v = fmaxf(v, __shfl_xor(v, off, 64));
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if (nw == 1) return v;
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float m = red[0];
    for (int i = 1; i < nw; ++i) m = fmaxf(m, red[i]);
    __syncthreads();
    return m;
}

// fp16 scale of a group from its absmax, and the float the codes divide by.
__device__ __forceinline__ void make_scale(float amax, float qmax, uint16_t &bits, float &sf)
{
    float s32 = amax / qmax;
    bits = f2h(s32);
    sf = h2f(bits);
    if (amax == 0.0f || sf == 0.0f) {
        bits = 0x3c00;
        sf = 1.0f;
    }
}

__device__ __forceinline__ int quant_code(float v, float sf, float qmin, float qmax)
{
    float q = __builtin_rintf(v / sf);
    q = fminf(fmaxf(q, qmin), qmax);
    return (int)q;
}

// One block per (row, group): fp32 in, 6-bit codes out.
__global__ void quant_w6_kernel(const float *__restrict__ w, int K, int G, int8_t *__restrict__ wq,
                                uint16_t *__restrict__ sw)
{
    __shared__ float red[16];
    const int groups = K / G;
    const long unit = blockIdx.x;
    const long row = unit / groups, g = unit % groups;
    const float *src = w + row * K + g * G;
    int8_t *dst = wq + row * K + g * G;
    float amax = 0.0f;
    for (int i = threadIdx.x; i < G; i += blockDim.x) amax = fmaxf(amax, fabsf(src[i]));
    amax = block_max(amax, red);
    uint16_t bits;
    float sf;
    make_scale(amax, 31.0f, bits, sf);
    if (threadIdx.x == 0) sw[unit] = bits;
    for (int i = threadIdx.x; i < G; i += blockDim.x)
        dst[i] = (int8_t)quant_code(src[i], sf, -32.0f, 31.0f);
}

// One thread per (tile, lane): 64 codes in, 48 packed bytes out.
__global__ __launch_bounds__(256) void pack_w6_kernel(const int8_t *__restrict__ wq, int N, int K,
                                                      uint8_t *__restrict__ packed)
{
    const long gid = (long)blockIdx.x * 256 + threadIdx.x;
    const int kt = K / FLEXQ_TILE_K;
    const long tiles = (long)(N / FLEXQ_TILE_ROWS) * kt;
    const long tile = gid >> 6;
    const int lane = (int)(gid & 63);
    if (tile >= tiles) return;
    const long nb = tile / kt, kb = tile % kt;
    const int r = lane & 31, h = lane >> 5;
    const int8_t *row = wq + (nb * FLEXQ_TILE_ROWS + r) * (long)K + kb * FLEXQ_TILE_K + 16 * h;
    uint8_t c[4][16];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint4 v = *reinterpret_cast<const uint4 *>(row + 32 * j);
        __builtin_memcpy(c[j], &v, 16);
    }
    uint8_t *dst = packed + tile * FLEXQ_TILE_BYTES + lane * 16;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        uint8_t o[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            unsigned code = c[j][t] & 63u;
            unsigned spare = ((c[3][t] & 63u) >> (4 - 2 * j)) & 3u;
            o[t] = (uint8_t)((code << 2) | spare);
        }
        uint4 v;
        __builtin_memcpy(&v, o, 16);
        *reinterpret_cast<uint4 *>(dst + 1024 * j) = v;
    }
}

__global__ __launch_bounds__(256) void unpack_w6_kernel(const uint8_t *__restrict__ packed, int N,
                                                        int K, int8_t *__restrict__ wq)
{
    const long gid = (long)blockIdx.x * 256 + threadIdx.x;
    const int kt = K / FLEXQ_TILE_K;
    const long tiles = (long)(N / FLEXQ_TILE_ROWS) * kt;
    const long tile = gid >> 6;
    const int lane = (int)(gid & 63);
    if (tile >= tiles) return;
    const long nb = tile / kt, kb = tile % kt;
    const int r = lane & 31, h = lane >> 5;
    PackedTile t = load_packed_tile_cached(
        reinterpret_cast<const v4i *>(packed + tile * FLEXQ_TILE_BYTES), lane);
    int8_t *row = wq + (nb * FLEXQ_TILE_ROWS + r) * (long)K + kb * FLEXQ_TILE_K + 16 * h;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        v4i d = unpack_kstep(t, j);            // bytes hold 4*w
        int8_t b[16];
        __builtin_memcpy(b, &d, 16);
#pragma unroll
        for (int i = 0; i < 16; ++i) b[i] = (int8_t)(b[i] >> 2);
        uint4 v;
        __builtin_memcpy(&v, b, 16);
        *reinterpret_cast<uint4 *>(row + 32 * j) = v;
    }
}

// Activations in tile order (tiles of 32 tokens x 128 k: four 1 KiB planes of int8, or
// the three planes of the packed 6-bit format) back to row-major int8 codes [M][K].
__global__ __launch_bounds__(256) void untile_act_kernel(const uint8_t *__restrict__ xt, int bits, int M,
                                                         int K, int8_t *__restrict__ xq)
{
    const long gid = (long)blockIdx.x * 256 + threadIdx.x;
    const int kt = K / FLEXQ_TILE_K;
    const long tiles = (long)((M + 31) / 32) * kt;
    const long tile = gid >> 6;
    const int lane = (int)(gid & 63);
    if (tile >= tiles) return;
    const long mb = tile / kt, kb = tile % kt;
    const int r = lane & 31, h = lane >> 5;
    if (mb * 32 + r >= M) return;                       // a padding row of the last block
    int8_t *row = xq + (mb * 32 + r) * (long)K + kb * FLEXQ_TILE_K + 16 * h;
    if (bits == 8) {
        const uint4 *src = reinterpret_cast<const uint4 *>(xt + tile * 4096) + lane;
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4 *>(row + 32 * j) = src[64 * j];
        return;
    }
    PackedTile t = load_packed_tile_cached(reinterpret_cast<const v4i *>(xt + tile * FLEXQ_TILE_BYTES), lane);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        v4i d = unpack_kstep(t, j);            // bytes hold 4*x
        int8_t b[16];
        __builtin_memcpy(b, &d, 16);
#pragma unroll
        for (int i = 0; i < 16; ++i) b[i] = (int8_t)(b[i] >> 2);
        uint4 v;
        __builtin_memcpy(&v, b, 16);
        *reinterpret_cast<uint4 *>(row + 32 * j) = v;
    }
}

// Scales into / out of the packed buffer.  group mode reorders [N][K/128] to
// tile order [N/32][K/128][32].
__global__ void scales_kernel(const uint16_t *__restrict__ src, int N, int K, int group,
                              uint16_t *__restrict__ dst, int to_packed)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (group == 0) {
        if (i < N) dst[i] = src[i];
        return;
    }
    const int kt = K / FLEXQ_TILE_K;
    if (i >= (long)N * kt) return;
    const long n = i / kt, g = i % kt;
    const long tiled = ((n / 32) * kt + g) * 32 + (n % 32);
    if (to_packed)
        dst[tiled] = src[i];
    else
        dst[i] = src[tiled];
}

__global__ void fill_zero_kernel(unsigned *p, long count)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0u;
}

}  // namespace

namespace flexq {

hipError_t launch_quant_w6(const float *w, int N, int K, int group, int8_t *wq, uint16_t *sw,
                           hipStream_t st)
{
    const int G = group == 0 ? K : group;
    const long units = (long)N * (K / G);
    const int threads = G >= 1024 ? 256 : 64;
    hipLaunchKernelGGL(quant_w6_kernel, dim3((unsigned)units), dim3(threads), 0, st, w, K, G, wq, sw);
    return hipGetLastError();
}

hipError_t launch_pack_w6(const int8_t *wq, const uint16_t *sw, int N, int K, int group,
                          void *packed, hipStream_t st)
{
    const long lanes = (long)(N / 32) * (K / 128) * 64;
    hipLaunchKernelGGL(pack_w6_kernel, dim3((unsigned)((lanes + 255) / 256)), dim3(256), 0, st, wq,
                       N, K, (uint8_t *)packed);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    uint16_t *dst = (uint16_t *)((uint8_t *)packed + (size_t)N * K * 6 / 8);
    const long count = group == 0 ? N : (long)N * (K / 128);
    hipLaunchKernelGGL(scales_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, sw, N,
                       K, group, dst, 1);
    return hipGetLastError();
}

hipError_t launch_unpack_w6(const void *packed, int N, int K, int group, int8_t *wq, uint16_t *sw,
                            hipStream_t st)
{
    const long lanes = (long)(N / 32) * (K / 128) * 64;
    hipLaunchKernelGGL(unpack_w6_kernel, dim3((unsigned)((lanes + 255) / 256)), dim3(256), 0, st,
                       (const uint8_t *)packed, N, K, wq);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const uint16_t *src = (const uint16_t *)((const uint8_t *)packed + (size_t)N * K * 6 / 8);
    const long count = group == 0 ? N : (long)N * (K / 128);
    hipLaunchKernelGGL(scales_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, src,
                       N, K, group, sw, 0);
    return hipGetLastError();
}

hipError_t launch_untile_act(const uint8_t *xt, int act_bits, int M, int K, int8_t *xq, hipStream_t st)
{
    const long lanes = (long)((M + 31) / 32) * (K / 128) * 64;
    hipLaunchKernelGGL(untile_act_kernel, dim3((unsigned)((lanes + 255) / 256)), dim3(256), 0, st, xt,
                       act_bits, M, K, xq);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t st)
{
    const long count = (long)(bytes / 4);
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st,
                       (unsigned *)p, count);
    return hipGetLastError();
}

}  // namespace flexq
