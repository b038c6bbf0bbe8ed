// Activation producers fused with the per-token quantizer (gfx950).
//
// Section 4.1.3 of the paper quantizes activations on the fly inside the
// operator that produces them, so the fp16 tensor never makes a round trip
// through HBM between the producer and the quantized GEMM.  Two producers are
// built here, the two that feed quantized linears in a LLaMA block:
//
//   MODE 0  RMS norm:    h = fp16( (x * rsqrt(mean(x^2) + eps)) * gamma )
//   MODE 1  gated SiLU:  h = fp16( (g / (1 + exp(-g))) * u ),  [g | u] fused
//   MODE 2  identity:    h = x, the stand-alone per-token quantizer
//
// followed by the quantizer of Section 2.1 on h: s = fp16(absmax(h) / qmax),
// code = clamp(rne(h / s)).  h is rounded to fp16 BEFORE it is quantized, so
// the codes are those the stand-alone quantizer gives for the stored fp16 h.
//
// One workgroup of T lanes owns a token.  The token's h values stay in
// registers (CH chunks of eight per lane) between the absmax pass and the
// emit pass, so HBM sees each input element once and each output byte once.
// Short rows take T = 256; long rows take T = 1024 so that a lane holds few
// chunks and the compute unit stays fully occupied (rows are at most 65536
// long, eight chunks per lane).
//
// The codes leave either row-major ([M][K] int8) or in TILE ORDER for the
// streaming kernel (Section 4.3.1 packs the activations online as well): tiles of
// 32 tokens x 128 k in which a lane of the consuming wavefront finds its MFMA
// operands as contiguous 16-byte pieces -- four 1 KiB planes of int8 (8-bit
// activations), or the three planes of the 6-bit weight tile format with tokens
// in the place of output channels (6-bit activations: 0.75 byte per value).
#include "flexq_device.h"
#include "flexq_kernels.h"

namespace {

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Wave results meet in LDS and are combined in a fixed order.
template <bool SUM, int WAVES>
__device__ __forceinline__ float block_reduce(float v, float *red)
{
    v = SUM ? wave_sum(v) : wave_max(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < WAVES; ++i) r = SUM ? r + red[i] : fmaxf(r, red[i]);
    __syncthreads();
    return r;
}

__device__ __forceinline__ unsigned pack_h2(float lo, float hi)
{
    return (unsigned)f2h(lo) | ((unsigned)f2h(hi) << 16);
}

// g / (1 + e^-g) through v_exp_f32 and v_rcp_f32: each is good to an ulp of
// fp32 and the product g * log2(e) to |g| * 2^-24 in the exponent, orders of
// magnitude inside the half ulp of the fp16 result.  e^-g overflowing to
// infinity gives g * 0 = -0, the correctly rounded value there.
__device__ __forceinline__ float silu(float g)
{
    return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.44269504088896341f));
}

template <int MODE, int CH, int T>
__global__ __launch_bounds__(T) void producer_kernel(const uint16_t *__restrict__ in,
                                                       const uint16_t *__restrict__ gamma,
                                                       float eps, int L, float qmax,
                                                       int8_t *__restrict__ xq,
                                                       uint16_t *__restrict__ sx,
                                                       uint16_t *__restrict__ h_out, int layout)
{
    __shared__ float red[T / 64];
    const long row = blockIdx.x;
    const int chunks = L / 8;
    const uint4 *src = reinterpret_cast<const uint4 *>(in + row * (long)(MODE == 1 ? 2 * L : L));
    const uint4 *up = src + chunks;                                  // MODE 1 only
    const uint4 *gam = reinterpret_cast<const uint4 *>(gamma);       // MODE 0 only
    uint4 held[CH], other[CH];            // other: gamma (MODE 0) or the up half (MODE 1)

    float inv = 0.0f;
    if (MODE == 0) {
        float ss = 0.0f;
        auto squares = [&](const uint4 &v) {
            unsigned w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float a = h2f((uint16_t)(w4[i] & 0xffffu)), b = h2f((uint16_t)(w4[i] >> 16));
                ss += a * a;
                ss += b * b;
            }
        };
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = threadIdx.x + T * i;
            if (c < chunks) held[i] = src[c];
        }
        // gamma does not wait for the norm: fetch it ahead of the reduction
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = threadIdx.x + T * i;
            if (c < chunks) other[i] = gam[c];
        }
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (threadIdx.x + T * i < chunks) squares(held[i]);
        ss = block_reduce<true, T / 64>(ss, red);
        inv = 1.0f / sqrtf(ss / (float)L + eps);
    }

    // eight h values of a chunk from its first operand (x, or the gate half) and its second
    auto make_h = [&](const uint4 &a, const uint4 &b) -> uint4 {
        if (MODE == 2) return a;
        unsigned a4[4] = {a.x, a.y, a.z, a.w}, b4[4] = {b.x, b.y, b.z, b.w}, o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float alo = h2f((uint16_t)(a4[i] & 0xffffu)), ahi = h2f((uint16_t)(a4[i] >> 16));
            const float blo = h2f((uint16_t)(b4[i] & 0xffffu)), bhi = h2f((uint16_t)(b4[i] >> 16));
            if (MODE == 0)
                o[i] = pack_h2((alo * inv) * blo, (ahi * inv) * bhi);
            else
                o[i] = pack_h2(silu(alo) * blo, silu(ahi) * bhi);
        }
        return make_uint4(o[0], o[1], o[2], o[3]);
    };

    // fp16 magnitudes of finite values order like their bit patterns
    unsigned best = 0;
    auto scan = [&](const uint4 &v) {
        unsigned w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            best = max(best, w4[i] & 0x7fffu);
            best = max(best, (w4[i] >> 16) & 0x7fffu);
        }
    };
    if (MODE != 0) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = threadIdx.x + T * i;
            if (c < chunks) {
                held[i] = src[c];
                if (MODE == 1) other[i] = up[c];
            }
        }
    }
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        if (threadIdx.x + T * i < chunks) {
            held[i] = make_h(held[i], other[i]);
            scan(held[i]);
        }
    }
    const float amax = block_reduce<false, T / 64>(h2f((uint16_t)best), red);

    float s32 = amax / qmax;
    uint16_t bits = f2h(s32);
    float sf = h2f(bits);
    if (amax == 0.0f || sf == 0.0f) {
        bits = 0x3c00;
        sf = 1.0f;
    }
    if (threadIdx.x == 0) sx[row] = bits;
    const float qmin = -qmax - 1.0f;

    uint2 *dst = reinterpret_cast<uint2 *>(xq + row * (long)L);
    uint4 *hdst = h_out ? reinterpret_cast<uint4 *>(h_out + row * (long)L) : nullptr;
    const float rf = 1.0f / sf;
    // Tile order (layout 6 or 8): chunk c holds the token's codes for k = 8c .. 8c+7, that
    // is k-step j = (c % 16) / 4, k-half h = (c % 16) / 2 % 2 of tile c / 16, first or second
    // eight of the lane's sixteen.  The sixteen chunks of a tile sit in sixteen consecutive
    // lanes (L is a multiple of 128 here), so the 6-bit form fetches the fourth k-step's
    // codes, whose bits it spreads over the low bits of the other three, by a shuffle.
    uint8_t *tiles = reinterpret_cast<uint8_t *>(xq);
    const int lane = threadIdx.x & 63;
    auto emit = [&](const uint4 &v, int c) {
        const uint2 q = quant8(v, sf, rf, qmin, qmax);
        if (layout == 0) {
            dst[c] = q;
        } else {
            const int cc = c & 15, j = cc >> 2;
            const long tile = (row >> 5) * (long)(L >> 7) + (c >> 4);
            const int in_plane = (32 * ((cc >> 1) & 1) + (int)(row & 31)) * 16 + 8 * (cc & 1);
            if (layout == 8) {
                *reinterpret_cast<uint2 *>(tiles + tile * 4096 + j * 1024 + in_plane) = q;
            } else {
                const int src = (lane & ~15) | 12 | (cc & 3);
                const unsigned x3 = (unsigned)__shfl((int)q.x, src, 64), y3 = (unsigned)__shfl((int)q.y, src, 64);
                if (j < 3) {
                    const int sh = 4 - 2 * j;
                    uint2 o;
                    o.x = ((q.x << 2) & 0xFCFCFCFCu) | ((x3 >> sh) & 0x03030303u);
                    o.y = ((q.y << 2) & 0xFCFCFCFCu) | ((y3 >> sh) & 0x03030303u);
                    *reinterpret_cast<uint2 *>(tiles + tile * 3072 + j * 1024 + in_plane) = o;
                }
            }
        }
        if (hdst) hdst[c] = v;
    };
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = threadIdx.x + T * i;
        if (c < chunks) emit(held[i], c);
    }
}

// Group-wise activation quantizer (Section 4.1.1: the activations are cut into the same
// groups of 128 along K as the weights).  Sixteen lanes own one (token, group): eight values
// each, the absmax meets by four shuffles, nothing crosses a wavefront.  Scales are written
// group-major, sxg[g][m], the order in which the linear-layer kernels consume them.
__global__ __launch_bounds__(256) void quant_act_g128_kernel(const uint16_t *__restrict__ x, int M,
                                                             int K, float qmax,
                                                             int8_t *__restrict__ xq,
                                                             uint16_t *__restrict__ sxg, int stride)
{
    const long gid = (long)blockIdx.x * 256 + threadIdx.x;
    const int G = K / 128;
    const long unit = gid >> 4;
    if (unit >= (long)M * G) return;           // the sixteen lanes of a unit leave together
    const long m = unit / G;
    const int g = (int)(unit - m * G), c = (int)(gid & 15);
    const long at = m * K + 128L * g + 8 * c;
    const uint4 v = *reinterpret_cast<const uint4 *>(x + at);
    const unsigned w4[4] = {v.x, v.y, v.z, v.w};
    unsigned best = 0;                         // fp16 magnitudes order like their bit patterns
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        best = max(best, w4[i] & 0x7fffu);
        best = max(best, (w4[i] >> 16) & 0x7fffu);
    }
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) best = max(best, (unsigned)__shfl_xor((int)best, off, 64));
    const float amax = h2f((uint16_t)best);
    uint16_t bits = f2h(amax / qmax);
    float sf = h2f(bits);
    if (amax == 0.0f || sf == 0.0f) {
        bits = 0x3c00;
        sf = 1.0f;
    }
    if (c == 0) sxg[(long)g * stride + m] = bits;
    *reinterpret_cast<uint2 *>(xq + at) = quant8(v, sf, 1.0f / sf, -qmax - 1.0f, qmax);
}

template <int MODE>
hipError_t launch(const uint16_t *in, const uint16_t *gamma, float eps, int M, int L, int act_bits,
                  int8_t *xq, uint16_t *sx, uint16_t *h_out, int layout, hipStream_t st)
{
    if (layout != 0 && (layout != act_bits || L % 128 != 0)) return hipErrorInvalidValue;
    const float qmax = act_bits == 6 ? 31.0f : 127.0f;
    const int chunks = L / 8;
#define FLEXQ_PRODUCER(CH, T)                                                                   \
    hipLaunchKernelGGL((producer_kernel<MODE, CH, T>), dim3(M), dim3(T), 0, st, in, gamma, eps, \
                       L, qmax, xq, sx, h_out, layout)
    if (chunks <= 256)
        FLEXQ_PRODUCER(1, 256);
    else if (chunks <= 512)
        FLEXQ_PRODUCER(2, 256);
    else if (chunks <= 1024)
        FLEXQ_PRODUCER(4, 256);
    else if (chunks <= 2048)
        FLEXQ_PRODUCER(4, 512);
    else if (chunks <= 4096)
        FLEXQ_PRODUCER(8, 512);
    else if (chunks <= 8192)
        FLEXQ_PRODUCER(8, 1024);
    else
        return hipErrorInvalidValue;            // rows longer than 65536: refused by the caller
#undef FLEXQ_PRODUCER
    return hipGetLastError();
}

}  // namespace

namespace flexq {

hipError_t launch_rmsnorm_quant(const uint16_t *x, const uint16_t *gamma, float eps, int M, int K,
                                int act_bits, int8_t *xq, uint16_t *sx, uint16_t *h_out,
                                hipStream_t st, int layout)
{
    return launch<0>(x, gamma, eps, M, K, act_bits, xq, sx, h_out, layout, st);
}

hipError_t launch_swiglu_quant(const uint16_t *gate_up, int M, int F, int act_bits, int8_t *xq,
                               uint16_t *sx, uint16_t *h_out, hipStream_t st, int layout)
{
    return launch<1>(gate_up, nullptr, 0.0f, M, F, act_bits, xq, sx, h_out, layout, st);
}

hipError_t launch_quant_act(const uint16_t *x, int M, int K, int act_bits, int8_t *xq, uint16_t *sx,
                            hipStream_t st, int layout)
{
    return launch<2>(x, nullptr, 0.0f, M, K, act_bits, xq, sx, nullptr, layout, st);
}

hipError_t launch_quant_act_g128(const uint16_t *x, int M, int K, int act_bits, int8_t *xq,
                                 uint16_t *sxg, int stride, hipStream_t st)
{
    const float qmax = act_bits == 6 ? 31.0f : 127.0f;
    const long lanes = (long)M * (K / 128) * 16;
    hipLaunchKernelGGL(quant_act_g128_kernel, dim3((unsigned)((lanes + 255) / 256)), dim3(256), 0, st,
                       x, M, K, qmax, xq, sxg, stride);
    return hipGetLastError();
}

}  // namespace flexq
