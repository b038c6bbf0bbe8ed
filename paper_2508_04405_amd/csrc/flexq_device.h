// Device-side helpers shared by the gfx950 kernels: the packed 6-bit tile
// layout, its in-register expansion to int8, and the i8 MFMA wrapper.
//
// Packed layout (this library's own; the paper's Section 4.3.1 packs 1-bit
// planes for binary tensor cores, which CDNA4 does not need):
//
//   The matrix Wq[N,K] is cut into tiles of 32 rows x 128 k.  Tile (nb, kb)
//   starts at byte (nb * K/128 + kb) * 3072, so the tiles of one 32-row block
//   follow each other along k.  A tile is three planes of 1024 bytes; plane j
//   gives lane l of a wavefront the 16 bytes at l*16, so one
//   global_load_dwordx4 per plane reads 1 KiB contiguous (eight 128-byte
//   lines) per wavefront.  Lane l serves row r = l & 31 and k-half h = l >> 5.
//   Byte t of plane j at lane l holds
//       bits 7..2 : the code of W[32nb + r][128kb + 32j + 16h + t]     (j=0,1,2)
//       bits 1..0 : bits (5-2j)..(4-2j) of the code of
//                   W[32nb + r][128kb + 96 + 16h + t]
//   i.e. three of every four weights sit in the top six bits of a byte and the
//   fourth is spread over the three spare bit pairs.  A byte whose low two
//   bits are cleared IS the int8 value 4*w, so the MFMA runs on 4*w and the
//   int32 sum is shifted right by two, exactly, afterwards.
//
//   After the 3072-byte tiles come the fp16 scales: [N] for per-channel mode,
//   or [N/32][K/128][32] (tile order) for group-128 mode.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

#define FLEXQ_TILE_ROWS 32
#define FLEXQ_TILE_K 128
#define FLEXQ_TILE_BYTES 3072

// One packed tile as a lane sees it: three 16-byte pieces.
struct PackedTile {
    v4i q0, q1, q2;
};

__device__ __forceinline__ PackedTile load_packed_tile(const v4i *tile_base, int lane)
{
    PackedTile t;
    t.q0 = __builtin_nontemporal_load(tile_base + lane);
    t.q1 = __builtin_nontemporal_load(tile_base + 64 + lane);
    t.q2 = __builtin_nontemporal_load(tile_base + 128 + lane);
    return t;
}

__device__ __forceinline__ PackedTile load_packed_tile_cached(const v4i *tile_base, int lane)
{
    PackedTile t;
    t.q0 = tile_base[lane];
    t.q1 = tile_base[64 + lane];
    t.q2 = tile_base[128 + lane];
    return t;
}

// k-step j (0..3) of a tile as the int8 MFMA operand of this lane: 16 values
// 4*w for k = 32j + 16h + 0..15 of row r.
__device__ __forceinline__ v4i unpack_kstep(const PackedTile &t, int j)
{
    const int top6 = (int)0xFCFCFCFC;
    const int low2 = 0x03030303;
    if (j == 0) return t.q0 & top6;
    if (j == 1) return t.q1 & top6;
    if (j == 2) return t.q2 & top6;
    return ((t.q0 & low2) << 6) | ((t.q1 & low2) << 4) | ((t.q2 & low2) << 2);
}

// One dword (four weights) of the same operand, for callers that spread the
// expansion between other instructions.
__device__ __forceinline__ int unpack_kstep_dword(const PackedTile &t, int j, int d)
{
    const int top6 = (int)0xFCFCFCFC;
    const int low2 = 0x03030303;
    if (j == 0) return t.q0[d] & top6;
    if (j == 1) return t.q1[d] & top6;
    if (j == 2) return t.q2[d] & top6;
    // three masks, two shift-ors, one shift (six operations; the flat form above takes seven)
    int r = t.q0[d] & low2;
    r = (r << 2) | (t.q1[d] & low2);
    r = (r << 2) | (t.q2[d] & low2);
    return r << 2;
}

// D[32x32] += A[32 x 32k] * B[32k x 32], int8 in, int32 out.  Lane l supplies
// row (l & 31) of A and column (l & 31) of B, 16 consecutive k each, k-half
// (l >> 5).  Register r of D at lane l is D[8*(r/4) + 4*(l>>5) + r%4][l & 31].
__device__ __forceinline__ v16i mfma_i8(v4i a, v4i b, v16i c)
{
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ int mfma_row(int r, int lane)
{
    return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}

__device__ __forceinline__ float h2f(uint16_t bits)
{
    _Float16 h;
    __builtin_memcpy(&h, &bits, 2);
    return (float)h;
}

__device__ __forceinline__ uint16_t f2h(float f)
{
    _Float16 h = (_Float16)f;          // v_cvt_f16_f32, round half to even
    uint16_t bits;
    __builtin_memcpy(&bits, &h, 2);
    return bits;
}

// The IEEE fp32 quotient v / s for many v and one s, without a division per
// element: r must be the correctly rounded 1 / s.  q = v * r is within an ulp;
// the fused remainder v - q * s is exact, and adding remainder * r rounds to
// the correctly rounded quotient (Markstein's correction; it needs the
// significand of s not to be all ones, and s is an fp16 value here).  Checked
// over every pair of finite fp16 values v and s > 0 by tests/check_exact_division.c.
__device__ __forceinline__ float div_by(float v, float s, float r)
{
    const float q = v * r;
    const float rem = __builtin_fmaf(-q, s, v);
    return __builtin_fmaf(rem, r, q);
}

// Eight fp16 values -> eight int8 codes clamp(rne(v / s), qmin, qmax).  The
// code is biased by 128 into a byte (v_cvt_pk_u8_f32 on an exact integer) and
// the bias is taken off four codes at a time by flipping the top bits.
__device__ __forceinline__ uint2 quant8(const uint4 &v, float s, float r, float qmin, float qmax)
{
    const unsigned w4[4] = {v.x, v.y, v.z, v.w};
    unsigned out[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float lo = __builtin_rintf(div_by(h2f((uint16_t)(w4[i] & 0xffffu)), s, r));
        float hi = __builtin_rintf(div_by(h2f((uint16_t)(w4[i] >> 16)), s, r));
        lo = __builtin_amdgcn_fmed3f(lo, qmin, qmax) + 128.0f;
        hi = __builtin_amdgcn_fmed3f(hi, qmin, qmax) + 128.0f;
        out[i >> 1] = __builtin_amdgcn_cvt_pk_u8_f32(lo, 2 * (i & 1), out[i >> 1]);
        out[i >> 1] = __builtin_amdgcn_cvt_pk_u8_f32(hi, 2 * (i & 1) + 1, out[i >> 1]);
    }
    return make_uint2(out[0] ^ 0x80808080u, out[1] ^ 0x80808080u);
}
