/*
 * flexq.h -- C ABI of the MI355X (gfx950) W6A6 / W6A8 quantized linear layer.
 *
 * The operation (paper Section 4.2, Eq. 5 and Eq. 7; Section 4.1.3):
 *
 *     Y[M,N] (fp16) = dequant( Xq[M,K] . Wq[N,K]^T )
 *
 * with Wq signed 6-bit codes in [-32,31] (one fp16 scale per output channel,
 * or per group of 128 consecutive k), Xq signed 6- or 8-bit codes carried in
 * int8 -- or, for batches of up to 32 tokens, in tile order with 6-bit codes
 * packed at 0.75 byte each -- (one fp16 scale per token, or per token and
 * group of 128), the integer product accumulated exactly in
 * int32, and the scales applied in the kernel's epilogue.  Weights are
 * quantized and packed once, offline; activations are quantized online
 * (Section 4.1.3, "FlexQ System Runtime").
 *
 * Conventions for every entry point:
 *   - every pointer marked "dev" is DEVICE memory owned by the caller; the
 *     library allocates nothing and frees nothing;
 *   - `stream` is a hipStream_t (NULL = the null stream); calls only enqueue
 *     work on it and never synchronize;
 *   - fp16 values travel as their 16-bit patterns (uint16_t);
 *   - the return value is FLEXQ_OK or a negative error; arguments are checked
 *     on the host BEFORE any GPU call, so a bad argument never launches work;
 *   - inputs must be finite; codes outside their stated range are a caller
 *     error that is not detected on the device.
 */
#ifndef FLEXQ_H
#define FLEXQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int flexq_status;

enum {
    FLEXQ_OK = 0,
    FLEXQ_EINVAL = -1, /* null pointer, M < 1, bad act_bits / group / mode    */
    FLEXQ_ESHAPE = -2, /* N % 32 != 0, K % 128 != 0, or K > FLEXQ_MAX_K       */
    FLEXQ_EALIGN = -3, /* a pointer is not 16-byte aligned                    */
    FLEXQ_EHIP = -4,   /* the HIP runtime reported an error at launch         */
    FLEXQ_EWORKSPACE = -5 /* workspace missing or smaller than required       */
};

/* Largest reduction length: keeps 4 * 32 * 128 * K below 2^31 with margin
 * (the kernels accumulate 4x the product and shift it back, exactly).       */
#define FLEXQ_MAX_K 65536

/* Human-readable name of a status code (static string, never NULL). */
const char *flexq_status_string(flexq_status s);

/* Version of the packed-weight layout; a packed buffer is only valid for the
 * library version that wrote it. */
int flexq_layout_version(void);

/*
 * Size in bytes of the packed form of Wq[N,K]: exactly N*K*6/8 bytes of codes
 * followed by the fp16 scales (N of them, or N*K/128 in group mode), rounded
 * up to 256 bytes.  group: 0 = one scale per output channel, 128 = one per 128
 * consecutive k.  Returns 0 for an invalid shape or group.
 * (Section 4.3.1: weights are bit-packed offline; Section 4.1.1: group 128.)
 */
size_t flexq_packed_bytes(int N, int K, int group);

/*
 * Offline weight quantization (Section 2.1 symmetric, Section 4.1.1 groups):
 * per channel (group = 0) or per 128-group, scale = fp16(absmax / 31), 1.0 if
 * that is zero; code = clamp(round_half_even(w / scale), -32, 31) with an IEEE
 * fp32 division.
 *   w   dev, fp32 [N,K] row-major (K contiguous)
 *   wq  dev, int8 [N,K], out
 *   sw  dev, fp16 [N] or [N, K/128], out
 */
flexq_status flexq_quant_w6(const float *w, int N, int K, int group, int8_t *wq,
                            uint16_t *sw, void *stream);

/*
 * Offline packing (Section 4.3.1, "Bit-level Data Packing", re-designed for
 * 16-byte-per-lane loads that cover whole 128-byte lines): a bijective repack
 * of the 6-bit two's-complement codes plus a copy of the scales.
 *   wq      dev, int8 [N,K], codes in [-32,31]
 *   sw      dev, fp16 [N] (group 0) or [N, K/128] (group 128)
 *   packed  dev, out, flexq_packed_bytes(N,K,group) bytes, 16-byte aligned
 */
flexq_status flexq_pack_w6(const int8_t *wq, const uint16_t *sw, int N, int K,
                           int group, void *packed, void *stream);

/* Inverse of flexq_pack_w6 (for round-trip checks): packed -> wq, sw. */
flexq_status flexq_unpack_w6(const void *packed, int N, int K, int group,
                             int8_t *wq, uint16_t *sw, void *stream);

/*
 * Online activation quantization (Section 4.1.3; Section 2.1): per token,
 * sx = fp16(absmax / qmax) (1.0 if zero), xq = clamp(round_half_even(x / sx))
 * with qmax = 31 (act_bits 6, range [-32,31]) or 127 (act_bits 8, [-128,127]).
 *   x   dev, fp16 [M,K] row-major, 16-byte aligned
 *   xq  dev, int8 [M,K], out, 16-byte aligned
 *   sx  dev, fp16 [M], out
 * K must be a multiple of 128.
 */
flexq_status flexq_quant_act(const uint16_t *x, int M, int K, int act_bits,
                             int8_t *xq, uint16_t *sx, void *stream);

/*
 * Activation producers with the quantizer fused in (Section 4.1.3: the
 * quantization of an activation happens inside the operator that produces it,
 * so no fp16 copy travels through HBM in between).  Both compute the producer
 * in fp32, round its output h to fp16, and quantize that fp16 h per token
 * exactly as flexq_quant_act would: the codes and scales are bit-identical to
 * flexq_quant_act applied to h.
 *
 * flexq_rmsnorm_quant:  h[m][k] = (x[m][k] / sqrt(mean_k x[m][k]^2 + eps)) * gamma[k]
 *   x      dev, fp16 [M,K] row-major, 16-byte aligned
 *   gamma  dev, fp16 [K], 16-byte aligned
 *   eps    > 0 (an all-zero token then gives h = 0)
 * flexq_swiglu_quant:   h[m][f] = silu(gate_up[m][f]) * gate_up[m][F + f],
 *                       silu(g) = g / (1 + exp(-g))
 *   gate_up  dev, fp16 [M, 2F] row-major (the output of a fused gate|up
 *            linear), 16-byte aligned
 * Common:
 *   xq     dev, int8 [M,K] (or [M,F]), out, 16-byte aligned
 *   sx     dev, fp16 [M], out
 *   h_out  dev, fp16 [M,K] (or [M,F]), out, 16-byte aligned, or NULL when the
 *          fp16 values are not needed (the fused case)
 * K and F must be multiples of 128 and at most FLEXQ_MAX_K.  Inputs must be
 * finite.  Nothing is allocated; the caller owns every buffer.
 */
flexq_status flexq_rmsnorm_quant(const uint16_t *x, const uint16_t *gamma,
                                 float eps, int M, int K, int act_bits,
                                 int8_t *xq, uint16_t *sx, uint16_t *h_out,
                                 void *stream);
flexq_status flexq_swiglu_quant(const uint16_t *gate_up, int M, int F,
                                int act_bits, int8_t *xq, uint16_t *sx,
                                uint16_t *h_out, void *stream);

/*
 * Bytes of workspace the GEMM / GEMV entry points need for (M,N,K): room for
 * split-K partial sums and their arrival counters, and for the quantized
 * activations when the quantize prologue is requested (M * K bytes, 32 * K for
 * fewer than 32 tokens: one block of tiles).  Never 0 for a valid
 * shape.  For M > 128, when the 256x256 output tiles do not come in a multiple
 * of 256 (the CUs of an MI355X), it includes up to 128 MiB (512 KiB per 128-k
 * stage of those tiles, at most 256 of them) in which the workgroups sharing a
 * tile of the last, partial round leave their int32 sums; for 65 to 128 tokens
 * on layers up to 22528 wide with rows of at least 3328, up to 22 MiB for the
 * same purpose (128 KiB per piece of a 128x256 tile cut along K).  It depends on
 * M, N and K only.  The workspace must be 256-byte aligned, and its first
 * FLEXQ_WORKSPACE_COUNTER_BYTES bytes must be zero before the first call that
 * uses it (flexq_workspace_init does that); every call leaves them zero again.
 * Calls that share a workspace must be ordered on one stream.
 */
#define FLEXQ_WORKSPACE_COUNTER_BYTES 16384
size_t flexq_workspace_bytes(int M, int N, int K);

/* Zero the counter area of a fresh workspace (a small fill kernel). */
flexq_status flexq_workspace_init(void *workspace, size_t workspace_bytes,
                                  void *stream);

/*
 * The quantized linear layer (Section 4.2 Eq. 5, Eq. 7; Section 4.3.4 fused
 * dequantization).  W6A6 and W6A8 differ only in the activation code range.
 *
 *   packed     dev, from flexq_pack_w6 with the same N, K, group
 *   group      0 or 128, as packed
 *   xq, sx     dev, quantized activations int8 [M,K] and fp16 scales [M];
 *              ignored (may be NULL) when x_fp16 is given
 *   x_fp16     dev or NULL.  Non-NULL: fp16 activations [M,K]; the call first
 *              quantizes them per token (6 bits for *_w6a6, 8 for *_w6a8) into
 *              the workspace, then multiplies
 *   y          dev, out, fp16 [M,N] row-major
 *   acc_out    dev or NULL.  Non-NULL (group 0 only): receives the exact int32
 *              accumulators [M,N]
 *   workspace  dev, flexq_workspace_bytes(M,N,K) bytes, counters zeroed
 *
 * y[m,n] = fp16( float(acc[m,n]) * (sx[m]*sw[n]) ) for group 0 (the product
 * of two fp16 scales is exact in fp32), and
 * y[m,n] = fp16( sx[m] * sum_g sw[n,g]*float(acc_g[m,n]) ) in fp32 for
 * group 128.  Any M >= 1 is accepted (the tiled kernel needs (M+256)*K and
 * 0.75*N*K below 2^32, else FLEXQ_ESHAPE); flexq_gemm_* pick the kernel from M,
 * flexq_gemv_* are the same calls under the name the decode path uses: for
 * M <= 32 (24 on layers wider than 32768; 64 on layers of at most 2^25 weights,
 * 128 on layers of at most 2^24) both run the bandwidth-bound streaming kernel.
 */
flexq_status flexq_gemm_w6a6(const void *packed, int group, const int8_t *xq,
                             const uint16_t *sx, const uint16_t *x_fp16, int M,
                             int N, int K, uint16_t *y, int32_t *acc_out,
                             void *workspace, size_t workspace_bytes,
                             void *stream);
flexq_status flexq_gemm_w6a8(const void *packed, int group, const int8_t *xq,
                             const uint16_t *sx, const uint16_t *x_fp16, int M,
                             int N, int K, uint16_t *y, int32_t *acc_out,
                             void *workspace, size_t workspace_bytes,
                             void *stream);
flexq_status flexq_gemv_w6a6(const void *packed, int group, const int8_t *xq,
                             const uint16_t *sx, const uint16_t *x_fp16, int M,
                             int N, int K, uint16_t *y, int32_t *acc_out,
                             void *workspace, size_t workspace_bytes,
                             void *stream);
flexq_status flexq_gemv_w6a8(const void *packed, int group, const int8_t *xq,
                             const uint16_t *sx, const uint16_t *x_fp16, int M,
                             int N, int K, uint16_t *y, int32_t *acc_out,
                             void *workspace, size_t workspace_bytes,
                             void *stream);

/*
 * Activations quantized straight into TILE ORDER for batched decode (Section
 * 4.3.1 packs the activations online too; Section 5.2's batch sizes).  The
 * quantizer of flexq_quant_act, same codes and scales, but the codes leave in
 * tiles of 32 tokens x 128 k laid out the way the streaming kernel's lanes
 * consume them: act_bits 8 as four 1 KiB planes of int8 (4096 bytes a tile),
 * act_bits 6 PACKED at 6 bits in the three-plane format of the weight tiles
 * with tokens in the place of output channels (3072 bytes a tile, 0.75 byte per
 * value).  Tile (mb, kb) -- tokens 32 mb .., k 128 kb .. -- lies at
 * (mb * K/128 + kb) * tile bytes; rows of the last block beyond M are never
 * written and never used.
 *   flexq_act_tiles_bytes  size of that buffer, 0 for an invalid shape
 *   flexq_quant_act_tiles  x dev fp16 [M,K] -> xt (dev, out, 16-byte aligned), sx dev fp16 [M]
 *   flexq_untile_act       xt -> xq dev int8 [M,K] row-major (for checks and for
 *                          callers that need the codes elsewhere)
 *   flexq_gemv_tiles       the linear layer of flexq_gemv_w6a6 / _w6a8 (act_bits
 *                          says which) on such activations: M <= 32 (else
 *                          FLEXQ_EINVAL), per-channel or group-128 weight scales,
 *                          same y / acc_out / workspace contract.
 * What it is for: beyond eight tokens the activations of an 8192-deep layer no
 * longer fit the kernel's LDS staging, and from row-major codes every lane then
 * fetches a scattered 128-byte line per token and k-step; from tiles it is
 * three or four coalesced KiB per tile, whatever the token count (a tile always
 * carries 32 token rows).  Measured break-even: about 17 tokens (6-bit), 24
 * (8-bit); the calls that take x_fp16 go this way by themselves from there on,
 * and below it the row-major calls are the faster ones.
 */
size_t flexq_act_tiles_bytes(int act_bits, int M, int K);
flexq_status flexq_quant_act_tiles(const uint16_t *x, int M, int K, int act_bits,
                                   void *xt, uint16_t *sx, void *stream);
flexq_status flexq_untile_act(const void *xt, int M, int K, int act_bits,
                              int8_t *xq, void *stream);
flexq_status flexq_gemv_tiles(int act_bits, const void *packed, int group,
                              const void *xt, const uint16_t *sx, int M, int N,
                              int K, uint16_t *y, int32_t *acc_out,
                              void *workspace, size_t workspace_bytes,
                              void *stream);

/*
 * The paper's full scheme (Section 4.1.1, Eq. 7): BOTH operands carry one fp16
 * scale per group of 128 along K,
 *   y[m,n] = fp16( sum_g sxg[g][m] * sw[n][g] * acc_g[m,n] ),
 * acc_g the exact int32 product over group g; fp32 arithmetic, one rounding.
 *
 * flexq_quant_act_g128: per token and group, scale = fp16(absmax / qmax)
 * (1.0 if zero), codes = clamp(round_half_even(x / scale)), as flexq_quant_act.
 *   x           dev, fp16 [M,K] row-major, 16-byte aligned
 *   xq          dev, int8 [M,K], out, 16-byte aligned
 *   sxg         dev, fp16 [K/128][sxg_stride], out: GROUP-major (the scales of
 *               one group for all tokens are contiguous), sxg_stride >= M;
 *               elements m >= M of a row are not written
 * flexq_linear_g128: the linear layer on such activations.
 *   packed      dev, from flexq_pack_w6 with group = 128
 *   xq, sxg     dev, as written by flexq_quant_act_g128 (A6 or A8 codes alike)
 *   y           dev, fp16 [M,N], out, 16-byte aligned
 *   workspace   as for flexq_gemm_*, flexq_workspace_bytes(M,N,K) bytes
 * Same shape and alignment rules and status codes as the calls above; any
 * M >= 1.  The tiled kernel (larger M) fetches the scales four bytes at a time
 * and needs an even sxg_stride; with an odd one the call still works, on the
 * streaming kernel, 128 tokens at a time.
 */
flexq_status flexq_quant_act_g128(const uint16_t *x, int M, int K, int act_bits,
                                  int8_t *xq, uint16_t *sxg, int sxg_stride,
                                  void *stream);
flexq_status flexq_linear_g128(const void *packed, const int8_t *xq,
                               const uint16_t *sxg, int sxg_stride, int M,
                               int N, int K, uint16_t *y, void *workspace,
                               size_t workspace_bytes, void *stream);

/*
 * The linear layers of one decoder block as one call (Section 4.1.3, "FlexQ System
 * Runtime": every GEMM is fed by the operator that produces its input, with the
 * activation quantizer fused in; Section 4.1.2: the activation width is chosen per
 * linear -- the paper's policy is 8 bits on the down projection, 6 elsewhere).
 *
 *   stage 0   RMS norm(x; gamma_attn) + quantize  ->  fused QKV      -> qkv  [M, QKV]
 *   stage 1   quantize(attn)                      ->  attention out  -> o    [M, H]
 *   stage 2   RMS norm(x_ffn; gamma_ffn) + quant  ->  fused gate|up  -> gate_up [M, 2F]
 *   stage 3   SiLU(gate) * up + quantize          ->  down           -> down [M, H]
 *
 * Attention itself and the residual additions are not part of this path: the caller
 * supplies the attention output `attn` and the input of the second norm `x_ffn` (it
 * may alias `o`), and may run the stages in two calls around its own attention with
 * first_stage / last_stage (0 <= first_stage <= last_stage <= 3).
 *
 * flexq_layer: H hidden size, F feed-forward width, QKV width of the fused QKV
 * projection (all multiples of 128); group 0 or 128 as the four packed buffers were
 * made (w_qkv [QKV,H], w_o [H,H], w_gate_up [2F,H] gate rows first, w_down [H,F]);
 * gamma_* fp16 [H]; eps > 0; bits_* 6 or 8.  flexq_layer_io: fp16 device buffers,
 * 16-byte aligned; h_* are optional outputs (NULL, or fp16 [M,H] / [M,F]) receiving
 * the fp16 values the fused producers quantized, for checks.  Only what the
 * requested stages touch is looked at.  Workspace: flexq_layer_workspace_bytes(L, M)
 * bytes, 256-byte aligned, its first FLEXQ_WORKSPACE_COUNTER_BYTES zero before the
 * first call (flexq_workspace_init), shared by the stages, which run in order on
 * `stream`.  Results of every stage are those of the corresponding single calls
 * (flexq_rmsnorm_quant / flexq_swiglu_quant / flexq_gemm_w6a6 / _w6a8), status codes
 * as theirs; nothing is launched if an argument of any requested stage is bad.
 */
typedef struct {
    int H, F, QKV, group;
    const void *w_qkv, *w_o, *w_gate_up, *w_down;
    const uint16_t *gamma_attn, *gamma_ffn;
    float eps;
    int bits_qkv, bits_o, bits_gate_up, bits_down;
} flexq_layer;

typedef struct {
    const uint16_t *x;        /* in  [M,H]   stage 0 */
    uint16_t *qkv;            /* out [M,QKV] stage 0 */
    const uint16_t *attn;     /* in  [M,H]   stage 1 */
    uint16_t *o;              /* out [M,H]   stage 1 */
    const uint16_t *x_ffn;    /* in  [M,H]   stage 2 */
    uint16_t *gate_up;        /* out [M,2F]  stage 2, in stage 3 */
    uint16_t *down;           /* out [M,H]   stage 3 */
    uint16_t *h_attn_norm, *h_ffn_norm, *h_swiglu;   /* optional outs: [M,H], [M,H], [M,F] */
} flexq_layer_io;

size_t flexq_layer_workspace_bytes(const flexq_layer *L, int M);
flexq_status flexq_layer_linears(const flexq_layer *L, int M, const flexq_layer_io *io,
                                 int first_stage, int last_stage, void *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * For callers that cannot allocate device memory -- code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc: flexq_gemv_w6a8 (same
 * arguments, same results, same status codes) without the workspace arguments.
 * The K-split counters, the partial sums and the quantize prologue's codes live in
 * a fixed array of FLEXQ_NOALLOC_SCRATCH_BYTES inside the library's device image
 * instead (one copy per GPU, held until the process ends).  The call allocates and
 * frees nothing and only enqueues kernels on `stream`: a small fill kernel that
 * zeroes the counter area, then what flexq_gemv_w6a8 would enqueue.  The first
 * call on a device looks up the array's address (once per device) and is best made
 * outside a capture.
 *   - FLEXQ_EWORKSPACE if flexq_workspace_bytes(M, N, K) exceeds
 *     FLEXQ_NOALLOC_SCRATCH_BYTES (decode shapes fit: the LLaMA-2-70B layers up to
 *     64 tokens need under 10 MiB); nothing is launched then.
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap on one
 *     GPU (different streams, no ordering between them) race, and must use
 *     flexq_gemv_w6a8 with workspaces of their own instead.
 */
#define FLEXQ_NOALLOC_SCRATCH_BYTES (16u << 20)
flexq_status flexq_gemv_w6a8_noalloc(const void *packed, int group, const int8_t *xq,
                                     const uint16_t *sx, const uint16_t *x_fp16, int M,
                                     int N, int K, uint16_t *y, int32_t *acc_out,
                                     void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FLEXQ_H */
