/*
 * flexq_dev.h -- C ABI of the DEVELOPMENT library, libflexq_dev.so.
 *
 * Test and measurement infrastructure, not part of the product: the same sources
 * as libflexq.so compiled with FLEXQ_DEV, which adds (a) the linear-layer call
 * with per-call overrides of the kernel choice, (b) kernel variants that undo one
 * design choice of the decode kernel (in the manner of the paper's Table 6) and
 * tile shapes the dispatch never picks, (c) two probes of the machine's ceilings.
 * libflexq.so exports none of this and contains none of those kernels.  Nothing
 * here keeps state between calls.  Conventions as in flexq.h.
 */
#ifndef FLEXQ_DEV_H
#define FLEXQ_DEV_H

#include "flexq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Overrides for ONE call; every field 0 = the library's own choice.
 *   kernel    1 = streaming (skinny) kernel, 2 = tiled GEMM kernels
 *   split_k   number of K splits (streaming kernel; 128x128 tiles), at most 64
 *   waves     wavefronts per workgroup of the streaming kernel: 4, 8 or 16
 *   gemm_cfg  tile configuration of the tiled kernels (the codes flexq_dev_linear
 *             reports back, below)
 *   ablate    undo one design choice of the streaming decode kernel (Table 6):
 *             1  weight tiles through ordinary cached loads instead of non-temporal
 *                ones (Section 4.3.2's evict-first hint, undone)
 *             2  one weight tile in flight per wavefront instead of four (Section
 *                4.3.6's multi-stage pipeline, undone)      3  two tiles in flight
 *             4  activations loaded per tile from global memory instead of staged
 *                once in LDS
 *             (per-channel scales, M <= 32, pre-quantized activations, waves = 8;
 *             other calls return FLEXQ_EHIP while a choice is set)
 *   fuse      the activation-quantize prologue inside the streaming kernel (fp16 in):
 *             1 = whenever the kernel can (up to 8 tokens whose K range fits LDS; the
 *             library's own choice is one token), 2 = never (a quantize launch first)
 *   tiles     fp16 activations of up to 32 tokens quantized into tile order (packed at 6
 *             bits for act_bits 6) for the streaming kernel: 1 = always, 2 = never (the
 *             library's own choice: 17 to 32 tokens, 24 to 32 with 8-bit activations,
 *             whose activation slice does not fit the kernel's LDS staging)
 *   spin      gemm_cfg 13 with every tile cut into the same number of pieces: how many
 *             times a piece polls its tile's counter for the other pieces' sums before
 *             it gives up and leaves its slabs to the piece that completes the count
 *             (0 = the library's 128; -1 = never wait, every piece gives up at once:
 *             the path a busy or smaller device takes; at most 1 << 20)
 * With gemm_cfg 13, split_k > 1 asks for that many pieces per tile of the last round.
 */
typedef struct {
    int kernel, split_k, waves, gemm_cfg, ablate, fuse, tiles, spin;
} flexq_dev_tuning;

/*
 * flexq_gemm_w6a6 / _w6a8 / flexq_linear_g128 (Section 4.2 Eq. 5, Eq. 7) with
 * overrides.  act_bits 6 or 8; sxg non-NULL selects group-wise activation scales
 * (then group must be 128, sx and x_fp16 NULL).  tuning NULL = automatic; any
 * field out of range -> FLEXQ_EINVAL before anything else happens.  *dispatched
 * (may be NULL) receives what was launched: 1000 * c + s, c = 1 for the streaming
 * kernel, else the tile configuration (5: 64x128, 7: 128x256, 8: 128x128,
 * 12: 256x256 with both operands through LDS, at most one workgroup per CU,
 * 13: the same with the tiles beyond the last whole round of 256 cut along K,
 * 14: with those tiles run as 256x128 half tiles, 15: 128x256 tiles of the same kernel,
 * for up to 128 tokens on very wide layers, 16: those tiles each cut along K into
 * split_k pieces -- 65 to 128 tokens on narrower layers; 17, forced only: 13 with the
 * tail cut into 256 runs that cross tile borders), s = the number of K splits
 * (for 13, 16, 17: the number of runs in all; for 14: of half tiles; 500 more
 * when the streaming kernel read its activations in tile order).  Results are the same
 * whatever the overrides.
 */
flexq_status flexq_dev_linear(const flexq_dev_tuning *tuning, int act_bits, const void *packed,
                              int group, const int8_t *xq, const uint16_t *sx,
                              const uint16_t *x_fp16, const uint16_t *sxg, int sxg_stride,
                              int M, int N, int K, uint16_t *y, int32_t *acc_out,
                              void *workspace, size_t workspace_bytes, void *stream,
                              int *dispatched);

/*
 * Measurement helpers (no arithmetic of the method): the ceilings a roofline
 * fraction can be read against on the machine at hand.
 *
 * flexq_dev_probe_hbm_read: a kernel that only reads `bytes` bytes at `src` (dev,
 * 16-byte aligned) with 16-byte loads, 12 KiB in flight per wavefront.  bytes /
 * its duration is the read bandwidth a streaming kernel can reach at that size.
 *
 * flexq_dev_probe_mfma_i8: `workgroups` workgroups of four wavefronts each issue
 * iters * 16 independent v_mfma_i32_32x32x32_i8 on operands held in registers,
 * taken from the first 16 KiB at a_operands (int8 activation codes) and
 * b_operands (packed weight bytes, low two bits cleared as the kernels do).
 * 2 * 32768 * 16 * iters * 4 * workgroups / its duration is the int8 rate the
 * matrix pipe sustains on such data.
 *
 * flexq_dev_probe_mfma_mix: the same pipe beside the other work of a GEMM
 * wavefront.  `workgroups` workgroups of `waves` (4 or 8: one or two per SIMD)
 * wavefronts each issue iters * 8 MFMAs (iters even), every one followed by
 * valu_per_mfma vector operations whose results feed later MFMAs (the shape of the
 * weight expansion), with lds_reads_per_8 16-byte LDS reads per eight MFMAs whose
 * data the next eight consume; no global loads, no barriers.  Built combinations
 * (valu_per_mfma, lds_reads_per_8): (0,0) (2,0) (3,0) (4,0) (6,0) (8,0) (0,4) (3,4)
 * (3,8); others -> FLEXQ_EINVAL.  Operands from the first 16 KiB of each buffer.
 * 2 * 32768 * 8 * iters * waves * workgroups / its duration is what the chip,
 * power-limited as it is, sustains on such a stream.
 *
 * `sink` (dev, 4 bytes) is never written in practice; it keeps the work alive.
 */
flexq_status flexq_dev_probe_hbm_read(const void *src, size_t bytes, void *sink, void *stream);
flexq_status flexq_dev_probe_mfma_i8(const void *a_operands, const void *b_operands, int iters,
                                     int workgroups, void *sink, void *stream);
flexq_status flexq_dev_probe_mfma_mix(const void *a_operands, const void *b_operands, int valu_per_mfma,
                                      int lds_reads_per_8, int iters, int workgroups, int waves, void *sink,
                                      void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FLEXQ_DEV_H */
