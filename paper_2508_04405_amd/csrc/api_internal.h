// What the C ABI in api.hip shares with the development entry points (dev_api.hip,
// built into libflexq_dev.so only): the one function behind every linear-layer call.
#pragma once
#include "../../include/flexq.h"

namespace flexq {

// Per-call overrides of the library's own kernel choice; all zero = automatic.
// The product entry points always pass all zeros.
struct Tuning {
    int kernel = 0;     // 1 = streaming kernel, 2 = tiled kernels
    int split_k = 0;    // K splits (streaming kernel, 128x128 tiles)
    int waves = 0;      // wavefronts per workgroup of the streaming kernel: 4, 8, 16
    int gemm_cfg = 0;   // tile configuration of the tiled kernels
    int ablate = 0;     // development build: one design choice of the streaming kernel undone
    int fuse = 0;       // quantize prologue inside the streaming kernel: 1 = whenever it can, 2 = never
    int tiles = 0;      // fp16 activations of up to 32 tokens quantized into tile order: 1 = always, 2 = never
    int spin = 0;       // evenly cut tiles of the 256-row kernel: polls before a piece gives up waiting; -1 = none
};

// The argument checks of linear_impl alone (host only, launches nothing).
flexq_status linear_check(const void *packed, int group, const int8_t *xq, const uint16_t *sx,
                          const uint16_t *x_fp16, int M, int N, int K, const uint16_t *y,
                          const int32_t *acc_out, const void *workspace, size_t workspace_bytes,
                          const uint16_t *sxg, int sxg_stride);

// act_bits 6 or 8.  sxg non-null: group-wise activation scales (group must be 128).
// *dispatched (may be null) receives 1000 * c + s: c = 1 for the streaming kernel, else
// the tile configuration that ran; s = its K splits (for the forms that cut their last
// round of tiles: the number of pieces).
flexq_status linear_impl(const Tuning &tune, int act_bits, const void *packed, int group,
                         const int8_t *xq, const uint16_t *sx, const uint16_t *x_fp16, int M, int N, int K,
                         uint16_t *y, int32_t *acc_out, void *workspace, size_t workspace_bytes,
                         void *stream, const uint16_t *sxg, int sxg_stride, int *dispatched, int xt = 0);
// xt = act_bits: `xq` holds the activations in tile order (flexq_quant_act_tiles), M <= 32.

// True where linear_impl, given fp16 activations, quantizes them into tile order: a caller
// that runs a fused producer itself makes it write tiles then, and passes xt.
bool linear_wants_tiles(int act_bits, int M, int N, int K, int group);

}  // namespace flexq
