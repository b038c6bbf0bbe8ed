// Entry points of the development library (libflexq_dev.so): the linear-layer call with
// per-call overrides of the kernel choice.  Tests use it to force every kernel and tile
// shape, tables to sweep them; nothing here keeps state between calls.
#include "../../include/flexq_dev.h"
#include "api_internal.h"

#pragma GCC visibility push(default)
extern "C" {

flexq_status flexq_dev_linear(const flexq_dev_tuning *tuning, int act_bits, const void *packed, int group,
                              const int8_t *xq, const uint16_t *sx, const uint16_t *x_fp16,
                              const uint16_t *sxg, int sxg_stride, int M, int N, int K, uint16_t *y,
                              int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream,
                              int *dispatched)
{
    flexq::Tuning t;
    if (tuning) {
        // every field is checked before any is used
        if (tuning->kernel < 0 || tuning->kernel > 2 || tuning->split_k < 0 || tuning->split_k > 64 ||
            (tuning->waves != 0 && tuning->waves != 4 && tuning->waves != 8 && tuning->waves != 16) ||
            tuning->gemm_cfg < 0 || tuning->gemm_cfg > 32 || tuning->ablate < 0 || tuning->ablate > 4 ||
            tuning->fuse < 0 || tuning->fuse > 2 || tuning->tiles < 0 || tuning->tiles > 2 ||
            tuning->spin < -1 || tuning->spin > (1 << 20))
            return FLEXQ_EINVAL;
        t.kernel = tuning->kernel;
        t.split_k = tuning->split_k;
        t.waves = tuning->waves;
        t.gemm_cfg = tuning->gemm_cfg;
        t.ablate = tuning->ablate;
        t.fuse = tuning->fuse;
        t.tiles = tuning->tiles;
        t.spin = tuning->spin;
    }
    if (act_bits != 6 && act_bits != 8) return FLEXQ_EINVAL;
    if (sxg && group != 128) return FLEXQ_EINVAL;
    return flexq::linear_impl(t, act_bits, packed, group, xq, sx, x_fp16, M, N, K, y, acc_out, workspace,
                              workspace_bytes, stream, sxg, sxg_stride, dispatched);
}

}  // extern "C"
#pragma GCC visibility pop
