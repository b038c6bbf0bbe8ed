// Host-side launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace flexq {

// A kernel that needs more than 64 KiB of dynamic LDS must be told so once per device
// (hipFuncSetAttribute).  `done` is that kernel's bit mask of devices already served.
inline hipError_t allow_dynamic_lds(const void *kernel, int bytes, std::atomic<unsigned long long> &done)
{
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (device & 63);
    if (done.load(std::memory_order_relaxed) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_relaxed);
    return e;
}

// Compute units of the current device (cached per device; 0 if the query fails).  The
// persistent launch forms and their tile order are laid out for the MI355X's 256 CUs in
// 8 XCDs and are only used when the device really has that many.
inline int device_cu_count()
{
    static std::atomic<int> cached[64];
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return 0;
    std::atomic<int> &slot = cached[device & 63];
    int n = slot.load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
        slot.store(n, std::memory_order_relaxed);
    }
    return n;
}

// Everything a GEMM / GEMV launch needs.  Pointers are device pointers.
struct LinearArgs {
    const void *packed;      // tiles, then scales
    const uint16_t *scales;  // = packed + N*K*6/8
    const int8_t *xq;        // [M,K]; or, with xt != 0, the activations in tile order
    int xt;                  // 0; or 6 / 8: activation tiles of 3072 / 4096 bytes (streaming kernel, M <= 32)
    const uint16_t *sx;      // [M]
    int M, N, K;
    int group;               // 0 or 128
    uint16_t *y;             // [M,N]
    int32_t *acc_out;        // [M,N] or null
    unsigned *counters;      // zero on entry, zero on exit
    void *partial;           // split-K partial sums
    size_t partial_bytes;    // capacity of that area
    int split_k;             // >= 1
    const uint16_t *x_fp16;  // streaming kernel only: quantize these fp16 activations in the
    float qmax;              // kernel (31 or 127) instead of reading xq / sx; else null
    const uint16_t *sxg;     // group-wise activation scales [K/128][sxg_stride] (group-major),
    int sxg_stride;          // or null: one scale per token in sx (sxg needs group == 128)
    int ablate;              // 0, or which design choice of the streaming kernel to undo (measurement)
    int spin = 128;          // evenly cut tiles: polls of a tile's counter (a microsecond or two each) before a piece
                             // gives up waiting -- the pieces of a tile end within microseconds of each other when they
                             // are resident together; when they are not, a short bound costs the least
};

hipError_t launch_quant_w6(const float *w, int N, int K, int group, int8_t *wq, uint16_t *sw,
                           hipStream_t st);
// `layout` 0 writes the codes row-major; layout == act_bits writes them in tile order for
// the streaming kernel (tiles of 32 tokens x 128 k: 4096 bytes of int8, or 3072 bytes in
// the packed 6-bit format of the weights); K must then be a multiple of 128 and the
// buffer hold ceil(M / 32) * (K / 128) tiles.
hipError_t launch_quant_act(const uint16_t *x, int M, int K, int act_bits, int8_t *xq,
                            uint16_t *sx, hipStream_t st, int layout = 0);
hipError_t launch_untile_act(const uint8_t *xt, int act_bits, int M, int K, int8_t *xq, hipStream_t st);
// Group-wise (128 along K) activation quantizer; sxg is [K/128][stride], group-major.
hipError_t launch_quant_act_g128(const uint16_t *x, int M, int K, int act_bits, int8_t *xq,
                                 uint16_t *sxg, int stride, hipStream_t st);
hipError_t launch_pack_w6(const int8_t *wq, const uint16_t *sw, int N, int K, int group,
                          void *packed, hipStream_t st);
hipError_t launch_unpack_w6(const void *packed, int N, int K, int group, int8_t *wq, uint16_t *sw,
                            hipStream_t st);
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t st);

// Producers fused with the per-token quantizer; h_out (fp16 copy of the
// producer's output) may be null.
hipError_t launch_rmsnorm_quant(const uint16_t *x, const uint16_t *gamma, float eps, int M, int K,
                                int act_bits, int8_t *xq, uint16_t *sx, uint16_t *h_out,
                                hipStream_t st, int layout = 0);
hipError_t launch_swiglu_quant(const uint16_t *gate_up, int M, int F, int act_bits, int8_t *xq,
                               uint16_t *sx, uint16_t *h_out, hipStream_t st, int layout = 0);

// Streaming kernel, M <= 128 per launch (the caller loops over row chunks).
hipError_t launch_skinny(const LinearArgs &a, int waves, hipStream_t st);
// True if the streaming kernel can quantize fp16 activations itself for this shape.
bool skinny_can_fuse(int M, int K, int split_k);
// True if the streaming kernel stages this shape's activation slice in LDS.
bool skinny_slice_fits(int M, int K, int split_k);
// Tiled MFMA kernel for large M.
// `chosen` (may be null) receives the tile configuration that ran and, for the persistent
// 256x256 form, the number of runs its tail was cut into.
hipError_t launch_gemm(const LinearArgs &a, int cfg, hipStream_t st, int *chosen = nullptr,
                       int *tail_runs = nullptr);
// 256-row tiles with both operands through LDS: per-channel scales, no K split.  The
// tiles beyond the last whole round of 256 ("the tail") run in one of three forms:
// tail_form 0: as whole 256x256 tiles; 1: as twice as many 256x128 tiles; 2: cut along K
// into tail_wgs equal runs of 128-k stages, whose partial sums meet in the partial-sum
// area (it must hold streamk_plan().partial_bytes; with less, and on a device that is not
// 256 CUs wide, form 0 runs instead).  tail_form 3: 128x256 tiles and nothing else; 5:
// those, each cut along K into tail_wgs / tiles pieces (the area must hold
// low_cut_bytes(tail_wgs); an error, not another form, if that or the piece count does not
// fit).  Every launch is persistent: at most one workgroup per CU.
constexpr int kStreamKGrid = 256;   // workgroups of the persistent form: one per CU of an MI355X
struct StreamKPlan {
    int tiles, full_tiles, tail_tiles;   // 256x256 tiles: all, those in whole rounds, the rest
    size_t partial_bytes;                // workspace for the partial sums of the rest
};
StreamKPlan streamk_plan(int M, int N, int K);
size_t low_cut_bytes(int pieces_in_all);
int low_cut_pieces(int M, int N, int K);
// The launch form estimated to be fastest (tail never cut if !may_cut), its estimated time
// in microseconds, and, for a cut tail, the number of runs (for half tiles: their number).
struct WldsChoice {
    double us;
    int tail_form, tail_wgs;
};
WldsChoice gemm_wlds_choose(int M, int N, int K, bool may_cut);
hipError_t launch_gemm_wlds(const LinearArgs &a, int tail_form, int tail_wgs, hipStream_t st);

}  // namespace flexq
