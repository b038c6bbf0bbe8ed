// flexq_gemv_w6a8 for callers that cannot allocate: the workspace is a fixed array in
// this library's device image.  Host code must not use the array's name as an address
// (it is a host-side stand-in); the address on each device is looked up once with
// hipGetSymbolAddress and kept.
#include "api_internal.h"
#include "flexq_kernels.h"

#include <atomic>

namespace {

static __device__ __align__(256) unsigned char scratch[FLEXQ_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];   // per device: each GPU holds its own copy

// The address of `scratch` on the current device (null on failure).
void *scratch_on_current_device()
{
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return nullptr;
    void *p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    g_scratch_ptr[device].store(p, std::memory_order_release);   // same value from any thread
    return p;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" flexq_status flexq_gemv_w6a8_noalloc(const void *packed, int group, const int8_t *xq,
                                                const uint16_t *sx, const uint16_t *x_fp16, int M, int N,
                                                int K, uint16_t *y, int32_t *acc_out, void *stream)
{
    // every argument is checked before anything is launched (a 256-byte aligned stand-in
    // for the workspace pointer: the array's address is not needed for that)
    void *const stand_in = reinterpret_cast<void *>(uintptr_t{256});
    if (flexq_status s = flexq::linear_check(packed, group, xq, sx, x_fp16, M, N, K, y, acc_out, stand_in,
                                             ~size_t{0}, nullptr, 0);
        s != FLEXQ_OK)
        return s;
    if (flexq_workspace_bytes(M, N, K) > FLEXQ_NOALLOC_SCRATCH_BYTES) return FLEXQ_EWORKSPACE;
    void *ws = scratch_on_current_device();
    if (!ws) return FLEXQ_EHIP;
    // The array keeps the last call's contents.  The counters must start at zero; every
    // completed call leaves them so, but a call that was cut short would not: clear them
    // (a fill kernel, not a memset node, so the call can be captured in a graph).
    if (flexq::launch_fill_zero(ws, FLEXQ_WORKSPACE_COUNTER_BYTES, (hipStream_t)stream) != hipSuccess)
        return FLEXQ_EHIP;
    const flexq::Tuning automatic{};
    return flexq::linear_impl(automatic, 8, packed, group, xq, sx, x_fp16, M, N, K, y, acc_out, ws,
                              FLEXQ_NOALLOC_SCRATCH_BYTES, stream, nullptr, 0, nullptr);
}
#pragma GCC visibility pop
