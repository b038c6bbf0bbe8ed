// Pieces shared by the tiled GEMM kernels: the swizzled LDS layout of an
// activation stage, counted waits on the vector-memory counter, and the
// LDS-only workgroup barrier.
#pragma once
#include <hip/hip_runtime.h>

namespace {

// swizzled byte offset of 16-byte chunk c (0..7) of row `row` in a stage
__device__ __forceinline__ int lds_off(int row, int c)
{
    return row * 128 + ((c ^ ((row >> 1) & 7)) << 4);
}

// s_waitcnt vmcnt(N): at most N of this wavefront's vector-memory loads (in
// issue order, LDS-DMA loads included) are still outstanding afterwards.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() (and any
// fence the compiler knows about) also waits for every outstanding global load
// -- LDS-DMA loads share the counter -- which would drain the prefetch pipeline
// at the end of each stage.  Here every wavefront has already waited, by count,
// for exactly the loads that must have landed; its own LDS reads are complete
// once lgkmcnt is zero.  The asm is opaque to the compiler, so no memory access
// moves across it.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace
