// How the workgroups of a min-plus launch get their instances, and the view of
// read-only tables the kernels of that stage share.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "themis_internal.h"

namespace themis {

// Tables written by earlier kernels are read-only here.  Viewing them through
// the constant address space tells the compiler so (a workgroup barrier
// otherwise counts as a possible writer), which lets it fetch wave-uniform
// entries with scalar loads into SGPRs.
#define AS_CONST __attribute__((address_space(4)))

template <typename T>
__device__ __forceinline__ const AS_CONST T* as_constant(const T* p)
{
    return (const AS_CONST T*)(uintptr_t)p;
}

// Instances are handed to the workgroups of a launch from the launch's list
// (one class, or several classes one after the other).  The first rounds are
// dealt out by workgroup index (round r: entry r * gridDim.x + blockIdx.x); the
// rest are pulled one at a time through an atomic cursor, so that a workgroup
// that drew long rows takes fewer.  One round is dealt out: read-modify-writes on
// one address complete at a rate of one per some tens of nanoseconds device-wide,
// which a launch of thousands of short rows that all begin (and end) with a pull
// would be bound by, and a launch whose list is no longer than its grid never
// touches the cursor at all.  Beyond that, pulling is what keeps the workgroups
// level: the lists are ordered longest rows first, and dealing out more rounds
// of unpruned rows was slower on every workload measured.  With SHORT_LISTS_DEALT
// (the kernel for pruned rows, whose instances take a few microseconds each and
// differ less) a list of up to four rounds is dealt out entirely.
template <bool SHORT_LISTS_DEALT = false>
__device__ __forceinline__ int static_rounds(int count, int grid)
{
    return SHORT_LISTS_DEALT && count <= 4 * grid ? (count + grid - 1) / grid : 1;
}

// The list index that follows `prev` for this workgroup without a pull, or -2
// when the next one has to be pulled (-1: the list is exhausted).  `prev` is the
// workgroup's previous index (-1 before the first).
template <bool SHORT_LISTS_DEALT = false>
__device__ __forceinline__ int next_static_index(int count, int prev)
{
    const int grid = (int)gridDim.x;
    const int dealt = static_rounds<SHORT_LISTS_DEALT>(count, grid) * grid;  // entries dealt out
    if (prev < dealt) {
        const int idx = prev < 0 ? (int)blockIdx.x : prev + grid;
        if (idx < dealt) return idx < count ? idx : -1;
    }
    return dealt < count ? -2 : -1;
}

// Returns the list index of the workgroup's next instance, or -1 when the list
// is exhausted; every wavefront of the workgroup gets the same answer.
// `prev` is the previous answer (-1 before the first call).
__device__ __forceinline__ int next_index(volatile uint32_t* slot, int32_t* cursor, int count,
                                          int prev)
{
    const int dealt_idx = next_static_index(count, prev);
    if (dealt_idx != -2) return dealt_idx;
    if (threadIdx.x == 0) *slot = (uint32_t)atomicAdd(cursor, 1);
    __syncthreads();
    const int idx = (int)gridDim.x + __builtin_amdgcn_readfirstlane((int)*slot);
    __syncthreads();  // slot may be rewritten by the next call
    return idx < count ? idx : -1;
}

// The list of a launch that serves the classes cls, cls - 1, ..., low, in that
// order: the longest rows start first and the launch ends on the shortest ones.
__device__ __forceinline__ int list_length(const int32_t* ctrl, int cls, int low)
{
    int n = 0;
    for (int c = cls; c >= low; --c) n += as_constant(ctrl)[c];
    return n;
}

__device__ __forceinline__ int list_entry(const int32_t* ctrl, const int32_t* order, int N,
                                          int cls, int low, int idx)
{
    for (int c = cls; c >= low; --c) {
        const int n = as_constant(ctrl)[c];
        if (idx < n) return as_constant(order)[(size_t)c * N + idx];
        idx -= n;
    }
    return -1;
}

// Workgroup barrier that orders LDS traffic only: global stores in flight are not
// waited for (the barrier of __syncthreads() waits until they have reached L2,
// a microsecond or more per model that nothing here depends on).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace themis
