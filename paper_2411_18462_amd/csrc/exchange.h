// Exchange of partial results between the workgroups of ONE kernel launch on gfx950, without a
// release fence.
//
// A row (or a sequence) is cut into slices, one workgroup per slice; the workgroup that finishes last
// combines the slices' results and does the row's remaining work, so a call needs no second kernel
// for it.  "Last" is decided by a ticket: every workgroup publishes its partial result, then adds 1 to
// the row's counter; whoever draws the final ticket knows that all other results are in memory.
//
// The L2 caches of the eight XCDs are not coherent with each other, so a device-scope release fence
// (__threadfence) writes back the whole L2 of the issuing XCD and invalidates it.  That costs about
// 0.3 us per fence and the fences of one XCD run one after another: a thousand workgroups that each
// fence once turn a 6 us kernel into a 47 us kernel.  The exchange here never puts anything into the
// L2 that another XCD needs:
//   publish_*    device-scope relaxed atomic stores: written through to memory (global_store ... sc1)
//   stores_done  s_waitcnt vmcnt(0): the stores above have been acknowledged by memory
//   take_ticket  device-scope relaxed atomic add on the counter, executed at memory
//   fetch_*      device-scope relaxed atomic loads (global_load ... sc1): served by memory, not by an
//                L2 line that may be stale
// Only the thread that published may take the ticket (program order + stores_done is what orders the
// two), and only data written through publish_* may be read by the last workgroup.  Nothing waits or
// spins: every workgroup runs to its end whatever the others do.  The last workgroup puts the counter
// back to zero, so counters only have to be cleared once, when the workspace is created.
#pragma once
#include <hip/hip_runtime.h>

namespace svip {

__device__ __forceinline__ void publish_u64(void *p, unsigned long long v)
{
    __hip_atomic_store(static_cast<unsigned long long *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_f64(double *p, double v) { publish_u64(p, (unsigned long long)__double_as_longlong(v)); }
__device__ __forceinline__ unsigned long long fetch_u64(const void *p)
{
    return __hip_atomic_load(static_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double fetch_f64(const double *p) { return __longlong_as_double((long long)fetch_u64(p)); }

__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Ticket of the calling workgroup, 0 .. arrivals - 1 in order of arrival.
__device__ __forceinline__ unsigned take_ticket(unsigned *counter)
{
    return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void reset_tickets(unsigned *counter)
{
    __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace svip
