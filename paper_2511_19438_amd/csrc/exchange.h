// The exchange of K-slice partial sums between workgroups, shared by the three GEMM kernels.
//
// Protocol.  Every workgroup of a column tile (one per K slice) writes its fp32 partial sums to scratch, then
// counts itself in at the tile's arrival counter; the workgroup that finds the counter at split_k - 1 is the last
// one, reads all slices' partial sums, adds them in slice order and stores the result.  No workgroup ever waits
// for another (nothing spins), so the protocol cannot hang whatever the order in which workgroups are scheduled.
//
// What orders it.  In the compiler: the partial stores, the counter update and the loads of the last arriver are
// all atomic operations separated by workgroup barriers (__syncthreads carries workgroup-scope release / acquire
// fences), which no memory operation may be moved across.  In the hardware (gfx942 / gfx950, eight XCDs with one
// L2 each, coherence point = the memory side behind them):
//   1. the partial sums are agent-scope atomic stores = global_store ... sc1: written THROUGH the XCD's L2 to the
//      coherence point, never left dirty in an L2;
//   2. every wavefront executes s_waitcnt vmcnt(0) after them: the counter of outstanding memory operations
//      reaches zero only when each write-through store has been acknowledged from the coherence point, so once
//      the following barrier lets thread 0 go on, the workgroup's partial sums are visible to every XCD;
//   3. the arrival counter is an agent-scope atomic read-modify-write, executed at the coherence point, issued
//      by thread 0 after that barrier;
//   4. the last arriver's loads are agent-scope atomic loads = global_load ... sc1, which bypass its L1 and L2,
//      and are issued after the counter's return value has passed through LDS and a second barrier.
// Steps 1-4 are stronger than "relaxed" in hardware but are not what the HIP memory model promises for relaxed
// agent-scope atomics: by the letter of the model the counter update should be a RELEASE at agent scope and the
// last arriver should execute an agent-scope ACQUIRE fence.  Building with -DGPTQ_FORMAL_EXCHANGE_FENCES=1 does
// exactly that (buffer_wbl2 sc1 before the counter update in every workgroup, buffer_inv sc1 in the last
// arriver).  Measured on MI355X it makes every K-split launch 25-65 % slower (down projection 11008x4096 at
// M = 1: 8.5 -> 10.8 us, at M = 16: 10.4 -> 16.1 us; 8192x10240 at M = 1: 12.2 -> 19.9 us): each write-back
// request walks the L2 although the write-through stores left nothing to write.  The default therefore stays
// with steps 1-4; tests/test_gpu_soak.py replays thousands of K-split launches of all three kernels and compares
// every result bit for bit with the first.
#pragma once

#include <hip/hip_runtime.h>

#ifndef GPTQ_FORMAL_EXCHANGE_FENCES
#define GPTQ_FORMAL_EXCHANGE_FENCES 0
#endif

namespace gptq {

// Thread 0 of a workgroup, after s_waitcnt vmcnt(0) in every wavefront and the barrier that follows the
// workgroup's partial stores: returns the number of workgroups that had arrived before.
__device__ __forceinline__ unsigned slice_arrive(unsigned *counter)
{
#if GPTQ_FORMAL_EXCHANGE_FENCES
    return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
#else
    return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#endif
}

// Every wavefront of the last arriver, before its first load of another workgroup's partial sums.
__device__ __forceinline__ void slice_acquire()
{
#if GPTQ_FORMAL_EXCHANGE_FENCES
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
#endif
}

}  // namespace gptq
