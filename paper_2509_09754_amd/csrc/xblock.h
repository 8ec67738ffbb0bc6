// Exchange of small results between workgroups of one kernel without cache-wide fences.
//
// A device-scope release fence writes back the whole L2 of the issuing XCD; issued by every
// workgroup of a large grid those write-backs serialise and dominate a bandwidth kernel.  The
// helpers below avoid that: values meant for other workgroups are written with device-scope
// atomic stores (write-through), the writer waits until its own stores have completed
// (vmcnt == 0) before it takes a ticket, and readers use device-scope atomic loads, which do not
// hit in caches that are not coherent across XCDs.  Nothing else is exchanged this way.
//
// What this rests on, and the rules that keep it valid:
//  * Hardware, not the language's memory model: on gfx942 / gfx950 a device-scope atomic store goes
//    through to memory that every XCD sees, its completion is what vmcnt counts, and a device-scope
//    atomic load is served from there and not from a per-XCD cache line filled earlier.  Relaxed
//    atomics carry no ordering of their own; the order "data, then ticket" comes from drain_vmem()
//    (the writer's stores have completed before the ticket is taken) and from the reader's data
//    dependence on the ticket it has seen.
//  * Every word of a published buffer is written ONLY with st_dev* and read by other workgroups ONLY
//    with ld_dev* (or device-scope atomic adds on both sides, as for histograms).  A plain store to
//    such a buffer may sit in the writer's L2 past the ticket; a plain load may hit a stale line.
//    Published buffers in this library: the statistic partials (ent_part), the statistics partials
//    of the persistent sweep and its unit / completion words, the selection's histograms, published
//    counts, state words and head_counts of a prepared selection.
//  * Counters and tickets must be zero before the launch that uses them: they are cleared by an
//    EARLIER kernel of the same call on the same stream (the value-norm / statistics launch, the
//    selection's init kernel) or by the same kernel before a grid-wide wait that every workgroup passes;
//    never by a memset node (a caller may capture the calls in a graph).
//  * Stress test: tests/test_gpu_parity.py runs launches of over a thousand workgroups thirty times and
//    requires the bits of the first run every time.
#pragma once

#include <hip/hip_runtime.h>

namespace lava {

__device__ __forceinline__ void st_dev(unsigned int* p, unsigned int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned int ld_dev(const unsigned int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_dev(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev_f2(float2* p, float a, float b) {
  st_dev(reinterpret_cast<unsigned long long*>(p),
         (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32));
}
__device__ __forceinline__ float2 ld_dev_f2(const float2* p) {
  const unsigned long long r = ld_dev(reinterpret_cast<const unsigned long long*>(p));
  return make_float2(__uint_as_float((unsigned int)(r & 0xffffffffull)), __uint_as_float((unsigned int)(r >> 32)));
}
__device__ __forceinline__ void st_dev_f64(double* p, double v) {
  st_dev(reinterpret_cast<unsigned long long*>(p), (unsigned long long)__double_as_longlong(v));
}
__device__ __forceinline__ double ld_dev_f64(const double* p) {
  return __longlong_as_double((long long)ld_dev(reinterpret_cast<const unsigned long long*>(p)));
}

// Every vector-memory operation this lane has issued is complete once this returns.
__device__ __forceinline__ void drain_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Arrivals are counted in two levels because device-scope atomics on ONE address serialise at
// a few tens of nanoseconds each: workgroup `id` of `n` bumps the counter of its group (at most
// 64 groups of at least 16 workgroups), and the workgroup that completes a group bumps the top
// counter.  Counters are monotonic: `round` is 1 for the first use after they were zeroed.
__device__ __forceinline__ unsigned int arrive_group_size(unsigned int n) {
  const unsigned int g = (n + 63u) / 64u;
  return g < 16u ? 16u : g;
}
__device__ __forceinline__ unsigned int arrive_groups(unsigned int n) {
  const unsigned int gs = arrive_group_size(n);
  return (n + gs - 1u) / gs;
}
constexpr int kArriveWords = 1 + 64;   // top counter + group counters

// Called by one lane.  Returns the value the top counter had before this arrival's increment if this
// workgroup completed its group in this round, or 0xffffffff otherwise.
__device__ __forceinline__ unsigned int arrive_two_level(unsigned int* ctr, unsigned int n, unsigned int id,
                                                         unsigned int round) {
  const unsigned int gs = arrive_group_size(n);
  const unsigned int grp = id / gs;
  const unsigned int members = (grp + 1u) * gs <= n ? gs : n - grp * gs;
  const unsigned int t = __hip_atomic_fetch_add(&ctr[1 + grp], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (t + 1u != round * members) return 0xffffffffu;
  return __hip_atomic_fetch_add(&ctr[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Ticket of a workgroup that has published its results with st_dev.  Returns true, in every
// thread, for the workgroup that arrives last.  `ctr` holds kArriveWords zeroed words, `s_flag`
// is a word of shared memory.
__device__ __forceinline__ bool arrive_last(unsigned int* ctr, unsigned int n, unsigned int id,
                                            unsigned int* s_flag) {
  drain_vmem();
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned int t = arrive_two_level(ctr, n, id, 1u);
    *s_flag = (t != 0xffffffffu && t + 1u == arrive_groups(n)) ? 1u : 0u;
  }
  __syncthreads();
  return *s_flag != 0u;
}

}  // namespace lava
