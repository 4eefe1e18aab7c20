// Wavefront-64 device helpers shared by the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adacgd {

__device__ __forceinline__ uint32_t lane_id() {
  return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}
__device__ __forceinline__ uint64_t ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
// set bits of m that belong to lanes below the caller
__device__ __forceinline__ uint32_t below(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}
__device__ __forceinline__ uint32_t popc64(uint64_t m) { return (uint32_t)__popcll(m); }

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    uint32_t w = __shfl_xor(v, o, 64);
    v = w > v ? w : v;
  }
  return v;
}

// Sum over a 256-thread block in a fixed order; result valid in every thread.
__device__ __forceinline__ double block_sum(double v, double* lds4) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = v;
  __syncthreads();
  return (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
}

// Exclusive prefix sum over the 256 threads of a block (thread order); *total gets the sum.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* lds4, uint32_t* total) {
  const uint32_t lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t t = __shfl_up(inc, o, 64);
    if (lane >= (uint32_t)o) inc += t;
  }
  __syncthreads();
  if (lane == 63) lds4[w] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (uint32_t i = 0; i < w; ++i) base += lds4[i];
  *total = lds4[0] + lds4[1] + lds4[2] + lds4[3];
  return base + inc - v;
}

// Data that one block writes and another block of the same launch reads goes through
// agent-scope atomic accesses only (relaxed atomic stores, loads and read-modify-writes):
// those are performed at the device's point of coherence, so no cache write-back or
// invalidate is needed to make them visible -- a release/acquire fence at agent scope
// would write back and invalidate the whole L2 of the XCD once per block.
template <typename T>
__device__ __forceinline__ T ld_coherent(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void st_coherent(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Every block of a node calls this once after its last coherent write.  Returns true in
// all threads of exactly one block per node: the one that arrived last.  That block may
// then read what the others wrote (with ld_coherent) and finish the node's work; the
// counters are back at zero when it returns.  No block ever waits for another.
// Ordering: each wave first waits until its own vector stores and atomics have completed
// (vmcnt reaches 0), the block barrier extends that to the whole block, and only then is
// the arrival counted.
// Arrivals are counted in two levels (kArriveFan first-level counters per node, then one
// second-level counter) because a few thousand read-modify-writes on one address -- or on
// one cache line -- take ~12 ns each, one after the other.  `counters` points at the node's
// kArriveFan + 1 counters, one per kCounterStride words (= one per 64-byte line); `block` is the
// caller's index among the nblocks blocks.
constexpr int kArriveFan = 32;
constexpr int kCounterStride = 16;

__device__ __forceinline__ bool arrive_last(uint32_t* counters, uint32_t nblocks, uint32_t block, int* lds_flag) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t sub = block % kArriveFan;
    const uint32_t nsub = (nblocks - sub + kArriveFan - 1) / kArriveFan;     // blocks sharing this counter
    const uint32_t nfan = nblocks < (uint32_t)kArriveFan ? nblocks : (uint32_t)kArriveFan;
    int last = 0;
    uint32_t prev = __hip_atomic_fetch_add(&counters[(1 + sub) * kCounterStride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (prev == nsub - 1) {
      __hip_atomic_store(&counters[(1 + sub) * kCounterStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      prev = __hip_atomic_fetch_add(&counters[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (prev == nfan - 1) {
        __hip_atomic_store(&counters[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last = 1;
      }
    }
    *lds_flag = last;
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  return *lds_flag != 0;
}

// The same for a few dozen blocks: one counter is enough.
__device__ __forceinline__ bool arrive_last_few(uint32_t* counter, uint32_t nblocks, int* lds_flag) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t prev = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = prev == nblocks - 1;
    if (last) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *lds_flag = last;
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  return *lds_flag != 0;
}

// LDS histogram increment by the lanes that call it (they may be a divergent subset).  The
// lanes that share the first active lane's bin are counted with one atomic: vectors with many
// equal magnitudes (zeros above all) would otherwise serialise up to 64 same-address atomics.
__device__ __forceinline__ void hist_add(uint32_t* hist, uint32_t bin) {
  const uint32_t first = __builtin_amdgcn_readfirstlane(bin);
  const uint64_t same = ballot(bin == first);
  if (bin != first) atomicAdd(&hist[bin], 1u);
  else if (below(same) == 0) atomicAdd(&hist[first], popc64(same));
}

__device__ __forceinline__ uint32_t fbits(float v) { return __float_as_uint(v); }
__device__ __forceinline__ uint32_t magkey(float v) { return __float_as_uint(v) & 0x7FFFFFFFu; }

}  // namespace adacgd
