// Shared device-side helpers: vector types of 1..16 bytes and streaming
// (non-temporal) global loads and stores for data that is touched exactly once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fastdiv.h"

namespace amoeba {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int BYTES> struct VecOf;
template <> struct VecOf<16> { using type = u32x4; };
template <> struct VecOf<8> { using type = u32x2; };
template <> struct VecOf<4> { using type = uint32_t; };
template <> struct VecOf<2> { using type = uint16_t; };
template <> struct VecOf<1> { using type = uint8_t; };

// Every buffer the library touches is device global memory; saying so in the pointer
// type keeps the accesses on the global_load/global_store path even when the address
// went through a select or a table.
#define AMOEBA_GLOBAL __attribute__((address_space(1)))

template <bool NT, typename V>
__device__ __forceinline__ V ld(const char* p) {
  const AMOEBA_GLOBAL V* g = (const AMOEBA_GLOBAL V*)(uintptr_t)p;
  if (NT) return __builtin_nontemporal_load(g);
  return *g;
}

template <bool NT, typename V>
__device__ __forceinline__ void st(char* p, V v) {
  AMOEBA_GLOBAL V* g = (AMOEBA_GLOBAL V*)(uintptr_t)p;
  if (NT)
    __builtin_nontemporal_store(v, g);
  else
    *g = v;
}

// A pointer that is the same for every lane (a kernel argument), pinned in scalar registers.
// Without this, a per-lane choice between two pointer arguments is compiled as a choice
// between their ADDRESSES in the argument block followed by a vector load of the chosen
// pointer: one more memory latency in front of every data load.
__device__ __forceinline__ const char* uniform_ptr(const char* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(v));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(v >> 32));
  return reinterpret_cast<const char*>((uint64_t(hi) << 32) | lo);
}

// XCD-aware work order.  Workgroups are dealt to the 8 XCDs (each with its own L2) round
// robin by workgroup id, so with work item = workgroup id the XCDs interleave on chunks of
// one tile.  Giving XCD x the x-th contiguous eighth of the items instead lets each XCD
// stream through one range.  Measured on a plain copy: workgroups of 2-8 wavefronts go from
// 6.1-6.5 to 6.6-6.65 TB/s; single-wavefront workgroups are best in plain order (6.7).
// Loop bound for n items: xcd_loop_bound(n); item of loop index w: xcd_item(w, n), which is
// >= n for the (at most 7) indices that have no item.
constexpr uint32_t kXcds = 8;
__device__ __forceinline__ uint32_t xcd_loop_bound(uint32_t n) { return ((n + kXcds - 1) / kXcds) * kXcds; }
__device__ __forceinline__ uint32_t xcd_item(uint32_t w, uint32_t n) {
  const uint32_t per = (n + kXcds - 1) / kXcds;
  return (w % kXcds) * per + w / kXcds;
}

constexpr int kThreads = 256;  // 4 wavefronts of 64 lanes per workgroup

// Largest power of two <= 16 that divides every value OR-ed into `bits`.
inline int common_alignment(uint64_t bits) {
  int a = 16;
  while (a > 1 && (bits & uint64_t(a - 1))) a >>= 1;
  return a;
}

}  // namespace amoeba
