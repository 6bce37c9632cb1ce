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

constexpr int kThreads = 256;  // 4 wavefronts of 64 lanes per workgroup

// Largest power of two <= 16 that divides every value OR-ed into `bits`.
inline int common_alignment(uint64_t bits) {
  int a = 16;
  while (a > 1 && (bits & uint64_t(a - 1))) a >>= 1;
  return a;
}

}  // namespace amoeba
