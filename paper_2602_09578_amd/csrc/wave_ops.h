// Wave-level building blocks shared by the attention kernels (gfx950, wave64): the
// 16x16x32 bf16 MFMA wrapper, bf16 packing, reductions over the four lanes that share a query
// row, and the flavours of global loads the kernels use.
#ifndef MARL_WAVE_OPS_H
#define MARL_WAVE_OPS_H
#include "marl_internal.h"

namespace marl {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma_16x16x32(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

// All-reduce over the four lanes l, l^16, l^32, l^48 (the lanes that share a q-row) with the
// gfx950 row-swap instructions, which stay in the vector ALU (a shuffle through the LDS
// crossbar costs a round trip in the middle of the softmax dependency chain).
// permlane16_swap(x, x) yields (rows 0,0,2,2 ; rows 1,1,3,3) of x; permlane32_swap(x, x)
// yields (rows 0,1,0,1 ; rows 2,3,2,3).
__device__ __forceinline__ float rows_allreduce_max(float x) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_allreduce_sum(float x) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Wave-uniform read of read-only input through the scalar cache.
__device__ __forceinline__ int ld_uniform(const int32_t* p) {
  return *reinterpret_cast<const int32_t __attribute__((address_space(4)))*>(
      reinterpret_cast<uintptr_t>(p));
}

// 16-byte load of KV data, which is read once: the non-temporal hint keeps it from
// displacing reusable lines (block tables, queries, partials) in the caches.
#ifndef MARL_NT_LOADS
#define MARL_NT_LOADS 1
#endif
__device__ __forceinline__ u32x4 ld_stream(const char* p) {
#if MARL_NT_LOADS
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
#else
  return *reinterpret_cast<const u32x4*>(p);
#endif
}
// K rows are fetched as 16 x 64 B per instruction, so every 128-byte line is touched by two
// consecutive instructions: K uses ordinary (cached) loads so that the second touch hits the
// vector cache; measured on a load-only replica of this pattern: 6.3 TB/s with non-temporal K,
// 6.9 TB/s with cached K and non-temporal V.
#ifndef MARL_NT_K
#define MARL_NT_K 0
#endif
__device__ __forceinline__ u32x4 ld_stream_k(const char* p) {
#if MARL_NT_K
  return ld_stream(p);
#else
  return *reinterpret_cast<const u32x4*>(p);
#endif
}

}  // namespace marl
#endif  // MARL_WAVE_OPS_H
