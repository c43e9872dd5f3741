// Wave-level building blocks shared by the attention kernels (gfx950, wave64): the
// 16x16x32 bf16 MFMA wrapper, bf16 packing, reductions over the four lanes that share a query
// row, and the flavours of global loads the kernels use.
#ifndef MARL_WAVE_OPS_H
#define MARL_WAVE_OPS_H
#include <type_traits>

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

// Reductions over the 64 lanes, result in every lane, inside the vector ALU: four DPP steps
// all-reduce each row of 16 lanes (swap neighbours, swap pairs, mirror the halves of 8, mirror
// the row), two row swaps combine the four rows.  (A shuffle-based reduction keeps six
// lane-address registers alive and goes through the LDS crossbar six times per call, each a
// dependent round trip.)
template <class T, class Op>
__device__ __forceinline__ T wave_allreduce(T v, Op op) {
  static_assert(sizeof(T) == 4, "32-bit values");
  auto dpp = [](T x, auto ctrl_tag) {
    constexpr int ctrl = decltype(ctrl_tag)::value;
    return __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), ctrl, 0xf, 0xf, false));
  };
  v = op(v, dpp(v, std::integral_constant<int, 0xB1>{}));    // quad_perm [1, 0, 3, 2]
  v = op(v, dpp(v, std::integral_constant<int, 0x4E>{}));    // quad_perm [2, 3, 0, 1]
  v = op(v, dpp(v, std::integral_constant<int, 0x141>{}));   // row_half_mirror
  v = op(v, dpp(v, std::integral_constant<int, 0x140>{}));   // row_mirror
  // (the swap results are copied to scalars first: a bit cast applied directly to an element of
  // the returned vector reads element 0 for both)
  const uint32_t u = __builtin_bit_cast(uint32_t, v);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const uint32_t a0 = a[0], a1 = a[1];
  v = op(__builtin_bit_cast(T, a0), __builtin_bit_cast(T, a1));
  const uint32_t w = __builtin_bit_cast(uint32_t, v);
  const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  const uint32_t b0 = b[0], b1 = b[1];
  return op(__builtin_bit_cast(T, b0), __builtin_bit_cast(T, b1));
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
