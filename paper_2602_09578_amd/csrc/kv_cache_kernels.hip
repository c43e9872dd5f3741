// KV-cache maintenance that precedes attention in a decode iteration: appending each
// sequence's new token to its paged suffix, and copying pages when a sample is forked from
// another one.  The paper only says that rollout manages large KV caches (Section 4.1) and
// that prompts are expanded into several samples (Section 5.1); the operations are the
// plain scatter / copy stated in marl_decode.h.  Pure data movement: results are bit-exact.
#include "marl_internal.h"

namespace marl {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// One workgroup of 128 threads per sequence, looping over the KV heads: thread c stores V channel
// c (2 bytes, the layout keeps a channel's 16 slots together), threads 0..15 store the key row
// (16 bytes each).  Every thread reads the old length before the barrier; thread 0 stores the
// new one after it.
__global__ __launch_bounds__(kD) void kv_append_kernel(KvAppendArgs a) {
  const int s = blockIdx.x;
  const int c = threadIdx.x;
  const int pos = a.suffix_lens[s];
  int flag = 0;
  int page = -1;
  if (pos < 0 || pos >= a.max_sp * kPage) flag = MARL_FLAG_LEN_CLAMPED;          // no room in the table row
  else {
    page = a.suffix_table[(size_t)s * a.max_sp + (pos >> 4)];
    if ((unsigned)page >= (unsigned)a.num_pages) { flag = MARL_FLAG_BAD_PAGE; page = -1; }
  }
  if (page >= 0) {
    const int slot = pos & (kPage - 1);
    for (int kvh = 0; kvh < a.Hkv; ++kvh) {
      const size_t blk = ((size_t)page * a.Hkv + kvh) * (kPage * kD);            // elements
      const uint16_t* kn = a.k_new + ((size_t)s * a.Hkv + kvh) * kD;
      const uint16_t* vn = a.v_new + ((size_t)s * a.Hkv + kvh) * kD;
      a.v_pages[blk + (size_t)c * kPage + slot] = vn[c];
      if (c < 16)
        *reinterpret_cast<u32x4*>(a.k_pages + blk + (size_t)slot * kD + c * 8) =
            *reinterpret_cast<const u32x4*>(kn + c * 8);
    }
  }
  if (flag && c == 0 && a.flags) atomicOr(a.flags, flag);
  __syncthreads();
  if (page >= 0 && c == 0) a.suffix_lens[s] = pos + 1;
}

// dst[i] <- src[i] for whole pages (all KV heads, K and V): one workgroup per (pair, K|V)
__global__ __launch_bounds__(256) void kv_copy_pages_kernel(KvCopyArgs a) {
  const int pair = blockIdx.x >> 1;
  uint16_t* base = (blockIdx.x & 1) ? a.v_pages : a.k_pages;
  const int src = a.src[pair], dst = a.dst[pair];
  if ((unsigned)src >= (unsigned)a.num_pages || (unsigned)dst >= (unsigned)a.num_pages) {
    if (threadIdx.x == 0 && a.flags) atomicOr(a.flags, MARL_FLAG_BAD_PAGE);
    return;
  }
  if (src == dst) return;
  const size_t page_vecs = (size_t)a.Hkv * (kPage * kD * 2 / 16);
  const u32x4* sp = reinterpret_cast<const u32x4*>(base) + (size_t)src * page_vecs;
  u32x4* dp = reinterpret_cast<u32x4*>(base) + (size_t)dst * page_vecs;
  for (size_t i = threadIdx.x; i < page_vecs; i += 256) dp[i] = sp[i];
}

}  // namespace

hipError_t launch_kv_append(const KvAppendArgs& a, hipStream_t st) {
  if (a.NS == 0) return hipSuccess;
  hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)a.NS), dim3(kD), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_kv_copy_pages(const KvCopyArgs& a, hipStream_t st) {
  if (a.n == 0) return hipSuccess;
  hipLaunchKernelGGL(kv_copy_pages_kernel, dim3(2u * a.n), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
