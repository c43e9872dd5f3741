// Gathers many tensors into one contiguous buffer, or scatters such a buffer back, with one
// kernel launch: the device side of synchronising a model's weights as a single copy instead
// of one operation per parameter (the paper's Discussion, "Hardware-Aware Abstraction").
//
// The bytes are cut into chunks of MARL_PACK_CHUNK_BYTES; chunk c belongs to the table entry e
// with first_chunk[e] <= c < first_chunk[e + 1] (binary search over the table, a few dependent
// scalar loads per 256 KB moved).  A persistent grid of workgroups takes chunks c = block,
// block + grid, ...: equal pieces, so a static split is balanced and needs no counter.  A chunk
// whose two addresses are 16-byte aligned is moved with non-temporal 16-byte loads and stores:
// 1024 threads x 16 loads in flight cover a whole chunk in one round (measured on 15 GB of
// 45 MB tensors: 5.9 TB/s of read + write; 256 threads x 4 loads, eight workgroups per CU: 5.1);
// anything else byte by byte (correct, slow: tensors from an allocator and the plan's 256-byte
// offsets never take that path).
#include "marl_internal.h"
#include "wave_ops.h"

namespace marl {
namespace {

#ifndef MARL_PACK_THREADS
#define MARL_PACK_THREADS 1024
#endif
#ifndef MARL_PACK_UNROLL
#define MARL_PACK_UNROLL 16
#endif
constexpr int kPackThreads = MARL_PACK_THREADS;
constexpr int kPackUnroll = MARL_PACK_UNROLL;   // 16-byte loads per thread in flight

__global__ __launch_bounds__(kPackThreads) void pack_kernel(PackArgs a) {
  const int tid = threadIdx.x;
  for (int c = blockIdx.x; c < a.total_chunks; c += gridDim.x) {
    // last entry whose first chunk is <= c (entries of zero bytes own no chunk and are skipped)
    int lo = 0, hi = a.n - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if ((long long)a.entries[mid].first_chunk <= c) lo = mid; else hi = mid - 1;
    }
    const marl_pack_entry e = a.entries[lo];
    const uint64_t begin = (uint64_t)(c - (long long)e.first_chunk) * MARL_PACK_CHUNK_BYTES;
    if (begin >= e.bytes) continue;   // cannot happen for a table made by marl_pack_plan
    const uint64_t len = min((uint64_t)MARL_PACK_CHUNK_BYTES, e.bytes - begin);
    char* tensor = static_cast<char*>(e.ptr) + begin;
    char* slot = a.packed + e.offset + begin;
    const char* src = a.unpack ? slot : tensor;
    char* dst = a.unpack ? tensor : slot;
    if (((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) == 0) {
      const uint64_t nvec = len >> 4;
      uint64_t v = tid;
      for (; v + (kPackUnroll - 1) * kPackThreads < nvec; v += kPackUnroll * kPackThreads) {
        u32x4 r[kPackUnroll];
#pragma unroll
        for (int u = 0; u < kPackUnroll; ++u) r[u] = ld_stream(src + ((v + u * kPackThreads) << 4));
#pragma unroll
        for (int u = 0; u < kPackUnroll; ++u)
          __builtin_nontemporal_store(r[u], reinterpret_cast<u32x4*>(dst + ((v + u * kPackThreads) << 4)));
      }
      for (; v < nvec; v += kPackThreads)
        __builtin_nontemporal_store(ld_stream(src + (v << 4)), reinterpret_cast<u32x4*>(dst + (v << 4)));
      for (uint64_t b = (nvec << 4) + tid; b < len; b += kPackThreads) dst[b] = src[b];
    } else {
      for (uint64_t b = tid; b < len; b += kPackThreads) dst[b] = src[b];
    }
  }
}

}  // namespace

hipError_t launch_pack(const PackArgs& a, int grid, hipStream_t st) {
  if (a.total_chunks == 0) return hipSuccess;
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)min(grid, a.total_chunks)), dim3(kPackThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
