// Plan kernel: builds, on the device, the group -> sequences CSR and the two work lists of
// one decode-attention call, so that sequence lengths never travel to the host.
//
// Why a work list at all: rollout load is heavily skewed across agents (the paper's
// Observation #2, Section 2.2) and response lengths have a long tail (Observation #1), so
// work is cut into token-sized items and listed longest first; the attention kernels then
// pull items from the list in order.  The rule is the one documented in marl_decode.h.
//
// One workgroup of 1024 threads; all of it is integer work.  Item order inside one cost
// class depends on atomics and may differ between runs; it only decides which workgroup
// processes an item, never a numerical result (every item owns its partial slot).
#include "marl_internal.h"

namespace marl {
namespace {

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// Read of a value another thread of this kernel wrote to global memory: bypasses the
// per-CU vector cache, which may still hold the line from before the write.
__device__ __forceinline__ int ld_agent(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ int wave_inclusive_scan(int v) {
  const int lane = lane_id();
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(v, d);
    if (lane >= d) v += t;
  }
  return v;
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

// out[i] = sum of in[0..i) for i < n (in and out may alias); returns the total to every
// thread.  tmp: 17 shared ints.  Must be called by all 1024 threads.  GLOBAL_IN: `in` is
// global memory written earlier in this kernel.
template <bool GLOBAL_IN>
__device__ int block_exclusive_scan(const int* in, int* out, int n, int* tmp) {
  int carry = 0;
  for (int base = 0; base < n; base += kPlanThreads) {
    const int i = base + threadIdx.x;
    const int v = i < n ? (GLOBAL_IN ? ld_agent(in + i) : in[i]) : 0;
    const int inc = wave_inclusive_scan(v);
    if (lane_id() == 63) tmp[wave_id()] = inc;
    __syncthreads();
    if (wave_id() == 0) {
      const int t = lane_id() < 16 ? tmp[lane_id()] : 0;
      const int ti = wave_inclusive_scan(t);
      if (lane_id() < 16) tmp[lane_id()] = ti - t;
      if (lane_id() == 15) tmp[16] = ti;
    }
    __syncthreads();
    if (i < n) out[i] = carry + tmp[wave_id()] + inc - v;
    carry += tmp[16];
    __syncthreads();
  }
  return carry;
}

__device__ __forceinline__ int clamp_len(int v, int hi, int& flags) {
  const int c = min(max(v, 0), hi);
  if (c != v) flags |= MARL_FLAG_LEN_CLAMPED;
  return c;
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(AttnArgs a) {
  __shared__ int hist_s[kNumClasses];
  __shared__ int hist_p[kNumClasses];
  __shared__ int tmp[17];
  __shared__ int n_long_items, n_short_partial_items;
  const int tid = threadIdx.x;
  const int Cs = a.Cs, Cp = a.Cp, R = a.R, QB = a.qblock_rows;
  const int ncls_s = Cs / 32, ncls_p = Cp / 32;
  const int max_st = a.max_sp * kPage, max_pt = a.max_pp * kPage;
  int flags = 0;

  for (int i = tid; i < kNumClasses; i += kPlanThreads) { hist_s[i] = 0; hist_p[i] = 0; }
  for (int g = tid; g < a.NG; g += kPlanThreads) a.group_count[g] = 0;
  if (tid < 64) a.counters[tid] = 0;
  if (tid == 0) { n_long_items = 0; n_short_partial_items = 0; }
  __threadfence();
  __syncthreads();

  // sequences: rank inside the group, histogram of suffix items by cost class
  // (full chunks and long items: counted per thread, added once per wave, since same-address LDS
  // atomics run one lane at a time)
  int nfull_mine = 0, nlong_mine = 0, nshort_partial_mine = 0;
  for (int s = tid; s < a.NS; s += kPlanThreads) {
    const int g = a.group_of_seq[s];
    int rank = -1;
    if ((unsigned)g < (unsigned)a.NG) rank = atomicAdd(&a.group_count[g], 1);
    else flags |= MARL_FLAG_BAD_GROUP;
    a.seq_rank[s] = rank;
    const int S = clamp_len(a.suffix_lens[s], max_st, flags);
    const int nfull = S / Cs, tail = S % Cs;
    nfull_mine += nfull;
    if (tail) atomicAdd(&hist_s[(Cs - tail) / 32], 1);
    nlong_mine += (Cs > kShortTokens ? nfull : 0) + (tail > kShortTokens ? 1 : 0);
    // short items (at most kShortTokens tokens) of sequences with several suffix chunks: they become partials
    if (nfull + (tail > 0) >= 2)
      nshort_partial_mine += (Cs <= kShortTokens ? nfull : 0) + ((tail > 0 && tail <= kShortTokens) ? 1 : 0);
  }
  nfull_mine = wave_sum(nfull_mine);
  nlong_mine = wave_sum(nlong_mine);
  nshort_partial_mine = wave_sum(nshort_partial_mine);
  if (lane_id() == 0) {
    if (nfull_mine) atomicAdd(&hist_s[0], nfull_mine);
    if (nlong_mine) atomicAdd(&n_long_items, nlong_mine);
    if (nshort_partial_mine) atomicAdd(&n_short_partial_items, nshort_partial_mine);
  }
  __threadfence();
  __syncthreads();

  // CSR offsets
  const int nseq_grouped = block_exclusive_scan<true>(a.group_count, a.group_start, a.NG, tmp);
  if (tid == 0) a.group_start[a.NG] = nseq_grouped;

  // groups: histogram of prefix items (one per chunk and per block of query rows)
  for (int g = tid; g < a.NG; g += kPlanThreads) {
    const int P = clamp_len(a.prefix_lens[g], max_pt, flags);
    const int nqb = (ld_agent(a.group_count + g) * R + QB - 1) / QB;
    const int nfull = P / Cp, tail = P % Cp;
    if (nqb) {
      if (nfull) atomicAdd(&hist_p[0], nfull * nqb);
      if (tail) atomicAdd(&hist_p[(Cp - tail) / 32], nqb);
    }
  }
  __threadfence();
  __syncthreads();

  // class start offsets; afterwards the histograms serve as per-class cursors
  const int n_suffix_items = block_exclusive_scan<false>(hist_s, hist_s, ncls_s, tmp);
  const int n_prefix_items = block_exclusive_scan<false>(hist_p, hist_p, ncls_p, tmp);

  for (int s = tid; s < a.NS; s += kPlanThreads) {
    // members of a group in arrival order first; put into ascending order further down
    const int rank = a.seq_rank[s];
    if (rank >= 0) a.group_tmp[ld_agent(a.group_start + a.group_of_seq[s]) + rank] = s;
    int dummy = 0;
    const int S = clamp_len(a.suffix_lens[s], max_st, dummy);
    const int P = rank >= 0 ? clamp_len(a.prefix_lens[a.group_of_seq[s]], max_pt, dummy) : 0;
    a.seq_chunks[s] = ((P + Cp - 1) / Cp) | (((S + Cs - 1) / Cs) << 16);
    const int nfull = S / Cs, tail = S % Cs;
    if (nfull) {
      const int pos = atomicAdd(&hist_s[0], nfull);
      for (int i = 0; i < nfull; ++i) a.suffix_items[pos + i] = make_int4(s, i * Cs, (i + 1) * Cs, 0);
    }
    if (tail) {
      const int pos = atomicAdd(&hist_s[(Cs - tail) / 32], 1);
      a.suffix_items[pos] = make_int4(s, nfull * Cs, S, 0);
    }
  }
  for (int g = tid; g < a.NG; g += kPlanThreads) {
    int dummy = 0;
    const int P = clamp_len(a.prefix_lens[g], max_pt, dummy);
    const int nqb = (ld_agent(a.group_count + g) * R + QB - 1) / QB;
    const int nfull = P / Cp, tail = P % Cp;
    if (nqb) {
      if (nfull) {
        const int pos = atomicAdd(&hist_p[0], nfull * nqb);
        for (int i = 0; i < nfull; ++i)
          for (int b = 0; b < nqb; ++b)
            a.prefix_items[pos + i * nqb + b] = make_int4(g, i * Cp, (i + 1) * Cp, b * QB);
      }
      if (tail) {
        const int pos = atomicAdd(&hist_p[(Cp - tail) / 32], nqb);
        for (int b = 0; b < nqb; ++b)
          a.prefix_items[pos + b] = make_int4(g, nfull * Cp, P, b * QB);
      }
    }
  }
  __threadfence();
  __syncthreads();

  // make the CSR order deterministic: inside every group of at most 64 sequences a member's
  // final place is the number of members with a smaller id (larger groups keep arrival
  // order; the order of rows never changes a result)
  for (int s = tid; s < a.NS; s += kPlanThreads) {
    const int rank = a.seq_rank[s];
    if (rank < 0) continue;
    const int g = a.group_of_seq[s];
    const int b = ld_agent(a.group_start + g), n = ld_agent(a.group_count + g);
    int place = rank;
    if (n <= 64) {
      place = 0;
      for (int k0 = 0; k0 < n; k0 += 8) {
        int v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (k0 + u < n) ? ld_agent(a.group_tmp + b + k0 + u) : 0x7fffffff;
#pragma unroll
        for (int u = 0; u < 8; ++u) place += v[u] < s;
      }
    }
    a.group_seqs[b + place] = s;
  }
  if (flags) atomicOr(&a.counters[MARL_CTR_FLAGS], flags);
  if (tid == 0) {
    a.counters[MARL_CTR_NUM_SUFFIX_ITEMS] = n_suffix_items;
    a.counters[MARL_CTR_NUM_PREFIX_ITEMS] = n_prefix_items;
    a.counters[MARL_CTR_NUM_LONG_SUFFIX_ITEMS] = n_long_items;
    a.counters[MARL_CTR_NUM_SHORT_PARTIAL_ITEMS] = n_short_partial_items;
  }
}

// ---------------------------------------------------------------------------------------
// Same plan for shapes whose bookkeeping fits in LDS (NS <= 8192, NG <= 2048, chunks <= 8192
// tokens): inputs are read once into registers, counts, offsets, member lists and histograms
// live in LDS, and global memory only sees the final stores.  The general kernel above pays
// a chain of ~30 dependent global round trips; this one pays one.
// ---------------------------------------------------------------------------------------
// Two sizes: up to 8192 sequences in 2048 groups (56 KB of LDS), and up to 32768 sequences in
// 8192 groups with 16-bit member ids (130 KB of the 160 KB).
constexpr int kSmallMaxClasses = 256;

template <int kSmallMaxSeqs, int kSmallMaxGroups, class MemberId>
__device__ __forceinline__ void plan_in_lds(const AttnArgs& a) {
  constexpr int kSeqsPerThread = kSmallMaxSeqs / kPlanThreads;
  constexpr int kGroupsPerThread = kSmallMaxGroups / kPlanThreads;
  __shared__ int cnt[kSmallMaxGroups];
  __shared__ int start[kSmallMaxGroups + 1];
  __shared__ MemberId members[kSmallMaxSeqs];
  __shared__ int hist_s[kSmallMaxClasses];
  __shared__ int hist_p[kSmallMaxClasses];
  __shared__ int tmp[17];
  __shared__ int n_long_items, n_short_partial_items;
  // clamped prefix lengths, where there is room for them (else they are re-read from global memory)
  constexpr bool kPrefixLensInLds = kSmallMaxGroups <= 2048;
  __shared__ int prefix_len[kPrefixLensInLds ? kSmallMaxGroups : 1];
  const int tid = threadIdx.x;
  const int Cs = a.Cs, Cp = a.Cp, R = a.R, QB = a.qblock_rows;
  const int ncls_s = Cs / 32, ncls_p = Cp / 32;
  const int max_st = a.max_sp * kPage, max_pt = a.max_pp * kPage;
  int flags = 0;

  // inputs -> registers (the only loads from global memory).  The larger size has no room for
  // 3 x 32 values per thread: it keeps only the ranks and re-reads group ids and lengths (cache
  // hits) in the later phases.
  constexpr bool kKeep = kSeqsPerThread <= 8;
  int g_keep[kKeep ? kSeqsPerThread : 1], S_keep[kKeep ? kSeqsPerThread : 1], rank_of[kSeqsPerThread];
  if constexpr (kKeep) {
#pragma unroll
    for (int k = 0; k < kSeqsPerThread; ++k) {
      const int s = tid + k * kPlanThreads;
      g_keep[k] = s < a.NS ? a.group_of_seq[s] : -1;
      S_keep[k] = s < a.NS ? a.suffix_lens[s] : 0;
    }
  }
  int ignored = 0;
  auto G = [&](int k) {   // group id of this thread's k-th sequence (only called for s < NS)
    if constexpr (kKeep) return g_keep[k]; else return a.group_of_seq[tid + k * kPlanThreads];
  };
  auto S_len = [&](int k) {   // its clamped suffix length
    if constexpr (kKeep) return S_keep[k]; else return clamp_len(a.suffix_lens[tid + k * kPlanThreads], max_st, ignored);
  };
  int P_of[kGroupsPerThread];
#pragma unroll
  for (int k = 0; k < kGroupsPerThread; ++k) {
    const int g = tid + k * kPlanThreads;
    P_of[k] = g < a.NG ? a.prefix_lens[g] : 0;
  }
  for (int i = tid; i < kSmallMaxGroups; i += kPlanThreads) cnt[i] = 0;
  for (int i = tid; i < kSmallMaxClasses; i += kPlanThreads) { hist_s[i] = 0; hist_p[i] = 0; }
  if (tid == 0) { n_long_items = 0; n_short_partial_items = 0; }
  if (tid < 64) a.counters[tid] = 0;
  __syncthreads();

  // full chunks and long items are counted per thread and added once per wave: nearly every
  // sequence contributes to these two words, and same-address LDS atomics run one lane at a time
  int nfull_mine = 0, nlong_mine = 0, nshort_partial_mine = 0;
#pragma unroll
  for (int k = 0; k < kSeqsPerThread; ++k) {
    const int s = tid + k * kPlanThreads;
    rank_of[k] = -1;
    if (s < a.NS) {
      const int g = G(k);
      if ((unsigned)g < (unsigned)a.NG) rank_of[k] = atomicAdd(&cnt[g], 1);
      else flags |= MARL_FLAG_BAD_GROUP;
      int S;
      if constexpr (kKeep) S = S_keep[k] = clamp_len(S_keep[k], max_st, flags);
      else S = clamp_len(a.suffix_lens[s], max_st, flags);
      const int nfull = S / Cs, tail = S % Cs;
      nfull_mine += nfull;
      if (tail) atomicAdd(&hist_s[(Cs - tail) / 32], 1);
      nlong_mine += (Cs > kShortTokens ? nfull : 0) + (tail > kShortTokens ? 1 : 0);
    // short items (at most kShortTokens tokens) of sequences with several suffix chunks: they become partials
    if (nfull + (tail > 0) >= 2)
      nshort_partial_mine += (Cs <= kShortTokens ? nfull : 0) + ((tail > 0 && tail <= kShortTokens) ? 1 : 0);
    }
  }
  nfull_mine = wave_sum(nfull_mine);
  nlong_mine = wave_sum(nlong_mine);
  nshort_partial_mine = wave_sum(nshort_partial_mine);
  if (lane_id() == 0) {
    if (nfull_mine) atomicAdd(&hist_s[0], nfull_mine);
    if (nlong_mine) atomicAdd(&n_long_items, nlong_mine);
    if (nshort_partial_mine) atomicAdd(&n_short_partial_items, nshort_partial_mine);
  }
  __syncthreads();
  const int nseq_grouped = block_exclusive_scan<false>(cnt, start, a.NG, tmp);
  if (tid == 0) start[a.NG] = nseq_grouped;

#pragma unroll
  for (int k = 0; k < kGroupsPerThread; ++k) {
    const int g = tid + k * kPlanThreads;
    if (g < a.NG) {
      P_of[k] = clamp_len(P_of[k], max_pt, flags);
      if constexpr (kPrefixLensInLds) prefix_len[g] = P_of[k];
      const int nqb = (cnt[g] * R + QB - 1) / QB;
      const int nfull = P_of[k] / Cp, tail = P_of[k] % Cp;
      if (nqb) {
        if (nfull) atomicAdd(&hist_p[0], nfull * nqb);
        if (tail) atomicAdd(&hist_p[(Cp - tail) / 32], nqb);
      }
    }
  }
  __syncthreads();
  const int n_suffix_items = block_exclusive_scan<false>(hist_s, hist_s, ncls_s, tmp);
  const int n_prefix_items = block_exclusive_scan<false>(hist_p, hist_p, ncls_p, tmp);

#pragma unroll
  for (int k = 0; k < kSeqsPerThread; ++k) {
    const int s = tid + k * kPlanThreads;
    if (s < a.NS) {
      const int g = G(k);
      if (rank_of[k] >= 0) members[start[g] + rank_of[k]] = (MemberId)s;
      const int S = S_len(k);
      int P = 0;
      if (rank_of[k] >= 0) {
        int dummy = 0;
        if constexpr (kPrefixLensInLds) P = prefix_len[g];
        else P = clamp_len(a.prefix_lens[g], max_pt, dummy);
      }
      a.seq_chunks[s] = ((P + Cp - 1) / Cp) | (((S + Cs - 1) / Cs) << 16);
      const int nfull = S / Cs, tail = S % Cs;
      if (nfull) {
        const int pos = atomicAdd(&hist_s[0], nfull);
        for (int i = 0; i < nfull; ++i) a.suffix_items[pos + i] = make_int4(s, i * Cs, (i + 1) * Cs, 0);
      }
      if (tail) {
        const int pos = atomicAdd(&hist_s[(Cs - tail) / 32], 1);
        a.suffix_items[pos] = make_int4(s, nfull * Cs, S, 0);
      }
    }
  }
#pragma unroll
  for (int k = 0; k < kGroupsPerThread; ++k) {
    const int g = tid + k * kPlanThreads;
    if (g < a.NG) {
      a.group_count[g] = cnt[g];
      a.group_start[g] = start[g];
      const int P = P_of[k];
      const int nqb = (cnt[g] * R + QB - 1) / QB;
      const int nfull = P / Cp, tail = P % Cp;
      if (nqb) {
        if (nfull) {
          const int pos = atomicAdd(&hist_p[0], nfull * nqb);
          for (int i = 0; i < nfull; ++i)
            for (int b = 0; b < nqb; ++b)
              a.prefix_items[pos + i * nqb + b] = make_int4(g, i * Cp, (i + 1) * Cp, b * QB);
        }
        if (tail) {
          const int pos = atomicAdd(&hist_p[(Cp - tail) / 32], nqb);
          for (int b = 0; b < nqb; ++b)
            a.prefix_items[pos + b] = make_int4(g, nfull * Cp, P, b * QB);
        }
      }
    }
  }
  if (tid == 0) a.group_start[a.NG] = nseq_grouped;
  __syncthreads();

  // ascending sequence id inside every group of at most 64 members (as in the general kernel)
#pragma unroll
  for (int k = 0; k < kSeqsPerThread; ++k) {
    const int s = tid + k * kPlanThreads;
    if (s < a.NS && rank_of[k] >= 0) {
      const int g = G(k);
      const int b = start[g], n = cnt[g];
      int place = rank_of[k];
      if (n <= 64) {
        place = 0;
        for (int m = 0; m < n; ++m) place += (int)members[b + m] < s;
      }
      a.group_seqs[b + place] = s;
    }
  }
  if (flags) atomicOr(&a.counters[MARL_CTR_FLAGS], flags);
  if (tid == 0) {
    a.counters[MARL_CTR_NUM_SUFFIX_ITEMS] = n_suffix_items;
    a.counters[MARL_CTR_NUM_PREFIX_ITEMS] = n_prefix_items;
    a.counters[MARL_CTR_NUM_LONG_SUFFIX_ITEMS] = n_long_items;
    a.counters[MARL_CTR_NUM_SHORT_PARTIAL_ITEMS] = n_short_partial_items;
  }
}

constexpr int kSmallMaxSeqs = 8192, kSmallMaxGroups = 2048;
constexpr int kMediumMaxSeqs = 32768, kMediumMaxGroups = 8192;
__global__ __launch_bounds__(kPlanThreads) void plan_kernel_small(AttnArgs a) {
  plan_in_lds<kSmallMaxSeqs, kSmallMaxGroups, int>(a);
}
__global__ __launch_bounds__(kPlanThreads) void plan_kernel_medium(AttnArgs a) {
  plan_in_lds<kMediumMaxSeqs, kMediumMaxGroups, uint16_t>(a);
}

}  // namespace

hipError_t launch_plan(const AttnArgs& a, hipStream_t st) {
  const bool classes_fit = a.Cs / 32 <= kSmallMaxClasses && a.Cp / 32 <= kSmallMaxClasses;
  if (classes_fit && a.NS <= kSmallMaxSeqs && a.NG <= kSmallMaxGroups)
    hipLaunchKernelGGL(plan_kernel_small, dim3(1), dim3(kPlanThreads), 0, st, a);
  else if (classes_fit && a.NS <= kMediumMaxSeqs && a.NG <= kMediumMaxGroups)
    hipLaunchKernelGGL(plan_kernel_medium, dim3(1), dim3(kPlanThreads), 0, st, a);
  else
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
