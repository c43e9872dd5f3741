// Group-normalised advantages of GRPO (Shao et al. 2024), the algorithm the paper trains every
// agent with (Section 8.1): within the G samples of one prompt,
//   adv[s] = (reward[s] - mean) / (std + eps),   std = sqrt(mean of squared deviations).
// One wave per group; the lanes walk the group's member list (CSR), sums are reduced in a
// fixed butterfly order, and the mean is subtracted before squaring (two passes over a
// handful of values that stay in cache).
#include "marl_internal.h"

namespace marl {
namespace {

constexpr int kGrpoThreads = 256;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

__global__ __launch_bounds__(kGrpoThreads) void grpo_advantage_kernel(GrpoArgs a) {
  const int g = blockIdx.x * (kGrpoThreads / 64) + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (g >= a.num_groups) return;
  const int b = a.group_start[g], e = a.group_start[g + 1];
  const int n = e - b;
  if (n <= 0) return;
  float sum = 0.f;
  for (int k = b + lane; k < e; k += 64) sum += a.rewards[a.group_seqs[k]];
  const float mean = wave_sum(sum) / (float)n;
  float sq = 0.f;
  for (int k = b + lane; k < e; k += 64) {
    const float d = a.rewards[a.group_seqs[k]] - mean;
    sq = __builtin_fmaf(d, d, sq);
  }
  const float denom = sqrtf(wave_sum(sq) / (float)n) + a.eps;
  for (int k = b + lane; k < e; k += 64) {
    const int s = a.group_seqs[k];
    const float d = a.rewards[s] - mean;
    a.out[s] = d == 0.f ? 0.f : d / denom;
  }
}

}  // namespace

hipError_t launch_grpo_advantages(const GrpoArgs& a, hipStream_t st) {
  if (a.num_groups == 0) return hipSuccess;
  const int per_block = kGrpoThreads / 64;
  hipLaunchKernelGGL(grpo_advantage_kernel, dim3((a.num_groups + per_block - 1) / per_block),
                     dim3(kGrpoThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
