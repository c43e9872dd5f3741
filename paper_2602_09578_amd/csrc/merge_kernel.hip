// Merge kernel: the second reduction of split-KV decode attention.  For every (sequence,
// query head) it combines the partials of the group's prefix chunks and of the sequence's
// own suffix chunks, in slot order (so the sum order never changes between runs):
//   m* = max_i m_i,  out = sum_i O_i 2^(m_i - m*) / sum_i l_i 2^(m_i - m*)
// (m in log2 units).  A row without any token gives zeros.  One wave per row.
#include "marl_internal.h"

namespace marl {
namespace {

constexpr int kMergeThreads = 256;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(AttnArgs a) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * (kMergeThreads / 64) + (threadIdx.x >> 6);
  if (row >= a.NS * a.Hq) return;
  const int s = row / a.Hq;
  const int g = a.group_of_seq[s];
  int npc = 0;
  if ((unsigned)g < (unsigned)a.NG) {
    const int P = min(max(a.prefix_lens[g], 0), a.max_pp * kPage);
    npc = (P + a.Cp - 1) / a.Cp;
  }
  const int S = min(max(a.suffix_lens[s], 0), a.max_sp * kPage);
  const int nsc = (S + a.Cs - 1) / a.Cs;
  const int n = npc + nsc;
  const int nslot = a.NCp + a.NCs;
  const float2* ml = a.partial_ml + (size_t)row * nslot;
  const float* po = a.partial_o + (size_t)row * nslot * kD;

  // pass 1: common max
  float mstar = -INFINITY;
  for (int base = 0; base < n; base += 64) {
    const int k = base + lane;
    float m = -INFINITY;
    if (k < n) m = ml[k < npc ? k : a.NCp + (k - npc)].x;
    mstar = fmaxf(mstar, wave_max(m));
  }
  // pass 2: weights, denominator and the weighted sum of partial outputs, in slot order
  float denom = 0.f;
  float2 acc = make_float2(0.f, 0.f);
  for (int base = 0; base < n; base += 64) {
    const int k = base + lane;
    float f = 0.f, lf = 0.f;
    int slot = 0;
    if (k < n) {
      slot = k < npc ? k : a.NCp + (k - npc);
      const float2 v = ml[slot];
      f = (v.x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(v.x - mstar);
      lf = v.y * f;
    }
    denom += wave_sum(lf);
    const int cnt = min(64, n - base);
    for (int t = 0; t < cnt; ++t) {
      const float ft = __shfl(f, t);
      const int st = __shfl(slot, t);
      const float2 o = *reinterpret_cast<const float2*>(po + (size_t)st * kD + 2 * lane);
      acc.x = __builtin_fmaf(o.x, ft, acc.x);
      acc.y = __builtin_fmaf(o.y, ft, acc.y);
    }
  }
  float2 r = make_float2(0.f, 0.f);
  if (n > 0 && denom > 0.f) {
    const float inv = 1.0f / denom;
    r.x = acc.x * inv;
    r.y = acc.y * inv;
  }
  if (a.out_dtype == MARL_OUT_F32) {
    *reinterpret_cast<float2*>(reinterpret_cast<float*>(a.out) + (size_t)row * kD + 2 * lane) = r;
  } else {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v = {(__bf16)r.x, (__bf16)r.y};
    *reinterpret_cast<bf16x2*>(reinterpret_cast<uint16_t*>(a.out) + (size_t)row * kD + 2 * lane) = v;
  }
}

}  // namespace

hipError_t launch_merge(const AttnArgs& a, hipStream_t st) {
  const long rows = (long)a.NS * a.Hq;
  if (rows == 0) return hipSuccess;
  const int grid = (int)((rows + kMergeThreads / 64 - 1) / (kMergeThreads / 64));
  hipLaunchKernelGGL(merge_kernel, dim3(grid), dim3(kMergeThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
