// Merge kernel: the second reduction of split-KV decode attention.  For every (sequence,
// query head) it combines the partials of the group's prefix chunks and of the sequence's
// own suffix chunks, in slot order (so the sum order never changes between runs):
//   m* = max_i m_i,  out = sum_i O_i 2^(m_i - m*) / sum_i l_i 2^(m_i - m*)
// (m in log2 units).  A row without any token gives zeros.  Rows of a sequence whose own tokens
// were a single item of the suffix kernel are not touched: that kernel has written them.
//
// The kernel is a chain of dependent loads with almost no arithmetic, so it is organised to
// keep that chain short: the plan kernel has already stored each sequence's chunk counts
// (one load instead of group id -> prefix length), half a wave handles one row with 16-byte
// loads, and the first four partials of a row (max/sum and output) are all requested before
// any of them is used.  Every lane recomputes the few scalar weights itself: no shuffles.
#include "marl_internal.h"

namespace marl {
namespace {

constexpr int kMergeThreads = 256;
constexpr int kRowsPerBlock = kMergeThreads / 32;
constexpr int kEager = 4;   // partials fetched up front
typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(AttnArgs a) {
  const int sub = threadIdx.x & 31;   // lane within the half wave: channels 4*sub .. 4*sub+3
  const int row = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 5);
  if (row >= a.NS * a.Hq) return;
  const int s = row / a.Hq;
  const int info = a.seq_chunks[s];
  const int npc = info & 0xffff, nsc = info >> 16;
  // a sequence whose own tokens are one item of the suffix kernel (more than kShortTokens tokens
  // in one chunk) was finished there
  if (nsc == 1 && min(max(a.suffix_lens[s], 0), a.max_sp * kPage) > kShortTokens) return;
  const int n = npc + nsc;
  const int nslot = a.NCp + a.NCs;
  const float2* ml = a.partial_ml + (size_t)row * nslot;
  const float* po = a.partial_o + (size_t)row * nslot * kD + 4 * sub;
  auto slot_of = [&](int k) { return k < npc ? k : a.NCp + (k - npc); };

  float2 mlk[kEager];
  f32x4 ok[kEager];
#pragma unroll
  for (int k = 0; k < kEager; ++k) {
    mlk[k] = make_float2(-INFINITY, 0.f);
    ok[k] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (k < n) {
      const int sl = slot_of(k);
      mlk[k] = ml[sl];
      ok[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(po + (size_t)sl * kD));
    }
  }
  float mstar = -INFINITY;
#pragma unroll
  for (int k = 0; k < kEager; ++k) mstar = fmaxf(mstar, mlk[k].x);
  for (int k = kEager; k < n; ++k) mstar = fmaxf(mstar, ml[slot_of(k)].x);

  float denom = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < kEager; ++k) {
    const float f = (mlk[k].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mlk[k].x - mstar);
    denom = __builtin_fmaf(mlk[k].y, f, denom);
    acc += ok[k] * f;
  }
  for (int k = kEager; k < n; ++k) {
    const int sl = slot_of(k);
    const float2 v = ml[sl];
    const f32x4 o = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(po + (size_t)sl * kD));
    const float f = (v.x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(v.x - mstar);
    denom = __builtin_fmaf(v.y, f, denom);
    acc += o * f;
  }
  f32x4 r = {0.f, 0.f, 0.f, 0.f};
  if (n > 0 && denom > 0.f) r = acc * (1.0f / denom);
  if (a.out_dtype == MARL_OUT_F32) {
    *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.out) + (size_t)row * kD + 4 * sub) = r;
  } else {
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    const bf16x4 v = {(__bf16)r[0], (__bf16)r[1], (__bf16)r[2], (__bf16)r[3]};
    *reinterpret_cast<bf16x4*>(reinterpret_cast<uint16_t*>(a.out) + (size_t)row * kD + 4 * sub) = v;
  }
}

}  // namespace

hipError_t launch_merge(const AttnArgs& a, hipStream_t st) {
  const long rows = (long)a.NS * a.Hq;
  if (rows == 0) return hipSuccess;
  const int grid = (int)((rows + kRowsPerBlock - 1) / kRowsPerBlock);
  hipLaunchKernelGGL(merge_kernel, dim3(grid), dim3(kMergeThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
