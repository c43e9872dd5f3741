// Per-token log-probability: out[r] = x[r, tok_r]/T - log sum_v exp(x[r, v]/T), the quantity
// GRPO training (which the paper uses, Section 8.1) consumes for every generated token.
// One streaming pass over the row's bf16 logits with a running (max, sum of exponentials)
// per lane, in base-2 units: y = x * log2(e)/T.  Lanes are combined inside the vector ALU (DPP
// row operations and the row-swap instructions), waves through LDS.  A row is cut into `slices` vocabulary slices when there are too few rows to
// fill the GPU; a small second kernel then combines the slices.
#include "marl_internal.h"
#include "wave_ops.h"

namespace marl {
namespace {

// 1024 threads: 2 workgroups per CU; measured 3-4 % faster than 8 workgroups of 256 on 2048 and on
// 16384 rows of 152064 logits
constexpr int kLpThreads = 1024;
constexpr int kUnroll = 4;

struct MaxSum {
  float m, s;
};

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

// exp2(a - b) that is 0 (not NaN) when a is -inf, whatever b is
__device__ __forceinline__ float ex2_diff(float a, float b) {
  return ex2(a - (b == -INFINITY ? 0.f : b));
}

__device__ __forceinline__ MaxSum combine(MaxSum a, MaxSum b) {
  const float m = fmaxf(a.m, b.m);
  return MaxSum{m, a.s * ex2_diff(a.m, m) + b.s * ex2_diff(b.m, m)};
}

__device__ __forceinline__ void add_one(MaxSum& st, float y) {
  const float m = fmaxf(st.m, y);
  st.s = st.s * ex2_diff(st.m, m) + ex2_diff(y, m);
  st.m = m;
}

// c > 0 (it is log2(e) / T), so the max of the scaled values is the scaled max of the raw ones:
// the scale is applied once to the max and folded into the exponent's fma for the rest.
__device__ __forceinline__ void add_vec(MaxSum& st, u32x4 v, float c) {
  float x[8];
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    x[2 * d] = __uint_as_float(v[d] << 16);
    x[2 * d + 1] = __uint_as_float(v[d] & 0xffff0000u);
  }
  const float x8 = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
  const float m = fmaxf(st.m, x8 * c);
  const float ms = (m == -INFINITY) ? 0.f : m;
  float sum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) sum += ex2(__builtin_fmaf(x[e], c, -ms));
  st.s = st.s * ex2(st.m - ms) + sum;
  st.m = m;
}

// (max, sum) of the wave in every lane: the maximum first, then the sums rescaled to it; both
// reductions have a fixed order, so reruns are bit-identical
__device__ __forceinline__ MaxSum wave_combine(MaxSum v) {
  const float m = wave_allreduce(v.m, [](float x, float y) { return fmaxf(x, y); });
  const float s = wave_allreduce(v.s * ex2_diff(v.m, m), [](float x, float y) { return x + y; });
  return MaxSum{m, s};
}

__device__ __forceinline__ float bf16_at(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }

__device__ __forceinline__ float finish_row(const LogprobArgs& a, int row, MaxSum t) {
  const int tok = a.tokens[row];
  if ((unsigned)tok >= (unsigned)a.vocab) return __uint_as_float(0x7fc00000u);
  const float y = bf16_at(a.logits + (size_t)row * a.vocab + tok) * a.inv_temp_log2e;
  return (y - (t.m + __builtin_amdgcn_logf(t.s))) * 0.69314718055994530942f;   // v_log_f32 is log2
}

__global__ __launch_bounds__(kLpThreads) void logprob_kernel(LogprobArgs a) {
  __shared__ MaxSum red[kLpThreads / 64];
  const int row = blockIdx.x / a.slices;
  const int slice = blockIdx.x % a.slices;
  const int tid = threadIdx.x;
  const float c = a.inv_temp_log2e;
  const long v0 = (long)slice * a.slice_len;
  const long v1 = min((long)a.vocab, v0 + a.slice_len);
  const uint16_t* x = a.logits + (size_t)row * a.vocab;
  MaxSum st{-INFINITY, 0.f};

  if (v0 < v1) {
    // elements before the first 16-byte boundary, then whole 16-byte vectors, then the rest
    const uintptr_t addr = reinterpret_cast<uintptr_t>(x + v0);
    const long head = min(v1 - v0, (long)(((16 - (addr & 15)) & 15) >> 1));
    if (tid < head) add_one(st, bf16_at(x + v0 + tid) * c);
    const long b0 = v0 + head;
    const long nvec = (v1 - b0) >> 3;
    const u32x4* xv = reinterpret_cast<const u32x4*>(x + b0);
    long k = tid;
    for (; k + (kUnroll - 1) * kLpThreads < nvec; k += kUnroll * kLpThreads) {
      u32x4 v[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(xv + k + u * kLpThreads);
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) add_vec(st, v[u], c);
    }
    for (; k < nvec; k += kLpThreads) add_vec(st, __builtin_nontemporal_load(xv + k), c);
    const long t0 = b0 + (nvec << 3);
    if (tid < v1 - t0) add_one(st, bf16_at(x + t0 + tid) * c);
  }

  st = wave_combine(st);
  if ((tid & 63) == 0) red[tid >> 6] = st;
  __syncthreads();
  if (tid == 0) {
    MaxSum t = red[0];
#pragma unroll
    for (int w = 1; w < kLpThreads / 64; ++w) t = combine(t, red[w]);
    if (a.slices == 1) a.out[row] = finish_row(a, row, t);
    else a.partials[(size_t)row * a.slices + slice] = make_float2(t.m, t.s);
  }
}

// one wave per row: combines the slices in a fixed order
__global__ __launch_bounds__(64) void logprob_finish_kernel(LogprobArgs a) {
  const int row = blockIdx.x;
  const int lane = threadIdx.x;
  MaxSum st{-INFINITY, 0.f};
  for (int k = lane; k < a.slices; k += 64) {
    const float2 p = a.partials[(size_t)row * a.slices + k];
    st = combine(st, MaxSum{p.x, p.y});
  }
  st = wave_combine(st);
  if (lane == 0) a.out[row] = finish_row(a, row, st);
}

}  // namespace

hipError_t launch_logprobs(const LogprobArgs& a, hipStream_t st) {
  if (a.rows == 0) return hipSuccess;
  hipLaunchKernelGGL(logprob_kernel, dim3((unsigned)a.rows * a.slices), dim3(kLpThreads), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_logprobs_finish(const LogprobArgs& a, hipStream_t st) {
  if (a.rows == 0 || a.slices == 1) return hipSuccess;
  hipLaunchKernelGGL(logprob_finish_kernel, dim3(a.rows), dim3(64), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
