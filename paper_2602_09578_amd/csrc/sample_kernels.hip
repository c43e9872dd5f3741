// Sampling fused with the log-probability: one streaming pass over a row's logits yields
// what is needed to draw a token from softmax(logits / T) by inverse-CDF with a uniform
// number supplied by the caller, and that token's log-probability (rollout produces both for
// every generated token; the paper trains with GRPO, Section 8.1, which consumes the latter).
//
// Pass 1 (streaming, the cost of the log-prob kernel): every wave takes contiguous chunks of
//   4096 logits and stores each chunk's (max, sum of 2^(y - max)), y = x * log2(e) / T.
// Pass 2 (one wave per row, re-reads 8 KB): an ordered scan over the chunk sums finds the chunk
//   in which the cumulative probability passes u, an ordered scan inside that chunk finds the
//   token.  Token = first t with sum_{v <= t} p_v > u; if rounding leaves none, the last token
//   with non-zero probability.
#include "marl_internal.h"

namespace marl {
namespace {

constexpr int kChunk = 4096;          // logits per wave chunk: 8 iterations x 64 lanes x 8
constexpr int kIters = kChunk / 512;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float ex2_diff(float a, float b) { return ex2(a - (b == -INFINITY ? 0.f : b)); }

// y values of the 8 logits at x[pos .. pos+8) that exist (pos + e < end); missing ones are -inf.
// Uses one 16-byte load when the address is aligned and all 8 exist.
__device__ __forceinline__ void load8(const uint16_t* x, long pos, long end, float c, float (&y)[8]) {
  const uint16_t* p = x + pos;
  if (pos + 8 <= end && (reinterpret_cast<uintptr_t>(p) & 15) == 0) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      y[2 * d] = __uint_as_float(v[d] << 16) * c;
      y[2 * d + 1] = __uint_as_float(v[d] & 0xffff0000u) * c;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      y[e] = pos + e < end ? __uint_as_float((uint32_t)p[e] << 16) * c : -INFINITY;
  }
}

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
__device__ __forceinline__ float wave_inclusive_scan(float v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const float t = __shfl_up(v, d);
    if (lane >= d) v += t;
  }
  return v;
}

// grid: rows * groups_per_row workgroups of 4 waves; a workgroup covers 4 * chunks_per_wave
// consecutive chunks of one row, wave w taking chunks first + w, first + w + 4, ...
__global__ __launch_bounds__(256) void sample_scan_kernel(SampleArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x / a.groups_per_row;
  const int first = (blockIdx.x % a.groups_per_row) * 4 * a.chunks_per_wave;
  const uint16_t* x = a.logits + (size_t)row * a.vocab;
  const float c = a.inv_temp_log2e;
  for (int k = 0; k < a.chunks_per_wave; ++k) {
    const int chunk = first + wave + 4 * k;
    if (chunk >= a.num_chunks) break;
    const long base = (long)chunk * kChunk;
    float y[kIters][8];
#pragma unroll
    for (int it = 0; it < kIters; ++it) load8(x, base + it * 512 + lane * 8, a.vocab, c, y[it]);
    float m = -INFINITY;
#pragma unroll
    for (int it = 0; it < kIters; ++it)
#pragma unroll
      for (int e = 0; e < 8; ++e) m = fmaxf(m, y[it][e]);
    m = wave_max(m);
    const float ms = m == -INFINITY ? 0.f : m;
    float s = 0.f;
#pragma unroll
    for (int it = 0; it < kIters; ++it)
#pragma unroll
      for (int e = 0; e < 8; ++e) s += ex2(y[it][e] - ms);
    s = wave_sum(s);
    if (lane == 0) a.partials[(size_t)row * a.num_chunks + chunk] = make_float2(m, s);
  }
}

__global__ __launch_bounds__(64) void sample_pick_kernel(SampleArgs a) {
  const int lane = threadIdx.x;
  const int row = blockIdx.x;
  const float2* part = a.partials + (size_t)row * a.num_chunks;
  const uint16_t* x = a.logits + (size_t)row * a.vocab;
  const float c = a.inv_temp_log2e;
  // global max and total, chunk sums rescaled to the global max
  float M = -INFINITY;
  for (int k = lane; k < a.num_chunks; k += 64) M = fmaxf(M, part[k].x);
  M = wave_max(M);
  float total = 0.f;
  for (int base = 0; base < a.num_chunks; base += 64) {   // fixed order: tiles of 64 chunks
    const int k = base + lane;
    total += wave_sum(k < a.num_chunks ? part[k].y * ex2_diff(part[k].x, M) : 0.f);
  }
  const float target = a.uniforms[row] * total;
  // the chunk in which the running sum passes the target
  float before = 0.f;
  int chunk = -1, last_nonzero = -1;
  for (int base = 0; base < a.num_chunks && chunk < 0; base += 64) {
    const int k = base + lane;
    const float v = k < a.num_chunks ? part[k].y * ex2_diff(part[k].x, M) : 0.f;
    const float cum = before + wave_inclusive_scan(v, lane);
    const unsigned long long hit = __builtin_amdgcn_ballot_w64(k < a.num_chunks && cum > target);
    const unsigned long long nz = __builtin_amdgcn_ballot_w64(v > 0.f);
    if (nz) last_nonzero = base + 63 - __builtin_clzll(nz);
    if (hit) {
      const int l = __builtin_ctzll(hit);
      chunk = base + l;
      before = __shfl(cum - v, l);
    } else {
      before = __shfl(cum, 63);
    }
  }
  if (chunk < 0) {   // rounding: u * total not below the last partial sum
    chunk = max(last_nonzero, 0);
    before = -INFINITY;   // any non-zero element of the chunk passes; the last one is taken below
  }
  const float want = target - before;   // remaining mass to pass inside the chunk (+inf = take the last)
  const long cbase = (long)chunk * kChunk;
  float run = 0.f;
  int tok = -1, last_tok = -1;
  float y_tok = 0.f, y_last = 0.f;
  for (int it = 0; it < kIters && tok < 0; ++it) {
    float y[8];
    const long pos = cbase + it * 512 + lane * 8;
    load8(x, pos, a.vocab, c, y);
    float w[8], s = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) { w[e] = ex2_diff(y[e], M); s += w[e]; }
    const float cum = run + wave_inclusive_scan(s, lane);
    const unsigned long long hit = __builtin_amdgcn_ballot_w64(cum > want);
    const unsigned long long nz = __builtin_amdgcn_ballot_w64(s > 0.f);
    if (nz) {   // remember the last token with non-zero probability seen so far
      const int l = 63 - __builtin_clzll(nz);
      int e_last = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) if (w[e] > 0.f) e_last = e;
      last_tok = __shfl((int)(pos + e_last), l);
      float ysel = y[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) if (e == e_last) ysel = y[e];
      y_last = __shfl(ysel, l);
    }
    if (hit) {
      const int l = __builtin_ctzll(hit);
      float acc = cum - s;     // mass before this lane's 8 logits
      int e_hit = 7;
      bool found = false;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        acc += w[e];
        if (!found && acc > want) { e_hit = e; found = true; }
      }
      float ysel = y[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) if (e == e_hit) ysel = y[e];
      tok = __shfl((int)(pos + e_hit), l);
      y_tok = __shfl(ysel, l);
    } else {
      run = __shfl(cum, 63);
    }
  }
  if (tok < 0) { tok = last_tok; y_tok = y_last; }
  if (lane == 0) {
    if (tok < 0) {   // a row of -inf logits (or NaN): no token can be drawn
      a.out_tokens[row] = -1;
      a.out_logprobs[row] = __uint_as_float(0x7fc00000u);
    } else {
      a.out_tokens[row] = tok;
      a.out_logprobs[row] = (y_tok - (M + __builtin_amdgcn_logf(total))) * 0.69314718055994530942f;
    }
  }
}

}  // namespace

int sample_num_chunks(int vocab) { return (vocab + kChunk - 1) / kChunk; }

hipError_t launch_sample(const SampleArgs& a, hipStream_t st) {
  if (a.rows == 0) return hipSuccess;
  hipLaunchKernelGGL(sample_scan_kernel, dim3((unsigned)a.rows * a.groups_per_row), dim3(256), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(sample_pick_kernel, dim3(a.rows), dim3(64), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
