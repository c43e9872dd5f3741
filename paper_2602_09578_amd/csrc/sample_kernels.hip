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
#include <type_traits>

#include "marl_internal.h"
#include "wave_ops.h"

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

// the 8 logits at x[pos .. pos+8) as four packed words (token 2d in the low half of word d);
// positions past the end read as -inf
__device__ __forceinline__ u32x4 load8_words(const uint16_t* x, long pos, long end) {
  const uint16_t* p = x + pos;
  if (pos + 8 <= end && (reinterpret_cast<uintptr_t>(p) & 15) == 0)
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  u32x4 v;
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t lo = pos + 2 * d < end ? p[2 * d] : 0xff80u;
    const uint32_t hi = pos + 2 * d + 1 < end ? p[2 * d + 1] : 0xff80u;
    v[d] = lo | (hi << 16);
  }
  return v;
}

template <class T>
__device__ __forceinline__ T wave_allreduce_sum(T v) { return wave_allreduce(v, [](T x, T y) { return x + y; }); }
__device__ __forceinline__ float wave_max(float v) { return wave_allreduce(v, [](float x, float y) { return fmaxf(x, y); }); }
__device__ __forceinline__ float wave_sum(float v) { return wave_allreduce_sum(v); }
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
  // the words of the wave's next chunk are requested before the current chunk is reduced
  u32x4 cur[kIters], nxt[kIters];
  auto fetch = [&](int chunk, u32x4 (&w)[kIters]) {
    const long base = (long)chunk * kChunk;
#pragma unroll
    for (int it = 0; it < kIters; ++it) w[it] = load8_words(x, base + it * 512 + lane * 8, a.vocab);
  };
  if (first + wave < a.num_chunks) fetch(first + wave, cur);
  for (int k = 0; k < a.chunks_per_wave; ++k) {
    const int chunk = first + wave + 4 * k;
    if (chunk >= a.num_chunks) break;
    const bool more = k + 1 < a.chunks_per_wave && chunk + 4 < a.num_chunks;   // wave-uniform
    if (more) fetch(chunk + 4, nxt);
    float m = -INFINITY;
#pragma unroll
    for (int it = 0; it < kIters; ++it)
#pragma unroll
      for (int d = 0; d < 4; ++d)
        m = fmaxf(m, fmaxf(__uint_as_float(cur[it][d] << 16), __uint_as_float(cur[it][d] & 0xffff0000u)));
    m = wave_max(m) * c;                 // c > 0: the scaled maximum is the maximum of the scaled values
    const float ms = m == -INFINITY ? 0.f : m;
    float s = 0.f;
#pragma unroll
    for (int it = 0; it < kIters; ++it)
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        s += ex2(__builtin_fmaf(__uint_as_float(cur[it][d] << 16), c, -ms));
        s += ex2(__builtin_fmaf(__uint_as_float(cur[it][d] & 0xffff0000u), c, -ms));
      }
    s = wave_sum(s);
    if (lane == 0) a.partials[(size_t)row * a.num_chunks + chunk] = make_float2(m, s);
    if (more) {
#pragma unroll
      for (int it = 0; it < kIters; ++it) cur[it] = nxt[it];
    }
  }
}

__global__ __launch_bounds__(64) void sample_pick_kernel(SampleArgs a) {
  const int lane = threadIdx.x;
  const int row = blockIdx.x;
  const float2* part = a.partials + (size_t)row * a.num_chunks;
  const uint16_t* x = a.logits + (size_t)row * a.vocab;
  const float c = a.inv_temp_log2e;
  // global max and total, chunk sums rescaled to the global max.  The few dozen chunk sums are
  // accumulated in double precision: they decide in which chunk the uniform number falls, and a
  // float32 running sum over the whole vocabulary would move a CDF step by up to ~1e-5.
  float M = -INFINITY;
  for (int k = lane; k < a.num_chunks; k += 64) M = fmaxf(M, part[k].x);
  M = wave_max(M);
  auto chunk_mass = [&](int k) -> double {
    return k < a.num_chunks ? (double)(part[k].y * ex2_diff(part[k].x, M)) : 0.0;
  };
  auto scan_d = [&](double v) {   // inclusive scan over the wave, fixed order
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const double t = __shfl_up(v, d);
      if (lane >= d) v += t;
    }
    return v;
  };
  double total = 0.0;
  for (int base = 0; base < a.num_chunks; base += 64)   // fixed order: tiles of 64 chunks
    total += __shfl(scan_d(chunk_mass(base + lane)), 63);
  const double target = (double)a.uniforms[row] * total;
  // the chunk in which the running sum passes the target
  double before = 0.0;
  bool take_last = false;
  int chunk = -1, last_nonzero = -1;
  for (int base = 0; base < a.num_chunks && chunk < 0; base += 64) {
    const int k = base + lane;
    const double v = chunk_mass(k);
    const double cum = before + scan_d(v);
    const unsigned long long hit = __builtin_amdgcn_ballot_w64(k < a.num_chunks && cum > target);
    const unsigned long long nz = __builtin_amdgcn_ballot_w64(v > 0.0);
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
    take_last = true;   // any non-zero element of the chunk passes; the last one is taken below
  }
  // remaining mass to pass inside the chunk (-inf: nothing passes, the last non-zero token is taken)
  const float want = take_last ? INFINITY : (float)(target - before);
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
      a.out_logprobs[row] = (y_tok - (M + __builtin_amdgcn_logf((float)total))) * 0.69314718055994530942f;
    }
  }
}

// ---------------------------------------------------------------------------------------
// Top-p (nucleus) sampling.  Tokens are ranked by probability (ties: lower index first); the
// nucleus is the shortest head of that ranking whose probability reaches top_p; the token is
// drawn from the nucleus by inverse CDF in INDEX order with the caller's uniform number scaled
// to the nucleus mass.  bf16 logits have at most 65536 distinct values and equal logits have
// equal probability, so the nucleus is "every token above a threshold value, plus the first c
// tokens at the threshold value": the kernel finds the threshold with an exact counting
// histogram over the values instead of sorting 150 k tokens.
//
// One workgroup of 512 threads owns a row and makes these passes over it.  Rows of up to
// kTpRegTiles * 4096 logits (163840: the vocabularies in use) are read from memory ONCE and kept
// in registers, 16 bytes per thread and tile (160 of a thread's 229 registers: with 1024 threads,
// i.e. 128 registers per thread, the compiler kept 6 of 20 tiles in scratch memory, 0.24 GB of
// writes per call on 2048 x 152064 logits; the time is the same either way); longer rows are
// re-read from the caches / HBM for every pass (16-byte loads):
//   1. maximum value and Z = sum 2^(y - M)  (running (max, sum) per thread, fixed-order merge);
//   2. count histogram in LDS over the 32768 values just below the maximum (order-preserving
//      16-bit key of the bf16 pattern; integer LDS atomics, so the result does not depend on
//      the order); a scan of value masses count * 2^(y(value) - M) from the top finds where the
//      cumulative mass reaches top_p * Z.  If that lies below the window (flat rows with top_p
//      near 1), the window moves down and the pass repeats (all 65536 values fit 2 windows);
//   3. per tile of 4096 tokens the nucleus mass and the number of threshold-value tokens; a
//      sequential walk over the tile sums finds the tile in which the scaled uniform is
//      passed, a workgroup scan inside that tile finds the token.
// ---------------------------------------------------------------------------------------
constexpr int kTpThreads = 512;
constexpr int kTpWaves = kTpThreads / 64;
constexpr int kWin = 32768;                  // histogram window, in values (keys)
constexpr int kTile = kTpThreads * 8;        // tokens per tile of pass 3
constexpr int kLowestKey = 0x0080;           // key of the most negative finite bf16; below: -inf, NaN
constexpr int kTpRegTiles = 40;              // tiles of a row that the register-resident variant holds
constexpr int kScanStep = 4;                 // scan positions per thread and round of the threshold search

__device__ __forceinline__ int key_of(uint32_t bits) {   // larger value <=> larger key; -0 counts as +0
  if ((bits & 0x7fffu) == 0) bits = 0;
  return (bits & 0x8000u) ? (int)(~bits & 0xffffu) : (int)(bits | 0x8000u);
}
__device__ __forceinline__ float value_of_key(int key) {
  const uint32_t bits = (key & 0x8000) ? (uint32_t)(key & 0x7fff) : (~(uint32_t)key & 0xffffu);
  return __uint_as_float(bits << 16);
}

struct TpShared {
  uint32_t hist[kWin];          // pass 2: counts; pass 3: per-(tile, wave) sums (reused)
  double wave_d[kTpWaves];
  float wave_f[kTpWaves];
  float wave_m[kTpWaves];
  int wave_i[kTpWaves];
  int found_at;                 // smallest scan position / thread index that meets a condition
  int thr_key, thr_cnt;         // threshold value (key) and how many tokens have it
  double thr_above;             // mass strictly above the threshold value
  int tile, ties_before;
  float want_in_tile;           // nucleus mass still to pass inside the chosen tile
  int out_tok;
  float out_y;
};

// exclusive scans over the workgroup in thread order (fixed order: bit-identical reruns)
__device__ __forceinline__ double block_excl_scan_d(double v, double& total, TpShared& sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  double inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const double t = __shfl_up(inc, d);
    if (lane >= d) inc += t;
  }
  __syncthreads();
  if (lane == 63) sh.wave_d[wave] = inc;
  __syncthreads();
  double before = 0.0, all = 0.0;
#pragma unroll
  for (int w = 0; w < kTpWaves; ++w) {
    if (w < wave) before += sh.wave_d[w];
    all += sh.wave_d[w];
  }
  total = all;
  return before + inc - v;
}
__device__ __forceinline__ float block_excl_scan_f(float v, TpShared& sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float inc = wave_inclusive_scan(v, lane);
  __syncthreads();
  if (lane == 63) sh.wave_f[wave] = inc;
  __syncthreads();
  float before = 0.f;
#pragma unroll
  for (int w = 0; w < kTpWaves; ++w)
    if (w < wave) before += sh.wave_f[w];
  return before + inc - v;
}
__device__ __forceinline__ int block_excl_scan_i(int v, TpShared& sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(inc, d);
    if (lane >= d) inc += t;
  }
  __syncthreads();
  if (lane == 63) sh.wave_i[wave] = inc;
  __syncthreads();
  int before = 0;
#pragma unroll
  for (int w = 0; w < kTpWaves; ++w)
    if (w < wave) before += sh.wave_i[w];
  return before + inc - v;
}

// One sweep over a row: calls fn(tile, the four 32-bit words that hold this thread's 8 tokens
// of the tile, token 2d in the low half of word d) for every tile in order; positions past the
// end of the row read as -inf.  Full tiles of a 16-byte aligned row are fetched four at a time
// (64 bytes per thread in flight) before any of them is used.
template <class F>
__device__ __forceinline__ void sweep_row(const uint16_t* x, long V, int tid, F&& fn) {
  const int ntiles = (int)((V + kTile - 1) / kTile);
  const int nfull = (reinterpret_cast<uintptr_t>(x) & 15) == 0 ? (int)(V / kTile) : 0;
  int t = 0;
  for (; t + 4 <= nfull; t += 4) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      v[u] = *reinterpret_cast<const u32x4*>(x + (long)(t + u) * kTile + (long)tid * 8);
#pragma unroll
    for (int u = 0; u < 4; ++u) fn(t + u, v[u]);
  }
  for (; t < ntiles; ++t) fn(t, load8_words(x, (long)t * kTile + (long)tid * 8, V));
}
// the two bf16 of a word widened to float
__device__ __forceinline__ float lo_val(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_val(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// a value that is the same in every lane, moved to a scalar register (frees a vector register)
__device__ __forceinline__ float uniform_f(float v) { return __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane((int)__float_as_uint(v))); }
__device__ __forceinline__ int uniform_i(int v) { return __builtin_amdgcn_readfirstlane(v); }

// NT > 0: the row's tiles live in NT 16-byte registers per thread (vocab <= NT * kTile);
// NT = 0: every pass reads the row from memory.
template <int NT>
__device__ __forceinline__ void sample_top_p_body(const TopPArgs& a) {
  __shared__ TpShared sh;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x;
  const uint16_t* x = a.logits + (size_t)row * a.vocab;
  const float c = a.inv_temp_log2e;
  const long V = a.vocab;
  const int ntiles = (int)((V + kTile - 1) / kTile);
  u32x4 held[NT > 0 ? NT : 1];
  if constexpr (NT > 0) {
    // every load is issued before the first use: NT * 16 bytes per thread in flight
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      held[t] = u32x4{0xff80ff80u, 0xff80ff80u, 0xff80ff80u, 0xff80ff80u};   // -inf
      if (t < ntiles) held[t] = load8_words(x, (long)t * kTile + (long)tid * 8, V);
    }
  }
  // one pass over the row in tile order: fn(tile, this thread's 8 tokens of the tile as 4 words)
  auto sweep = [&](auto&& fn) {
    if constexpr (NT > 0) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        if (t < ntiles) {   // workgroup-uniform
          // a copy whose value the compiler cannot trace back to the held row: otherwise it
          // hoists per-token results of a pass (the 8 * NT keys) out of the loops around the
          // pass and keeps them in scratch memory
          u32x4 v = held[t];
          asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]));
          fn(t, v);
        }
      }
    } else {
      sweep_row(x, V, tid, fn);
    }
  };

  // ---- pass 1: largest value and Z relative to it, in one sweep -------------------------------
  // per thread a running (largest y so far, sum relative to it); merged in thread order
  float xrun = -INFINITY, mrun = -INFINITY, zrun = 0.f;   // largest raw logit, the same times c, sum
  sweep([&](int, u32x4 v) {
    float r[8];
#pragma unroll
    for (int d = 0; d < 4; ++d) { r[2 * d] = lo_val(v[d]); r[2 * d + 1] = hi_val(v[d]); }
    const float x8 = fmaxf(fmaxf(fmaxf(r[0], r[1]), fmaxf(r[2], r[3])), fmaxf(fmaxf(r[4], r[5]), fmaxf(r[6], r[7])));
    if (x8 > xrun) {                       // c > 0: the largest raw logit is the largest scaled one
      const float m8 = x8 * c;
      zrun *= ex2(mrun - m8);              // mrun = -inf: zrun is 0 and stays 0
      xrun = x8;
      mrun = m8;
    }
    if (xrun > -INFINITY) {
      float s8 = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) s8 += ex2(__builtin_fmaf(r[e], c, -mrun));
      zrun += s8;
    }
  });
  float xmax = xrun;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) xmax = fmaxf(xmax, __shfl_xor(xmax, d));
  if (lane == 0) sh.wave_m[wave] = xmax;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kTpWaves; ++w) xmax = fmaxf(xmax, sh.wave_m[w]);
  xmax = uniform_f(xmax);
  const float M = uniform_f(xmax * c);
  double ztot;
  block_excl_scan_d(xrun > -INFINITY ? (double)zrun * (double)ex2(mrun - M) : 0.0, ztot, sh);
  const double Z = ztot;
  if (!(xmax > -INFINITY) || !(Z > 0.0) || !(Z < 1e300)) {   // no finite logit, or +inf / NaN: nothing to draw
    if (tid == 0) {
      a.out_tokens[row] = -1;
      a.out_logprobs[row] = __uint_as_float(0x7fc00000u);
    }
    return;
  }
  const int kmax = key_of(__float_as_uint(xmax) >> 16);
  // the weight of a value, computed the same way everywhere: 2^(fma(value, c, -M))
  auto weight = [&](int key) { return key >= kLowestKey ? ex2(__builtin_fmaf(value_of_key(key), c, -M)) : 0.f; };

  // ---- pass 2: the threshold value --------------------------------------------------------
  // thr_key = -1: every token with a finite logit is in the nucleus
  if (tid == 0) { sh.thr_key = -1; sh.thr_cnt = 0; sh.thr_above = 0.0; }
  if (a.top_p < 1.f) {
    const double tau = (double)a.top_p * Z;
    double above = 0.0;                       // mass of the values above the window
    for (int hi = kmax; hi >= kLowestKey; hi -= kWin) {
      const int lo = hi - (kWin - 1);
      for (int i = tid; i < kWin; i += kTpThreads) sh.hist[i] = 0;
      if (tid == 0) sh.found_at = kWin;
      __syncthreads();
      const int lo_eff = max(lo, kLowestKey);
      const unsigned span = (unsigned)(hi - lo_eff);
      sweep([&](int, u32x4 v) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const int k0 = key_of(v[d] & 0xffffu), k1 = key_of(v[d] >> 16);
          if ((unsigned)(k0 - lo_eff) <= span) atomicAdd(&sh.hist[k0 - lo], 1u);
          if ((unsigned)(k1 - lo_eff) <= span) atomicAdd(&sh.hist[k1 - lo], 1u);
        }
      });
      __syncthreads();
      // Position j of the scan is the value hi - j.  The window is scanned in rounds of
      // kScanStep positions per thread (thread t owns j = base + kScanStep t .. + kScanStep - 1)
      // and the scan stops at the round in which the cumulative mass reaches tau: for peaked
      // rows that is the first round, a few hundred values below the maximum.
      auto mass_at = [&](int pos) {
        const int key = hi - pos;
        const uint32_t cnt = sh.hist[key - lo];
        return cnt ? (double)cnt * (double)weight(key) : 0.0;
      };
      double window_total = 0.0;
      for (int base = 0; base < kWin; base += kScanStep * kTpThreads) {
        const int p0 = base + tid * kScanStep;
        double mine = 0.0;
#pragma unroll
        for (int q = 0; q < kScanStep; ++q) mine += mass_at(p0 + q);
        double round_total;
        const double before = above + window_total + block_excl_scan_d(mine, round_total, sh);
        // first scan position at which the cumulative mass reaches tau: every thread at or past
        // the crossing proposes its first such position, the smallest wins (robust against the
        // last-bit differences between neighbouring threads' scan values)
        int my_pos = kWin;
        double my_above = 0.0;
        if (before + mine >= tau) {
          double run = before;
#pragma unroll 1
          for (int q = 0; q < kScanStep; ++q) {
            const double m = mass_at(p0 + q);
            if (m > 0.0 && run + m >= tau) { my_pos = p0 + q; my_above = run; break; }
            run += m;
          }
          if (my_pos < kWin) atomicMin(&sh.found_at, my_pos);
        }
        __syncthreads();
        if (my_pos < kWin && my_pos == sh.found_at) {
          const int key = hi - my_pos;
          sh.thr_key = key;
          sh.thr_cnt = (int)sh.hist[key - lo];
          sh.thr_above = my_above;
        }
        __syncthreads();
        if (sh.found_at < kWin) break;        // workgroup-uniform
        window_total += round_total;
      }
      if (sh.found_at < kWin) break;          // workgroup-uniform
      above += window_total;
    }
  }
  __syncthreads();
  const int thr_key = uniform_i(sh.thr_key);
  // how many of the threshold-value tokens (in index order) the nucleus takes
  int ties_kept = 0;
  float thr_w = 0.f;
  double nucleus = Z;
  if (thr_key >= 0) {
    thr_w = uniform_f(weight(thr_key));
    const double need = ((double)a.top_p * Z - sh.thr_above) / (double)thr_w;
    ties_kept = uniform_i((int)fmin(fmax(ceil(need), 1.0), (double)sh.thr_cnt));
    nucleus = sh.thr_above + (double)ties_kept * (double)thr_w;
  }
  // the walk over the tile sums runs in double precision (a float32 running sum over the whole
  // vocabulary would move a CDF step by up to ~1e-5 of the nucleus mass); inside the chosen tile
  // float32 sums start from zero again and are compared with the mass that is left to pass
  const double target = (double)a.uniforms[row] * nucleus;
  // pass 3 compares raw logit values (every bf16 is exact in float; -0 == +0 as in the keys);
  // with no threshold every finite logit is above it
  const float thr_x = uniform_f(thr_key >= 0 ? value_of_key(thr_key) : -INFINITY);
  const float log2_Z = uniform_f(__builtin_amdgcn_logf((float)Z));

  // ---- pass 3: inverse CDF over the nucleus in index order ----------------------------------
  // per tile and wave: mass of the tokens above the threshold, number of tokens at it
  float* part_m = reinterpret_cast<float*>(sh.hist);             // [ntiles][kTpWaves]
  int* part_n = reinterpret_cast<int*>(sh.hist) + kWin / 2;      // [ntiles][kTpWaves]
  __syncthreads();                                               // the histogram is no longer read
  sweep([&](int t, u32x4 v) {
    float m8 = 0.f;
    int n8 = 0;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const float r0 = lo_val(v[d]), r1 = hi_val(v[d]);
      const float w0 = ex2(__builtin_fmaf(r0, c, -M)), w1 = ex2(__builtin_fmaf(r1, c, -M));
      m8 += r0 > thr_x ? w0 : 0.f;
      m8 += r1 > thr_x ? w1 : 0.f;
      n8 += (r0 == thr_x) + (r1 == thr_x);
    }
    m8 = wave_allreduce_sum(m8);
    n8 = wave_allreduce_sum(n8);
    if (lane == 0) { part_m[t * kTpWaves + wave] = m8; part_n[t * kTpWaves + wave] = n8; }
  });
  __syncthreads();
  if (tid == 0) {
    double cum = 0.0, last_cum = 0.0;
    int ties = 0, tile = -1, last_tile = 0, last_ties = 0;
    for (int t = 0; t < ntiles && tile < 0; ++t) {
      double m = 0.0;
      int n = 0;
      for (int w = 0; w < kTpWaves; ++w) { m += (double)part_m[t * kTpWaves + w]; n += part_n[t * kTpWaves + w]; }
      const double kept = m + (double)thr_w * (double)min(n, max(0, ties_kept - ties));
      if (kept > 0.0) { last_tile = t; last_cum = cum; last_ties = ties; }
      if (cum + kept > target) { tile = t; break; }
      cum += kept;
      ties += n;
    }
    if (tile < 0) {               // rounding left the target at or above the total: the last token
      tile = last_tile;           // of the nucleus is taken (inside the tile, below)
      cum = last_cum;
      ties = last_ties;
    }
    sh.tile = tile;
    sh.want_in_tile = (float)(target - cum);
    sh.ties_before = ties;
    sh.found_at = kTpThreads;
    sh.out_tok = -1;
  }
  __syncthreads();
  {
    const int t = sh.tile;
    const long pos = (long)t * kTile + (long)tid * 8;
    u32x4 v;
    if constexpr (NT > 0) {
      v = held[0];
#pragma unroll
      for (int u = 1; u < NT; ++u)
        if (u == t) v = held[u];
    } else {
      v = load8_words(x, pos, V);
    }
    float r[8];
#pragma unroll
    for (int d = 0; d < 4; ++d) { r[2 * d] = lo_val(v[d]); r[2 * d + 1] = hi_val(v[d]); }
    int n8 = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) n8 += r[e] == thr_x;
    int rank = sh.ties_before + block_excl_scan_i(n8, sh);       // threshold-value tokens before this thread
    float w8[8], m8 = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float w = 0.f;
      if (r[e] > thr_x) w = ex2(__builtin_fmaf(r[e], c, -M));
      else if (r[e] == thr_x) { if (rank < ties_kept) w = thr_w; ++rank; }
      w8[e] = w;
      m8 += w;
    }
    const float want = sh.want_in_tile;
    const float before = block_excl_scan_f(m8, sh);
    const bool pass = before + m8 > want && m8 > 0.f;
    if (pass) atomicMin(&sh.found_at, tid);
    // the last thread of the tile that holds a nucleus token, for the rounding fallback
    if (m8 > 0.f) atomicMax(&sh.out_tok, tid);
    __syncthreads();
    const int winner = sh.found_at < kTpThreads ? sh.found_at : sh.out_tok;
    const bool fallback = sh.found_at >= kTpThreads;
    if (winner < 0 && tid == 0) {   // no nucleus token in the tile: cannot happen for Z > 0
      a.out_tokens[row] = -1;
      a.out_logprobs[row] = __uint_as_float(0x7fc00000u);
    }
    if (tid == winner) {
      float run = before;
      int e_pick = -1;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (w8[e] > 0.f) {
          run += w8[e];
          if (fallback) e_pick = e;                               // last nucleus token of the thread
          else if (e_pick < 0 && run > want) e_pick = e;
        }
      }
      if (e_pick < 0) {                                           // cannot happen: pass implies a hit
#pragma unroll
        for (int e = 0; e < 8; ++e) if (w8[e] > 0.f) e_pick = e;
      }
      float r_pick = r[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) if (e == e_pick) r_pick = r[e];
      a.out_tokens[row] = (int)(pos + e_pick);
      a.out_logprobs[row] = (__builtin_fmaf(r_pick, c, -M) - log2_Z) * 0.69314718055994530942f;
    }
  }
}

__global__ __launch_bounds__(kTpThreads) void sample_top_p_kernel(TopPArgs a) { sample_top_p_body<kTpRegTiles>(a); }
__global__ __launch_bounds__(kTpThreads) void sample_top_p_kernel_long(TopPArgs a) { sample_top_p_body<0>(a); }

}  // namespace

int sample_num_chunks(int vocab) { return (vocab + kChunk - 1) / kChunk; }

int top_p_max_vocab() { return (kWin / 2 / kTpWaves) * kTile; }   // tile sums must fit the LDS buffer

hipError_t launch_sample_top_p(const TopPArgs& a, hipStream_t st) {
  if (a.rows == 0) return hipSuccess;
  if (a.vocab <= kTpRegTiles * kTile)
    hipLaunchKernelGGL(sample_top_p_kernel, dim3((unsigned)a.rows), dim3(kTpThreads), 0, st, a);
  else
    hipLaunchKernelGGL(sample_top_p_kernel_long, dim3((unsigned)a.rows), dim3(kTpThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_sample(const SampleArgs& a, hipStream_t st) {
  if (a.rows == 0) return hipSuccess;
  hipLaunchKernelGGL(sample_scan_kernel, dim3((unsigned)a.rows * a.groups_per_row), dim3(256), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(sample_pick_kernel, dim3(a.rows), dim3(64), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
