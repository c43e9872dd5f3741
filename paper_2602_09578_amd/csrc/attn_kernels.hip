// Decode attention over the paged KV cache: the prefix kernel (a group's prefix KV is
// streamed once and applied to all of the group's query rows), the suffix kernel (each
// sequence's own generated tokens) and the merge kernel.  The first two produce
// flash-decoding style partials (running max, running sum, unnormalised output) per (query
// row, chunk of tokens), which the merge kernel combines; a sequence whose own tokens are a
// single work item is finished by whoever processes that item instead.
//
// Context in the paper: rollout is memory-bound on KV caches (Section 4.1), every prompt is
// expanded into several samples that share its prefix (Section 5.1) and lengths are skewed
// (Section 2.2); the paper gives no kernel, so the design below is this library's own.
//
// Wave-level scheme (gfx950, wave64, v_mfma_f32_16x16x32_bf16).  A wave handles 32 tokens
// (two pages) per step and up to MT tiles of 16 query rows.  Lane l = 16*j + i.
//   scores:  D[token-row][q-row] = K-tile (A operand) x Q^T (B operand).  A-row i of tile T
//            is the token 8*(i/4) + 4*T + i%4 of the 32, so that after both tiles lane
//            (i, j) holds the scores of q-row i for tokens 8j..8j+7: exactly the B operand
//            layout the second product needs, with no data movement.
//   output:  D[channel][q-row] += V^T-tile (A operand) x P^T (B operand), 8 channel tiles.
//            V pages are stored [channel][slot], so lane (i, j) loads its 8 tokens of
//            channel 16*ct + i with one 16-byte load.
// Suffix kernel: K and V go straight from global memory into MFMA operand registers (16-byte
// loads; per instruction a wave reads 16 x 64 B of K or 2 x 512 B of V); LDS only combines
// the four waves of a workgroup, which split the item's tokens between them.
// Prefix kernel: the four waves split the query rows instead and share each K/V step
// through a double-buffered LDS tile (described at the kernel).
#include <type_traits>

#include "marl_internal.h"
#include "wave_ops.h"

namespace marl {
namespace {

constexpr int kWaves = kAttnThreads / 64;

// LDS per workgroup for the cross-wave combine: (max, sum) and the row index of every q-row, and
// every wave's accumulators in row-major order (a row is 128 floats, padded to 132 so that the
// 16 rows a wave instruction writes start in different banks).
constexpr int kAccRowFloats = kD + 4;
template <int MT>
struct ItemLds {
  float m[kWaves][MT * 16];
  float l[kWaves][MT * 16];
  int row[MT * 16];
  __attribute__((aligned(16))) float acc[kWaves][MT * 16][kAccRowFloats];
};

// Processes tokens [tok_begin, tok_end) of one block-table row for MT tiles of query rows
// and writes one partial per valid row.  NW is the number of waves that share the item:
//   NW = 4: called by all four waves of the workgroup, which take the 32-token steps in
//           turn and are combined through LDS (workgroup barriers inside);
//   NW = 1: called by one wave on its own (no LDS, no barrier): for short items.
//   row_index[qt]: for this lane's q-row (i) of tile qt, seq*Hq + head, or -1 if the row
//   does not exist.  slot: partial slot of this chunk.
//   finish (uniform over the callers): the item holds all of the sequence's own tokens, so the
//   rows' only other partials are the n_prefix_partials prefix partials of its group, which an
//   earlier kernel has completed: they are merged with the item's own result (the merge
//   kernel's formula and order: prefix slots first) and the final output rows are written
//   instead of a partial.
template <int MT, int NW>
__device__ __forceinline__ void process_item(const AttnArgs& a, const int32_t* __restrict__ table_row,
                                             const int tok_begin, const int tok_end, const int kvh,
                                             const int (&row_index)[MT], const int slot,
                                             ItemLds<MT>& lds, int& bad_page,
                                             const bool finish = false, const int n_prefix_partials = 0) {
  const int lane = threadIdx.x & 63;
  const int wave = NW == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int i = lane & 15, j = lane >> 4;
  // scores are kept in log2 units; a zero scale becomes a tiny one so that -inf * sc stays -inf
  const float sc = fmaxf(fabsf(a.scale) * 1.44269504088896340736f, 1e-30f);
  const uint32_t sign_flip = a.scale < 0.f ? 0x80008000u : 0u;
  const int nslot = a.NCp + a.NCs;

  // Q^T operand: lane (i, j) holds channels 8*(4*kk + j) .. +8 of q-row i
  u32x4 qreg[MT][4];
#pragma unroll
  for (int qt = 0; qt < MT; ++qt) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (row_index[qt] >= 0) {
        v = *reinterpret_cast<const u32x4*>(a.q + (size_t)row_index[qt] * kD + (4 * kk + j) * 8);
        v ^= sign_flip;
      }
      qreg[qt][kk] = v;
    }
  }

  f32x4 acc[MT][8];
  float m_run[MT], l_run[MT];
#pragma unroll
  for (int qt = 0; qt < MT; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) acc[qt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const size_t page_bytes = (size_t)a.Hkv * (kPage * kD * 2);
  const char* kbase = reinterpret_cast<const char*>(a.k_pages) + (size_t)kvh * (kPage * kD * 2) +
                      ((8 * ((i >> 2) & 1) + (i & 3)) * (kD * 2) + j * 16);
  const char* vbase = reinterpret_cast<const char*>(a.v_pages) + (size_t)kvh * (kPage * kD * 2) +
                      (i * (kPage * 2) + (j & 1) * 16);

  // Page ids of the 32-token step that starts at token t (wave-uniform, scalar loads).
  auto load_pages = [&](int t, int& p0, int& p1) {
    p0 = ld_uniform(table_row + (t >> 4));
    p1 = (t + kPage < tok_end) ? ld_uniform(table_row + (t >> 4) + 1) : p0;
    if ((unsigned)p0 >= (unsigned)a.num_pages) { p0 = 0; bad_page = 1; }
    if ((unsigned)p1 >= (unsigned)a.num_pages) { p1 = 0; bad_page = 1; }
  };
  u32x4 kr[2][4], vr[8];
  auto issue_k = [&](int p0, int p1) {
    const char* kp = kbase + (size_t)(i < 8 ? p0 : p1) * page_bytes;
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        kr[T][kk] = ld_stream_k(kp + T * (4 * kD * 2) + kk * 64);
  };
  auto issue_v = [&](int p0, int p1) {
    const char* vp = vbase + (size_t)(j < 2 ? p0 : p1) * page_bytes;
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) vr[ct] = ld_stream(vp + ct * (16 * kPage * 2));
  };

  // Software pipeline: the K registers are refilled for the next step as soon as the score
  // MFMAs have consumed them, the V registers as soon as the output MFMAs have; page ids are
  // fetched one step ahead.  So a wave keeps 16 KB of loads in flight while it computes.
  // The last step of a wave is peeled (no refill; it alone can be ragged) so that the loop
  // body has no conditional loads and every wait leaves the younger 8 loads in flight.
  constexpr int stride = NW * kBlockTok;
  int t0 = tok_begin + wave * kBlockTok;
  int tn = t0 + stride;
  int n0 = 0, n1 = 0;

  auto step = [&](auto has_next_tag) {
    constexpr bool kHasNext = decltype(has_next_tag)::value;
    f32x4 s[MT][2];
#pragma unroll
    for (int qt = 0; qt < MT; ++qt)
#pragma unroll
      for (int T = 0; T < 2; ++T) {
        s[qt][T] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) s[qt][T] = mfma_16x16x32(kr[T][kk], qreg[qt][kk], s[qt][T]);
      }
    if constexpr (kHasNext) issue_k(n0, n1);

    if constexpr (!kHasNext) {
      if (t0 + kBlockTok > tok_end) {   // wave-uniform: the ragged end of a chunk
        // tokens past the end: score -inf (weight 0), and zero their value slots, which may
        // hold anything (NaN included)
#pragma unroll
        for (int qt = 0; qt < MT; ++qt)
#pragma unroll
          for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (t0 + 8 * j + 4 * T + e >= tok_end) s[qt][T][e] = -INFINITY;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const int tok = t0 + 8 * j + 2 * d;
          const uint32_t mask = (tok < tok_end ? 0x0000ffffu : 0u) | (tok + 1 < tok_end ? 0xffff0000u : 0u);
#pragma unroll
          for (int ct = 0; ct < 8; ++ct) vr[ct][d] &= mask;
        }
      }
    }

    u32x4 pb[MT];
#pragma unroll
    for (int qt = 0; qt < MT; ++qt) {
      const f32x4 s0 = s[qt][0], s1 = s[qt][1];
      float mx = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                       fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
      mx = rows_allreduce_max(mx);
      const float m_new = fmaxf(m_run[qt], mx * sc);
      const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_new);
      float p[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[e], sc, -m_new));
        p[4 + e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[e], sc, -m_new));
      }
      const float psum = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
      if (__builtin_amdgcn_ballot_w64(m_new > m_run[qt]) != 0) {   // wave-uniform
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) acc[qt][ct] *= alpha;
      }
      l_run[qt] = l_run[qt] * alpha + psum;
      m_run[qt] = m_new;
      pb[qt] = u32x4{pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
    }
#pragma unroll
    for (int ct = 0; ct < 8; ++ct)
#pragma unroll
      for (int qt = 0; qt < MT; ++qt) acc[qt][ct] = mfma_16x16x32(vr[ct], pb[qt], acc[qt][ct]);

    if constexpr (kHasNext) {
      issue_v(n0, n1);
      t0 = tn;
      tn += stride;
      if (tn < tok_end) load_pages(tn, n0, n1);
    }
  };

  if (t0 < tok_end) {
    load_pages(t0, n0, n1);
    issue_k(n0, n1);
    issue_v(n0, n1);
    if (tn < tok_end) load_pages(tn, n0, n1);
    while (tn < tok_end) step(std::true_type{});
    step(std::false_type{});
  }

  // the four lanes that share a q-row each hold a part of its sum
#pragma unroll
  for (int qt = 0; qt < MT; ++qt) {
    l_run[qt] = rows_allreduce_sum(l_run[qt]);
  }

  if constexpr (NW > 1) {
    // Combine the waves: every wave puts its (max, sum) and its accumulators, row-major, into
    // LDS; after one barrier all threads share the 16 x 128 outputs, each computing a float4 as
    // the sum over the waves in wave order (fixed order: bit-identical reruns) rescaled to the
    // common max, and the workgroup writes every row's 512 bytes as full cache lines.
    static_assert(MT == 1, "the workgroup-wide combine handles one 16-row tile");
    if (j == 0) {
      lds.m[wave][i] = m_run[0];
      lds.l[wave][i] = l_run[0];
      if (wave == 0) lds.row[i] = row_index[0];
    }
#pragma unroll
    for (int ct = 0; ct < 8; ++ct)
      *reinterpret_cast<f32x4*>(&lds.acc[wave][i][16 * ct + 4 * j]) = acc[0][ct];
    __syncthreads();
    constexpr int kPerThread = 16 * (kD / 4) / (NW * 64);   // float4 outputs per thread
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      const int e = threadIdx.x + k * NW * 64;
      const int r = e / (kD / 4), c4 = e % (kD / 4);
      const int ridx = lds.row[r];
      if (ridx >= 0) {
        float mm = lds.m[0][r];
#pragma unroll
        for (int w = 1; w < NW; ++w) mm = fmaxf(mm, lds.m[w][r]);
        float ll = 0.f;
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          const float mw = lds.m[w][r];
          const float f = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mm);
          ll += lds.l[w][r] * f;
          o += *reinterpret_cast<const f32x4*>(&lds.acc[w][r][4 * c4]) * f;
        }
        if (!finish) {
          const size_t ps = (size_t)ridx * nslot + slot;
          *reinterpret_cast<f32x4*>(a.partial_o + ps * kD + 4 * c4) = o;
          if (c4 == 0) a.partial_ml[ps] = make_float2(mm, ll);
        } else {
          const size_t p0 = (size_t)ridx * nslot;
          float mstar = mm;
          for (int k = 0; k < n_prefix_partials; ++k) mstar = fmaxf(mstar, a.partial_ml[p0 + k].x);
          float denom = 0.f;
          f32x4 sum = {0.f, 0.f, 0.f, 0.f};
          for (int k = 0; k < n_prefix_partials; ++k) {
            const float2 v = a.partial_ml[p0 + k];
            const f32x4 ok = *reinterpret_cast<const f32x4*>(a.partial_o + (p0 + k) * kD + 4 * c4);
            const float f = (v.x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(v.x - mstar);
            denom = __builtin_fmaf(v.y, f, denom);
            sum += ok * f;
          }
          {
            const float f = (mm == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mm - mstar);
            denom = __builtin_fmaf(ll, f, denom);
            sum += o * f;
          }
          f32x4 res = {0.f, 0.f, 0.f, 0.f};
          if (denom > 0.f) res = sum * (1.0f / denom);
          if (a.out_dtype == MARL_OUT_F32) {
            *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.out) + (size_t)ridx * kD + 4 * c4) = res;
          } else {
            typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
            const bf16x4 v = {(__bf16)res[0], (__bf16)res[1], (__bf16)res[2], (__bf16)res[3]};
            *reinterpret_cast<bf16x4*>(reinterpret_cast<uint16_t*>(a.out) + (size_t)ridx * kD + 4 * c4) = v;
          }
        }
      }
    }
    // the next use of this LDS comes after the workgroup's next trip to the work queue, which
    // has barriers of its own
  } else {
    // one wave on its own: lane (i, j) holds channels 16*ct + 4*j .. +3 of q-row i
#pragma unroll
    for (int qt = 0; qt < MT; ++qt) {
      if (row_index[qt] >= 0) {
        if (!finish) {
          const size_t ps = (size_t)row_index[qt] * nslot + slot;
          float* dst = a.partial_o + ps * kD + 4 * j;
#pragma unroll
          for (int ct = 0; ct < 8; ++ct) *reinterpret_cast<f32x4*>(dst + 16 * ct) = acc[qt][ct];
          if (j == 0) a.partial_ml[ps] = make_float2(m_run[qt], l_run[qt]);
        } else {
          const size_t p0 = (size_t)row_index[qt] * nslot;
          float mstar = m_run[qt];
          for (int k = 0; k < n_prefix_partials; ++k) mstar = fmaxf(mstar, a.partial_ml[p0 + k].x);
          float denom = 0.f;
          f32x4 sum[8];
#pragma unroll
          for (int ct = 0; ct < 8; ++ct) sum[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
          for (int k = 0; k < n_prefix_partials; ++k) {
            const float2 v = a.partial_ml[p0 + k];
            const float f = (v.x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(v.x - mstar);
            denom = __builtin_fmaf(v.y, f, denom);
            const float* src = a.partial_o + (p0 + k) * kD + 4 * j;
#pragma unroll
            for (int ct = 0; ct < 8; ++ct) sum[ct] += *reinterpret_cast<const f32x4*>(src + 16 * ct) * f;
          }
          {
            const float f = (m_run[qt] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run[qt] - mstar);
            denom = __builtin_fmaf(l_run[qt], f, denom);
#pragma unroll
            for (int ct = 0; ct < 8; ++ct) sum[ct] += acc[qt][ct] * f;
          }
          const float inv = denom > 0.f ? 1.0f / denom : 0.f;
#pragma unroll
          for (int ct = 0; ct < 8; ++ct) {
            const f32x4 res = sum[ct] * inv;
            const size_t at = (size_t)row_index[qt] * kD + 16 * ct + 4 * j;
            if (a.out_dtype == MARL_OUT_F32) {
              *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.out) + at) = res;
            } else {
              typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
              const bf16x4 v = {(__bf16)res[0], (__bf16)res[1], (__bf16)res[2], (__bf16)res[3]};
              *reinterpret_cast<bf16x4*>(reinterpret_cast<uint16_t*>(a.out) + at) = v;
            }
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Suffix kernels: one work item = (sequence, chunk of its generated tokens, KV head); the
// R = Hq/Hkv query heads of that KV head are the (zero-padded) 16-row tile.
//
// The item list is sorted longest first, so it splits into a head of long items (more than
// kShortTokens tokens) and a tail of short ones.
//   suffix_kernel:       long items, one per workgroup (waves take the 32-token steps in
//                        turn), taken from the queue only when the workgroup is free
//                        (reserving an item early would undo the longest-first balancing).
//   short_suffix_items:  short items, one per wave, split round-robin over all waves of the
//                        grid with no LDS traffic, barrier or atomic, so a batch of tiny
//                        sequences does not pay a workgroup's fixed costs per sequence.
//                        Where they run: a sequence whose own tokens are one short item (the
//                        usual case) is finished in the first phase of the MERGE kernel, after
//                        the prefix partials are complete: its rows never pass through a partial.
//                        The short items of sequences with several suffix chunks must be
//                        partials before the merge kernel starts: they run as the first phase of
//                        the PREFIX kernel's workgroups (as a phase of the suffix kernel they
//                        slowed the long items' hot loop down by a few percent through the
//                        shared register allocation, and a kernel of their own cost one more
//                        launch per call).
// ---------------------------------------------------------------------------------------
#ifndef MARL_SUFFIX_WAVES_PER_EU
#define MARL_SUFFIX_WAVES_PER_EU 3
#endif
#ifndef MARL_SUFFIX_WAVES
#define MARL_SUFFIX_WAVES 4
#endif
constexpr int kSuffixWaves = MARL_SUFFIX_WAVES;   // waves that share one long item (= workgroup size / 64)
__global__ __launch_bounds__(kSuffixWaves * 64)
__attribute__((amdgpu_waves_per_eu(MARL_SUFFIX_WAVES_PER_EU, MARL_SUFFIX_WAVES_PER_EU)))
void suffix_kernel(AttnArgs a) {
  __shared__ ItemLds<1> lds;
  __shared__ int next_item;
  const int n_work = a.counters[MARL_CTR_NUM_LONG_SUFFIX_ITEMS] * a.Hkv;
  int bad_page = 0;
  // the first item of a workgroup is its block index (no trip to the shared counter, on which
  // a whole grid starting at once would queue up); later ones come from the counter
  for (bool first = true;; first = false) {
    int qi = blockIdx.x;
    if (!first) {
      if (threadIdx.x == 0) next_item = gridDim.x + atomicAdd(&a.counters[MARL_CTR_SUFFIX_CURSOR], 1);
      __syncthreads();
      qi = next_item;
      __syncthreads();
    }
    if (qi >= n_work) break;
    const int4 it = a.suffix_items[qi / a.Hkv];
    const int kvh = qi % a.Hkv;
    const int s = it.x;
    const int i = threadIdx.x & 15;
    const int row_index[1] = {i < a.R ? s * a.Hq + kvh * a.R + i : -1};
    // a sequence whose own tokens are this one item: the output rows are finished here
    const int chunks = ld_uniform(a.seq_chunks + s);
    process_item<1, kSuffixWaves>(a, a.suffix_table + (size_t)s * a.max_sp, it.y, it.z, kvh, row_index,
                                  a.NCp + it.y / a.Cs, lds, bad_page, (chunks >> 16) == 1, chunks & 0xffff);
  }
  if (bad_page) atomicOr(&a.counters[MARL_CTR_FLAGS], MARL_FLAG_BAD_PAGE);
}

// Short suffix items: wave w of the grid takes the entries n_long + w, n_long + w + W, ...
// (W = waves in the grid) with no LDS, no barrier and no atomic: the entries are sorted by
// size, so a round-robin split is balanced, and a shared queue counter would serialise
// thousands of waves on one address.  The next record is fetched while the current item runs.
// kFinish = false (first phase of the prefix kernel): the items of sequences with several
// suffix chunks, as partials.  kFinish = true (first phase of the merge kernel, after the
// prefix partials are complete): the items of sequences whose own tokens are that one item,
// finished to output rows, so that they never travel through a partial.
template <bool kFinish>
__device__ __forceinline__ void short_suffix_items(const AttnArgs& a, int& bad_page) {
  const int n_long = a.counters[MARL_CTR_NUM_LONG_SUFFIX_ITEMS] * a.Hkv;
  const int n_work = a.counters[MARL_CTR_NUM_SUFFIX_ITEMS] * a.Hkv;
  const int waves_per_block = blockDim.x >> 6;
  const int stride = gridDim.x * waves_per_block;
  int cur = n_long + blockIdx.x * waves_per_block + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (cur >= n_work) return;
  const int i = threadIdx.x & 15;
  int4 rec = a.suffix_items[cur / a.Hkv];
  while (cur < n_work) {
    const int nxt = cur + stride;
    const int4 nrec = nxt < n_work ? a.suffix_items[nxt / a.Hkv] : make_int4(0, 0, 0, 0);
    const int kvh = cur % a.Hkv;
    const int s = rec.x;
    const int chunks = ld_uniform(a.seq_chunks + s);
    if (((chunks >> 16) == 1) == kFinish) {
      const int row_index[1] = {i < a.R ? s * a.Hq + kvh * a.R + i : -1};
      ItemLds<1>* no_lds = nullptr;   // the one-wave path never touches it
      process_item<1, 1>(a, a.suffix_table + (size_t)s * a.max_sp, rec.y, rec.z, kvh, row_index,
                         a.NCp + rec.y / a.Cs, *no_lds, bad_page, kFinish, chunks & 0xffff);
    }
    cur = nxt;
    rec = nrec;
  }
}

// ---------------------------------------------------------------------------------------
// Prefix kernel: one work item = (group, chunk of prefix tokens, block of up to 128 (or 256)
// query rows, KV head).  Query row rho of a group is (its rho / R -th sequence, head kvh*R + rho % R).
//
// Here the NW (4 or 8) waves split the QUERY rows (16-row tile t belongs to wave t % NW) and
// every wave sees all tokens, so the group's K/V must reach all of them: each 32-token step (two
// pages, 16 KB of K and V) is fetched once by the workgroup with fully coalesced 16-byte
// loads (a wave reads 1 KB contiguous per instruction), staged in registers, written to a
// triple-buffered LDS tile and read back in MFMA operand layout.  Loads run three steps
// ahead (48 KB in flight per workgroup).  No cross-wave reduction is needed.
//
// LDS tile of one step (16 KB): K as 32 token rows of 256 B, the 16-byte chunk index of
// row tau XOR-ed with a 4-bit key made of bits 0, 1, 3, 4 of tau: the 16 rows that the 16 lanes
// of one operand read touch differ in exactly those bits, so they hit 16 different 16-byte bank
// groups (measured: 4.1 cycles per wave instruction per CU against 7.3 with a 3-bit key, 4.0 for
// a plain linear read); V as [page][channel][2 halves of 8 slots], the 16-byte unit index u
// XOR-ed with (u>>3)&1 for the same reason.
// ---------------------------------------------------------------------------------------
constexpr int kStepBytes = 2 * kBlockTok * kD * 2;   // K + V of one 32-token step
// the pipelined prefix item rescales its accumulators only when a row's score maximum exceeds the
// running reference by more than this (log2 units): weights then stay below 2^kRescaleSlack
constexpr float kRescaleSlack = 8.0f;
// s_waitcnt immediate (gfx9 encoding): vector-memory counter <= vm, LDS/scalar counter <= lgkm
constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 0xf) | ((vm >> 4) << 14) | (7 << 4) | ((lgkm & 0xf) << 8); }
struct PrefixLds {
  __attribute__((aligned(16))) char buf[3][kStepBytes];
};

template <int MTW, int NW>
__device__ __forceinline__ void prefix_item(const AttnArgs& a, const int4 it, const int kvh,
                                            PrefixLds& lds, int& bad_page) {
  constexpr int kQBlock = 32 * NW;              // query rows of one item: two 16-row tiles per wave
  constexpr int kLoads = 1024 / (NW * 64);      // 16-byte loads per thread and step (16 KB per step)
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i = lane & 15, j = lane >> 4;
  const int g = it.x, tok_begin = it.y, tok_end = it.z, row_begin = it.w;
  const int gstart = a.group_start[g];
  const int nrows = a.group_count[g] * a.R;
  const int32_t* table_row = a.prefix_table + (size_t)g * a.max_pp;
  const float sc = fmaxf(fabsf(a.scale) * 1.44269504088896340736f, 1e-30f);
  const uint32_t sign_flip = a.scale < 0.f ? 0x80008000u : 0u;
  const int nslot = a.NCp + a.NCs;
  const int slot = tok_begin / a.Cp;

  // this wave's tiles: wave, wave + 4, ...; nt of them hold at least one real row
  const int tiles_total = (min(kQBlock, nrows - row_begin) + 15) >> 4;
  const int nt = max(0, min(MTW, (tiles_total - wave + NW - 1) / NW));   // wave-uniform
  int row_index[MTW];
  u32x4 qreg[MTW][4];
#pragma unroll
  for (int qt = 0; qt < MTW; ++qt) {
    const int rho = row_begin + (qt * NW + wave) * 16 + i;
    int idx = -1;
    if (rho < nrows && (qt * NW + wave) * 16 < kQBlock)
      idx = a.group_seqs[gstart + rho / a.R] * a.Hq + kvh * a.R + rho % a.R;
    row_index[qt] = idx;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (idx >= 0) {
        v = *reinterpret_cast<const u32x4*>(a.q + (size_t)idx * kD + (4 * kk + j) * 8);
        v ^= sign_flip;
      }
      qreg[qt][kk] = v;
    }
  }
  f32x4 acc[MTW][8];
  float m_run[MTW], l_run[MTW];
#pragma unroll
  for (int qt = 0; qt < MTW; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) acc[qt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int nsteps = (tok_end - tok_begin + kBlockTok - 1) / kBlockTok;
  const size_t page_bytes = (size_t)a.Hkv * (kPage * kD * 2);

  // Page ids and page addresses are wave-uniform (scalar registers, a handful of scalar instructions
  // per step) and every lane adds one 32-bit offset that never changes: with two waves per SIMD the
  // instruction count of a step is a cost of its own (measured on the 8-wave shape, whose loop it
  // bounds).
  //
  // Page ids of step n: two scalar loads, unconditional (a step past the end repeats the last page,
  // and so does the second page of a step that has only one).  They are issued at the top of an
  // iteration and taken after its first wait for LDS data, which waits for scalar loads as well
  // (one counter, and scalar loads return out of order); fetched and checked in one place they
  // would cost two scalar-memory latencies per step, one after the other.
  const int first_page = tok_begin >> 4;
  const int last_page = max(first_page, (tok_end - 1) >> 4);
  uint32_t id_max = 0;   // largest id seen (as unsigned): checked against the pool once, after the loop
  auto fetch_ids = [&](int n, int& r0, int& r1) {
    r0 = ld_uniform(table_row + min(first_page + 2 * n, last_page));
    r1 = ld_uniform(table_row + min(first_page + 2 * n + 1, last_page));
  };
  // the ids as the loads use them: page 0 (bytes nobody uses, from cache) for a step past the end
  // and for an id outside the pool
  auto take_ids = [&](int n, int r0, int r1, int& p0, int& p1) {
    id_max = max(id_max, max((uint32_t)r0, (uint32_t)r1));
    const uint32_t limit = n < nsteps ? (uint32_t)a.num_pages : 0u;
    p0 = (uint32_t)r0 < limit ? r0 : 0;
    p1 = (uint32_t)r1 < limit ? r1 : 0;
    // (an empty statement the compiler may not move: without it the loads and the check sink to
    // the end of the iteration, in front of the next use, and are waited for there)
    asm volatile("" : "+s"(p0), "+s"(p1));
  };
  // A step is 1024 16-byte vectors: K of page 0, K of page 1, V of page 0, V of page 1 (256
  // each, contiguous in memory).  Thread tid fetches vectors tid + k * (threads), k < kLoads.
  // Of a page's 256 vectors, vector w is slot w/16, chunk w%16 of K, or 16-byte unit w of V.
  // Which of the four regions a load belongs to is the same for a whole wave.
  static_assert(NW % 4 == 0, "a wave's 64 vectors must lie in one 256-vector region");
  const int w = tid & 255;
  const uint32_t lane_off = (uint32_t)kvh * (kPage * kD * 2) + (uint32_t)w * 16;
  auto region_of = [&](int k) { return NW == 4 ? k : k * (NW / 4) + (wave >> 2); };   // wave-uniform
  int lds_off[kLoads];
#pragma unroll
  for (int k = 0; k < kLoads; ++k) {
    const int region = region_of(k);
    const bool is_v = region >> 1;
    // K rows of page 1 are tau = 16 + slot; swizzle key of row tau: bits 0, 1, 3, 4 of tau
    const int slot = w >> 4;
    const int key = ((region & 1) << 3) | ((slot >> 3) << 2) | (slot & 3);
    lds_off[k] = is_v ? 2 * kBlockTok * kD + (region & 1) * 4096 + ((w ^ ((w >> 3) & 1)) << 4)
                      : ((region & 1) * 16 + slot) * 256 + (((w & 15) ^ key) << 4);
  }
  // The loads are unconditional so that every wait in the loop knows exactly how many younger loads
  // are in flight.
  auto issue = [&](int p0, int p1, u32x4 (&st)[kLoads]) {
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const int region = region_of(k);
      const char* base = reinterpret_cast<const char*>((region >> 1) ? a.v_pages : a.k_pages) +
                         (size_t)(uint32_t)((region & 1) ? p1 : p0) * page_bytes;   // scalar
      st[k] = ld_stream(base + lane_off);
    }
  };
  auto stage_to_lds = [&](const u32x4 (&st)[kLoads], char* buf) {
#pragma unroll
    for (int k = 0; k < kLoads; ++k) *reinterpret_cast<u32x4*>(buf + lds_off[k]) = st[k];
  };
  // operand reads: K row tau = 8*(i/4) + 4T + i%4, whose swizzle key is i
  const int k_rd = (8 * (i >> 2) + (i & 3)) * 256;
  const int v_rd = 2 * kBlockTok * kD + (j >> 1) * 4096;

  int r0, r1;   // ids in flight: those of the step that the next iteration requests
  int p0, p1;   // the ids the next request uses
  auto compute = [&](int n, const char* buf) {
    const int t0 = tok_begin + n * kBlockTok;
    const bool ragged = t0 + kBlockTok > tok_end;   // wave-uniform; only the chunk's last step
    u32x4 pb[MTW];
    if (nt == 0) take_ids(n + 4, r0, r1, p0, p1);   // (a wave without tiles only moves data)
    {
      u32x4 kr[2][4];
#pragma unroll
      for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          kr[T][kk] = *reinterpret_cast<const u32x4*>(buf + k_rd + T * 4 * 256 + (((4 * kk + j) ^ i) << 4));
#pragma unroll
      for (int qt = 0; qt < MTW; ++qt) {
        pb[qt] = u32x4{0u, 0u, 0u, 0u};
        if (qt < nt) {   // wave-uniform
          f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            s0 = mfma_16x16x32(kr[0][kk], qreg[qt][kk], s0);
            s1 = mfma_16x16x32(kr[1][kk], qreg[qt][kk], s1);
          }
          if (qt == 0) take_ids(n + 4, r0, r1, p0, p1);   // (the K reads have been waited for)
          if (ragged) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if (t0 + 8 * j + e >= tok_end) s0[e] = -INFINITY;
              if (t0 + 8 * j + 4 + e >= tok_end) s1[e] = -INFINITY;
            }
          }
          float mx = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                           fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
          mx = rows_allreduce_max(mx);
          const float m_new = fmaxf(m_run[qt], mx * sc);
          const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_new);
          float p[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[e], sc, -m_new));
            p[4 + e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[e], sc, -m_new));
          }
          const float psum = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
          if (__builtin_amdgcn_ballot_w64(m_new > m_run[qt]) != 0) {   // wave-uniform
#pragma unroll
            for (int ct = 0; ct < 8; ++ct) acc[qt][ct] *= alpha;
          }
          l_run[qt] = l_run[qt] * alpha + psum;
          m_run[qt] = m_new;
          pb[qt] = u32x4{pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
        }
      }
    }
    u32x4 vr[8];
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) {
      const int u = 2 * (16 * ct + i) + (j & 1);
      vr[ct] = *reinterpret_cast<const u32x4*>(buf + v_rd + ((u ^ ((i >> 2) & 1)) << 4));
    }
    if (ragged) {
      // value slots no token owns may hold anything (NaN included): zero them
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const int tok = t0 + 8 * j + 2 * d;
        const uint32_t mask = (tok < tok_end ? 0x0000ffffu : 0u) | (tok + 1 < tok_end ? 0xffff0000u : 0u);
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) vr[ct][d] &= mask;
      }
    }
#pragma unroll
    for (int qt = 0; qt < MTW; ++qt)
      if (qt < nt) {
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) acc[qt][ct] = mfma_16x16x32(vr[ct], pb[qt], acc[qt][ct]);
      }
  };

  // Three register stages and three LDS buffers: while step n is computed from buffer n%3,
  // the loads of steps n+1, n+2 and n+3 are in flight (48 KB per workgroup); step n+1 moves
  // from its registers to buffer (n+1)%3 at the end of the iteration, one barrier per step.
  u32x4 st0[kLoads], st1[kLoads], st2[kLoads];
  fetch_ids(0, r0, r1);
  take_ids(0, r0, r1, p0, p1);
  issue(p0, p1, st0);
  fetch_ids(1, r0, r1);
  take_ids(1, r0, r1, p0, p1);
  issue(p0, p1, st1);
  fetch_ids(2, r0, r1);
  take_ids(2, r0, r1, p0, p1);
  issue(p0, p1, st2);
  fetch_ids(3, r0, r1);
  take_ids(3, r0, r1, p0, p1);
  stage_to_lds(st0, lds.buf[0]);
  __syncthreads();
  for (int n = 0; n < nsteps; n += 3) {
    issue(p0, p1, st0);          // step n+3
    fetch_ids(n + 4, r0, r1);
    compute(n, lds.buf[0]);      // (takes the ids of step n+4)
    stage_to_lds(st1, lds.buf[1]);
    __syncthreads();
    if (n + 1 < nsteps) {
      issue(p0, p1, st1);        // step n+4
      fetch_ids(n + 5, r0, r1);
      compute(n + 1, lds.buf[1]);
      stage_to_lds(st2, lds.buf[2]);
      __syncthreads();
    }
    if (n + 2 < nsteps) {
      issue(p0, p1, st2);        // step n+5
      fetch_ids(n + 6, r0, r1);
      compute(n + 2, lds.buf[2]);
      stage_to_lds(st0, lds.buf[0]);
      __syncthreads();
    }
  }
  if (id_max >= (uint32_t)a.num_pages) bad_page = 1;
  // a workgroup-wide barrier has been passed since the last LDS read: the next item may
  // overwrite the buffers

#pragma unroll
  for (int qt = 0; qt < MTW; ++qt) {
    const float l = rows_allreduce_sum(l_run[qt]);
    if (row_index[qt] >= 0) {
      const size_t ps = (size_t)row_index[qt] * nslot + slot;
      float* dst = a.partial_o + ps * kD + 4 * j;
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) *reinterpret_cast<f32x4*>(dst + 16 * ct) = acc[qt][ct];
      if (j == 0) a.partial_ml[ps] = make_float2(m_run[qt], l);
    }
  }
}

// Prefix item, software-pipelined.  Data path as before (global memory -> staging registers, three
// steps ahead -> LDS ring of three step buffers -> operand registers); what changes is the order
// inside an iteration, chosen so that no LDS read is waited for where it is issued and so that the
// K and V operand registers share one set of 32 registers:
//   iteration n:  loads of step n+3 -> staging registers
//                 output products of step n-1, first half  (its V and weights are in registers)
//                 read K(n), first half   (into the V registers the first half has released)
//                 output products of step n-1, second half
//                 read K(n), second half
//                 score products of step n (first the half whose K has arrived)
//                 read V(n)               (into the K registers)
//                 softmax of step n       (covers the V read; leaves the bf16 weights)
//                 step n+1: staging registers -> LDS; workgroup barrier
// The hot loop has no per-tile branch (the number of active tiles is a template parameter), the
// ragged last step is peeled, and accumulators are rescaled only when a row's score maximum exceeds
// the running reference by more than 2^tau (weights stay below 2^tau), right before the output
// products that need it, so that branch is taken a handful of times per chunk.  Row sums come out
// of the matrix core (a product with an all-ones tile), from the same bf16-rounded weights that
// multiply V.
template <int MTW, int NW>
__device__ __forceinline__ void prefix_item_pipelined(const AttnArgs& a, const int4 it, const int kvh,
                                               PrefixLds& lds, int& bad_page) {
  constexpr int kQBlock = 32 * NW;
  constexpr int kLoads = 1024 / (NW * 64);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i = lane & 15, j = lane >> 4;
  const int g = it.x, tok_begin = it.y, tok_end = it.z, row_begin = it.w;
  const int32_t* table_row = a.prefix_table + (size_t)g * a.max_pp;
  const int nsteps = (tok_end - tok_begin + kBlockTok - 1) / kBlockTok;
  const size_t page_bytes = (size_t)a.Hkv * (kPage * kD * 2);

  // Page ids, as in the plain item; here a wave's loads of a step all belong to one page (the
  // waves of the lower half of the workgroup fetch the step's first page, the others its second),
  // so a wave needs one id per step.
  const int first_page = tok_begin >> 4;
  const int last_page = max(first_page, (tok_end - 1) >> 4);
  const int my_half = NW == 8 ? (wave >> 2) : 0;
  uint32_t id_max = 0;
  auto fetch_ids = [&](int n, int& r0, int& r1) {
    if constexpr (NW == 8) {
      r0 = ld_uniform(table_row + min(first_page + 2 * n + my_half, last_page));
      r1 = r0;
    } else {
      r0 = ld_uniform(table_row + min(first_page + 2 * n, last_page));
      r1 = ld_uniform(table_row + min(first_page + 2 * n + 1, last_page));
    }
  };
  auto take_ids = [&](int n, int r0, int r1, int& p0, int& p1) {
    id_max = max(id_max, max((uint32_t)r0, (uint32_t)r1));
    const uint32_t limit = n < nsteps ? (uint32_t)a.num_pages : 0u;
    p0 = (uint32_t)r0 < limit ? r0 : 0;
    p1 = (uint32_t)r1 < limit ? r1 : 0;
    asm volatile("" : "+s"(p0), "+s"(p1));   // (keeps the loads and the check where they are written)
  };
  // A step is 1024 16-byte vectors: K of page 0, K of page 1, V of page 0, V of page 1 (256 each,
  // contiguous in memory).  Thread tid fetches vectors tid + k * threads, k < kLoads.  Of a page's
  // 256 vectors, vector w is slot w/16, chunk w%16 of K, or 16-byte unit w of V.
  // LDS tile: K as 32 token rows of 256 B, the 16-byte chunk index XOR-ed with a 4-bit key made of
  // bits 0, 1, 3, 4 of the row (the 16 rows one operand read touches differ exactly in those bits,
  // so its 16 lanes hit 16 different bank groups); V as [page][channel][2 halves of 8 slots], the
  // unit index u XOR-ed with (u >> 3) & 1.
  // Which of the four regions a load belongs to is the same for a whole wave (wave-uniform), so a
  // page's base address is scalar arithmetic and every lane adds the same 32-bit offset for all loads.
  static_assert(NW % 4 == 0, "a wave's 64 vectors must lie in one 256-vector region");
  const int w = tid & 255;
  const uint32_t lane_off = (uint32_t)kvh * (kPage * kD * 2) + (uint32_t)w * 16;
  const int sl = w >> 4;
  const int lds_k = sl * 256 + (((w & 15) ^ (((sl >> 3) << 2) | (sl & 3))) << 4);   // page 0; page 1: + 4096, chunk ^ 8
  const int lds_v = 2 * kBlockTok * kD + ((w ^ ((w >> 3) & 1)) << 4);              // page 0; page 1: + 4096
  auto region_of = [&](int k) { return NW == 4 ? k : k * (NW / 4) + (wave >> 2); };   // wave-uniform
  // (unconditional loads: a step past the end reads page 0, bytes nobody uses, from cache, so that
  // every wait knows how many loads are in flight)
  auto issue = [&](int p0, int p1, u32x4 (&st)[kLoads]) {
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const int region = region_of(k);
      const int pid = NW == 8 ? p0 : ((region & 1) ? p1 : p0);   // (with 8 waves p0 is this wave's page)
      const char* base = reinterpret_cast<const char*>((region >> 1) ? a.v_pages : a.k_pages) +
                         (size_t)(uint32_t)pid * page_bytes;   // scalar
      st[k] = ld_stream(base + lane_off);
    }
  };
  auto stage_to_lds = [&](const u32x4 (&st)[kLoads], char* buf) {
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const int region = region_of(k);
      const int off = (region >> 1) ? lds_v + (region & 1) * 4096 : (lds_k + (region & 1) * 4096) ^ ((region & 1) << 7);
      *reinterpret_cast<u32x4*>(buf + off) = st[k];
    }
  };
  // the first three steps are requested before anything else of the item: the chain of dependent
  // loads that leads to the query rows then runs while they are in flight
  u32x4 st[3][kLoads];   // steps in flight: three register stages
  int p0, p1, r0, r1;
#pragma unroll
  for (int s0 = 0; s0 < 3; ++s0) {
    fetch_ids(s0, r0, r1);
    take_ids(s0, r0, r1, p0, p1);
    issue(p0, p1, st[s0]);
  }
  fetch_ids(3, r0, r1);
  take_ids(3, r0, r1, p0, p1);

  const int gstart = a.group_start[g];
  const int nrows = a.group_count[g] * a.R;
  const float sc = fmaxf(fabsf(a.scale) * 1.44269504088896340736f, 1e-30f);
  const uint32_t sign_flip = a.scale < 0.f ? 0x80008000u : 0u;
  const int nslot = a.NCp + a.NCs;
  const int slot = tok_begin / a.Cp;
  const int tiles_total = (min(kQBlock, nrows - row_begin) + 15) >> 4;
  const int nt = max(0, min(MTW, (tiles_total - wave + NW - 1) / NW));   // wave-uniform
  int row_index[MTW];
  u32x4 qreg[MTW][4];
#pragma unroll
  for (int qt = 0; qt < MTW; ++qt) {
    const int rho = row_begin + (qt * NW + wave) * 16 + i;
    int idx = -1;
    if (rho < nrows && (qt * NW + wave) * 16 < kQBlock)
      idx = a.group_seqs[gstart + rho / a.R] * a.Hq + kvh * a.R + rho % a.R;
    row_index[qt] = idx;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (idx >= 0) {
        v = *reinterpret_cast<const u32x4*>(a.q + (size_t)idx * kD + (4 * kk + j) * 8);
        v ^= sign_flip;
      }
      qreg[qt][kk] = v;
    }
  }
  f32x4 acc[MTW][8];
  f32x4 lacc[MTW];          // row sums accumulated by the matrix core (all four elements equal)
  float m_run[MTW];
#pragma unroll
  for (int qt = 0; qt < MTW; ++qt) {
    m_run[qt] = -INFINITY;
    lacc[qt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) acc[qt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int k_rd = (8 * (i >> 2) + (i & 3)) * 256;
  const int v_rd = 2 * kBlockTok * kD + (j >> 1) * 4096;
  auto read_k_half = [&](const char* buf, int T, u32x4 (&kr)[4]) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      kr[kk] = *reinterpret_cast<const u32x4*>(buf + k_rd + T * 4 * 256 + (((4 * kk + j) ^ i) << 4));
  };
  auto read_v_half = [&](const char* buf, int h, u32x4 (&vr)[4]) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int u = 2 * (16 * (4 * h + c) + i) + (j & 1);
      vr[c] = *reinterpret_cast<const u32x4*>(buf + v_rd + ((u ^ ((i >> 2) & 1)) << 4));
    }
  };
  const u32x4 ones = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};

  auto run = [&](auto nt_tag) {
    constexpr int NTraw = decltype(nt_tag)::value;
    constexpr int NT = NTraw > 0 ? NTraw : 1;   // (no zero-length arrays; a wave without tiles only moves data)
    // xa / xb: the two halves of the operand registers: V(n-1) channel tiles 0-3 / 4-7 at the top of
    // iteration n, then K(n) token half 0 / 1, then V(n)
    u32x4 xa[4], xb[4], pb[NT];
    float alpha_pending[NT];
    bool rescale_pending = false;   // wave-uniform

    auto rescale_if_pending = [&]() {
      if (rescale_pending) {
#pragma unroll
        for (int qt = 0; qt < NT; ++qt) {
#pragma unroll
          for (int ct = 0; ct < 8; ++ct) acc[qt][ct] *= alpha_pending[qt];
          lacc[qt] *= alpha_pending[qt];
        }
      }
    };
    auto output_half = [&](int h, const u32x4 (&vr)[4]) {
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int qt = 0; qt < NT; ++qt) acc[qt][4 * h + c] = mfma_16x16x32(vr[c], pb[qt], acc[qt][4 * h + c]);
      if (h == 0) {
#pragma unroll
        for (int qt = 0; qt < NT; ++qt) lacc[qt] = mfma_16x16x32(ones, pb[qt], lacc[qt]);
      }
    };
    auto scores_half = [&](int T, const u32x4 (&kr)[4], f32x4 (&s)[NT][2]) {
#pragma unroll
      for (int qt = 0; qt < NT; ++qt) s[qt][T] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int qt = 0; qt < NT; ++qt) s[qt][T] = mfma_16x16x32(kr[kk], qreg[qt][kk], s[qt][T]);
    };
    // softmax of step n from its scores: leaves the bf16 weights in pb (and masks, in the ragged last
    // step, the scores and the value slots no token owns)
    auto softmax = [&](auto last_tag, int n, f32x4 (&s)[NT][2]) {
      constexpr bool kLast = decltype(last_tag)::value;
      if constexpr (kLast) {
        const int t0 = tok_begin + n * kBlockTok;
        if (t0 + kBlockTok > tok_end) {   // wave-uniform: the ragged end of the chunk
#pragma unroll
          for (int qt = 0; qt < NT; ++qt)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if (t0 + 8 * j + e >= tok_end) s[qt][0][e] = -INFINITY;
              if (t0 + 8 * j + 4 + e >= tok_end) s[qt][1][e] = -INFINITY;
            }
          // value slots no token owns may hold anything (NaN included): zero them
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            const int tok = t0 + 8 * j + 2 * d;
            const uint32_t mask = (tok < tok_end ? 0x0000ffffu : 0u) | (tok + 1 < tok_end ? 0xffff0000u : 0u);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              xa[c][d] &= mask;
              xb[c][d] &= mask;
            }
          }
        }
      }
      float mx[NT];
      bool moved = false;
#pragma unroll
      for (int qt = 0; qt < NT; ++qt) {
        const f32x4 s0 = s[qt][0], s1 = s[qt][1];
        mx[qt] = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                       fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3]))) * sc;   // this lane's 8 tokens
        moved |= mx[qt] > m_run[qt] + kRescaleSlack;
      }
      // (the rows' maxima, a reduction over the four lanes of a row, are needed only when some lane
      // has seen a score that far above its row's reference)
      rescale_pending = __builtin_amdgcn_ballot_w64(moved) != 0;   // wave-uniform; rare after a chunk's first step
      if (rescale_pending) {
#pragma unroll
        for (int qt = 0; qt < NT; ++qt) {
          mx[qt] = rows_allreduce_max(mx[qt]);
          const float m_new = mx[qt] > m_run[qt] + kRescaleSlack ? mx[qt] : m_run[qt];
          alpha_pending[qt] = __builtin_amdgcn_exp2f(m_run[qt] - m_new);   // 1 where the row did not move
          m_run[qt] = m_new;
        }
      }
#pragma unroll
      for (int qt = 0; qt < NT; ++qt) {
        float p[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qt][0][e], sc, -m_run[qt]));
          p[4 + e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qt][1][e], sc, -m_run[qt]));
        }
        pb[qt] = u32x4{pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
      }
    };
    // iteration n (n % 3 == PH): buf[PH] holds step n; the staging set PH takes the loads of step
    // n+3; set PH+1 (step n+1) goes to buf[PH+1]
    auto iteration = [&](auto first_tag, auto last_tag, auto phase_tag, int n) {
      constexpr bool kFirst = decltype(first_tag)::value;
      constexpr int PH = decltype(phase_tag)::value;
      const char* bufr = lds.buf[PH];
      char* bufw = lds.buf[(PH + 1) % 3];
      issue(p0, p1, st[PH]);
      fetch_ids(n + 4, r0, r1);
      if constexpr (NTraw == 0) take_ids(n + 4, r0, r1, p0, p1);
      if constexpr (NTraw > 0) {
        f32x4 s[NT][2];
        if constexpr (!kFirst) {
          rescale_if_pending();
          output_half(0, xa);
          __builtin_amdgcn_sched_barrier(0);
        }
        read_k_half(bufr, 0, xa);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (!kFirst) {
          output_half(1, xb);
          __builtin_amdgcn_sched_barrier(0);
        }
        read_k_half(bufr, 1, xb);
        __builtin_amdgcn_sched_barrier(0);
        scores_half(0, xa, s);
        __builtin_amdgcn_sched_barrier(0);
        scores_half(1, xb, s);
        take_ids(n + 4, r0, r1, p0, p1);   // (all of K has been waited for, and the scalar loads with it)
        __builtin_amdgcn_sched_barrier(0);
        read_v_half(bufr, 0, xa);
        read_v_half(bufr, 1, xb);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (decltype(last_tag)::value)
          __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));   // the ragged step masks the values it has just read
        softmax(last_tag, n, s);
      }
      // step n+1 goes from its staging registers to LDS once it has landed (the loads of the two
      // younger steps stay in flight), then the barrier
      __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * kLoads, 15));
      stage_to_lds(st[(PH + 1) % 3], bufw);
      __syncthreads();
    };
    const std::true_type yes{};
    const std::false_type no{};
    using P0 = std::integral_constant<int, 0>;

    // step 0 into LDS
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * kLoads, 15));
    stage_to_lds(st[0], lds.buf[0]);
    __syncthreads();
    if (nsteps == 1) {
      iteration(yes, yes, P0{}, 0);
    } else {
      iteration(yes, no, P0{}, 0);
      int n = 1;
      // the steps that are neither first nor last, phases 1, 2, ..., 3-1, 0 in turn
      auto middle = [&](auto ph) {
        if (n + 1 >= nsteps) return false;
        iteration(no, no, ph, n);
        ++n;
        return true;
      };
      auto cycle = [&](auto... ph) { return (middle(ph) && ...); };
      while (n + 1 < nsteps) {
        cycle(std::integral_constant<int, 1>{}, std::integral_constant<int, 2>{}, P0{});
      }
      const int last = nsteps - 1;
      const int lp = last % 3;
      if (lp == 0) iteration(no, yes, P0{}, last);
      else if (lp == 1) iteration(no, yes, std::integral_constant<int, 1>{}, last);
      else iteration(no, yes, std::integral_constant<int, 2>{}, last);
    }
    if constexpr (NTraw > 0) {   // the last step's output products
      rescale_if_pending();
      output_half(0, xa);
      output_half(1, xb);
    }
    // every wave has passed a barrier since its last LDS read: the next item may refill the ring
  };
  if (nt == MTW) run(std::integral_constant<int, MTW>{});
  else if (MTW == 2 && nt == 1) run(std::integral_constant<int, 1>{});
  else run(std::integral_constant<int, 0>{});
  if (id_max >= (uint32_t)a.num_pages) bad_page = 1;

#pragma unroll
  for (int qt = 0; qt < MTW; ++qt) {
    if (row_index[qt] >= 0) {
      const size_t ps = (size_t)row_index[qt] * nslot + slot;
      float* dst = a.partial_o + ps * kD + 4 * j;
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) *reinterpret_cast<f32x4*>(dst + 16 * ct) = acc[qt][ct];
      if (j == 0) a.partial_ml[ps] = make_float2(m_run[qt], lacc[qt][0]);
    }
  }
}

template <int NW>
__device__ __forceinline__ void prefix_kernel_body(const AttnArgs& a) {
  __shared__ PrefixLds lds;
  __shared__ int next_item;
  const int n_work = a.counters[MARL_CTR_NUM_PREFIX_ITEMS] * a.Hkv;
  int bad_page = 0;
  // The short suffix items go first: each round is a chain of dependent memory accesses with
  // little data, which is cheap while every workgroup has other work to overlap it with and
  // expensive at the tail of a kernel, where only a few workgroups are left.
  // (skipped when the plan found no such item: the scan of the short entries is a chain of
  // dependent loads at the very start of the kernel)
  if (a.counters[MARL_CTR_NUM_SHORT_PARTIAL_ITEMS] > 0) short_suffix_items<false>(a, bad_page);
  __syncthreads();
  for (bool first = true;; first = false) {   // first item = block index, as in the suffix kernel
    int qi = blockIdx.x;
    if (!first) {
      if (threadIdx.x == 0) next_item = gridDim.x + atomicAdd(&a.counters[MARL_CTR_PREFIX_CURSOR], 1);
      __syncthreads();
      qi = next_item;
      __syncthreads();
    }
    if (qi >= n_work) break;
    const int4 it = a.prefix_items[qi / a.Hkv];
    const int kvh = qi % a.Hkv;
    const int rows = min(32 * NW, a.group_count[it.x] * a.R - it.w);
    // (workgroup-uniform)  The 8-wave shape, whose items are bound by the matrix and vector units,
    // runs the pipelined item; the 4-wave shape, bound by HBM, the plain one (measured faster there).
    if constexpr (NW == 8) {
      if (rows <= 16 * NW) prefix_item_pipelined<1, NW>(a, it, kvh, lds, bad_page);
      else prefix_item_pipelined<2, NW>(a, it, kvh, lds, bad_page);
    } else {
      if (rows <= 16 * NW) prefix_item<1, NW>(a, it, kvh, lds, bad_page);
      else prefix_item<2, NW>(a, it, kvh, lds, bad_page);
    }
  }
  if (bad_page) atomicOr(&a.counters[MARL_CTR_FLAGS], MARL_FLAG_BAD_PAGE);
}

// Two shapes of the same kernel: 4 waves and blocks of 128 query rows (two workgroups per CU),
// or 8 waves and blocks of 256 rows (one workgroup per CU) for groups with more than 128 rows,
// whose prefix KV would otherwise be streamed once per 128-row block.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void prefix_kernel(AttnArgs a) { prefix_kernel_body<4>(a); }
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void prefix_kernel_wide(AttnArgs a) { prefix_kernel_body<8>(a); }

// ---------------------------------------------------------------------------------------
// Merge kernel: the second reduction of split-KV decode attention.  For every (sequence,
// query head) it combines the partials of the group's prefix chunks and of the sequence's
// own suffix chunks, in slot order (so the sum order never changes between runs):
//   m* = max_i m_i,  out = sum_i O_i 2^(m_i - m*) / sum_i l_i 2^(m_i - m*)
// (m in log2 units).  A row without any token gives zeros.  Rows of a sequence whose own tokens
// are a single item are written where that item is processed (the suffix kernel, or this
// kernel's first phase for short items) and are not touched by the row loop.
//
// The kernel is a chain of dependent loads with almost no arithmetic, so it is organised to
// keep that chain short: the plan kernel has already stored each sequence's chunk counts
// (one load instead of group id -> prefix length), half a wave handles one row with 16-byte
// loads, and the first four partials of a row (max/sum and output) are all requested before
// any of them is used.  Every lane recomputes the few scalar weights itself: no shuffles.
// ---------------------------------------------------------------------------------------
constexpr int kMergeThreads = 256;
constexpr int kRowsPerBlock = kMergeThreads / 32;
constexpr int kEager = 4;   // partials fetched up front

__global__ __launch_bounds__(kMergeThreads) __attribute__((amdgpu_waves_per_eu(3, 3)))
void merge_kernel(AttnArgs a) {
  // first the sequences whose own tokens are one short item: attention over those tokens and
  // the merge with the group's prefix partials in one go, one item per wave
  {
    int bad_page = 0;
    short_suffix_items<true>(a, bad_page);
    if (bad_page) atomicOr(&a.counters[MARL_CTR_FLAGS], MARL_FLAG_BAD_PAGE);
  }
  const int sub = threadIdx.x & 31;   // lane within the half wave: channels 4*sub .. 4*sub+3
  const int row = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 5);
  if (row >= a.NS * a.Hq) return;
  const int s = row / a.Hq;
  const int info = a.seq_chunks[s];
  const int npc = info & 0xffff, nsc = info >> 16;
  // a sequence whose own tokens are one item was finished where that item was processed: above
  // (at most kShortTokens tokens) or in the suffix kernel
  if (nsc == 1) return;
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

int prefix_blocks_per_cu(bool wide) {
  int n = 0;
  const hipError_t e = wide ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, prefix_kernel_wide, 512, 0)
                            : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, prefix_kernel, 256, 0);
  if (e != hipSuccess || n < 1) n = 1;
  return n;
}
int suffix_blocks_per_cu() {
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, suffix_kernel, kSuffixWaves * 64, 0) != hipSuccess || n < 1) n = 1;
  return n;
}

hipError_t launch_prefix(const AttnArgs& a, int grid, hipStream_t st) {
  if (a.qblock_rows == 256) hipLaunchKernelGGL(prefix_kernel_wide, dim3(grid), dim3(512), 0, st, a);
  else hipLaunchKernelGGL(prefix_kernel, dim3(grid), dim3(256), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_suffix(const AttnArgs& a, int grid, hipStream_t st) {
  hipLaunchKernelGGL(suffix_kernel, dim3(grid), dim3(kSuffixWaves * 64), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_merge(const AttnArgs& a, hipStream_t st) {
  const long rows = (long)a.NS * a.Hq;
  if (rows == 0) return hipSuccess;
  const int grid = (int)((rows + kRowsPerBlock - 1) / kRowsPerBlock);
  hipLaunchKernelGGL(merge_kernel, dim3(grid), dim3(kMergeThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
