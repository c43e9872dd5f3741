// Prefill (prompt) attention over the paged KV cache, and the scatter that puts a prompt's
// keys and values into its pages.  This is the step that creates, once per prompt, the prefix
// every sample of that prompt then shares (Parallel Sampling, Section 5.1 of the paper); the
// paper leaves the computation to its inference backend, so the operation is the textbook
// causal attention stated in marl_decode.h:
//   query token at position t of group g attends to positions 0..t of the group's pages.
// A group may bring only a chunk of its prompt (positions pos0 .. pos0+n-1): the earlier
// positions are then context that is already in the cache (chunked prefill).
//
// Structure.  Query rows of a (group, KV head) are flattened as rho = token * R + head-in-group
// and cut into equal blocks of at most kQB = 192 rows; one work item = (group, row block, KV
// head).  The item streams keys/values 0 .. (last position of the block) through a ring of four
// LDS step buffers, 32 tokens (two pages, 16 KB) per step, in the XOR-swizzled layout of the
// decode prefix kernel; the four waves split the block's 16-row tiles (up to three each).  The
// steps go from global memory straight into LDS (global_load_lds_dwordx4, no staging
// registers), which is what leaves room for the third tile: the kernel is bound by the LDS
// operand reads (every wave reads the whole step for its rows), so more rows per wave is what
// makes it faster.  Causality costs little: a block spans kQB / R consecutive tokens, so only
// its last one or two steps need the per-row mask, and a tile skips steps that lie entirely
// beyond its rows.  A block sees all of its keys, so the output is normalised and written
// directly (no partials, no merge).
//
// Work distribution: a one-workgroup plan kernel turns q_start into the running number of
// row blocks per group and lists the blocks (group, first row), inside a group last-first
// (most keys first); workgroups then draw (block, KV head) indices from a counter.
#include "marl_internal.h"
#include "wave_ops.h"

namespace marl {
namespace {

#ifndef MARL_PREFILL_MT
#define MARL_PREFILL_MT 3
#endif
#ifndef MARL_PREFILL_NW
#define MARL_PREFILL_NW 4
#endif
#ifndef MARL_PREFILL_WAVES_PER_EU
#define MARL_PREFILL_WAVES_PER_EU 2
#endif
constexpr int kMT = MARL_PREFILL_MT;          // 16-row tiles per wave
constexpr int kNW = MARL_PREFILL_NW;          // waves per workgroup
constexpr int kQB = 16 * kMT * kNW;           // most query rows of one work item
constexpr int kPfThreads = 64 * kNW;
constexpr int kPfStepBytes = 2 * kBlockTok * kD * 2;   // K + V of one 32-token step
constexpr int kPlanThreadsPf = 1024;

// LDS step buffers, filled by direct global-to-LDS loads (two workgroups of 64 KB per CU)
constexpr int kPfStages = 4;
struct PrefillLds {
  __attribute__((aligned(16))) char buf[kPfStages][kPfStepBytes];
};
// s_waitcnt immediate that waits only for the vector-memory counter to drop to n (gfx9 encoding)
constexpr int pf_vmcnt_imm(int n) { return (n & 0xf) | ((n >> 4) << 14) | (7 << 4) | (0xf << 8); }

// counters at the head of the workspace (same slots as the decode plan uses, so that
// marl_attn_read_flags reads this workspace too); block_start[NG + 1] follows the header
constexpr int kPfCursor = MARL_CTR_PREFIX_CURSOR, kPfFlags = MARL_CTR_FLAGS;

// n_g usable query tokens of group g (clamped to the q array and to the table row)
__device__ __forceinline__ int group_tokens(const PrefillArgs& a, int g, int& flag) {
  const int b = a.q_start[g], e = a.q_start[g + 1], p0 = a.q_pos0[g];
  int n = e - b;
  if (b < 0 || e > a.NT || n < 0 || p0 < 0) { flag |= MARL_FLAG_BAD_GROUP; return 0; }
  const long room = (long)a.max_pp * kPage - p0;
  if (n > room) { flag |= MARL_FLAG_LEN_CLAMPED; n = room > 0 ? (int)room : 0; }
  return n;
}

// A group's nrows query rows are cut into ceil(nrows / kQB) blocks of equal size (a multiple of
// 16 rows), not into full blocks and a remainder: 224 rows are two blocks of 112 (7 tiles each
// over the waves), not 192 + 32.
__device__ __forceinline__ int blocks_of(long nrows) { return (int)((nrows + kQB - 1) / kQB); }
__device__ __forceinline__ int block_rows(long nrows) {
  const long nb = (nrows + kQB - 1) / kQB;
  return nb ? (int)(((nrows + nb - 1) / nb + 15) / 16 * 16) : 0;
}

__global__ __launch_bounds__(kPlanThreadsPf) void prefill_plan_kernel(PrefillArgs a) {
  __shared__ long long part[kPlanThreadsPf];   // 64-bit: inconsistent inputs must not wrap the sums
  __shared__ long long carry;
  __shared__ int flags_all, end_all;
  const int tid = threadIdx.x;
  int flag = 0;
  if (tid == 0) { carry = 0; flags_all = end_all = 0; }
  __syncthreads();
  for (int g0 = 0; g0 < a.NG; g0 += kPlanThreadsPf) {
    const int g = g0 + tid;
    int nb = 0;
    long nrows = 0;
    if (g < a.NG) {
      nrows = (long)group_tokens(a, g, flag) * a.R;
      nb = blocks_of(nrows);
    }
    // groups that overlap in q could ask for more blocks than the workspace was sized for
    // (its bound assumes they share no rows): such a group is dropped
    if (nb > a.max_blocks) { nb = 0; flag |= MARL_FLAG_BAD_GROUP; }
    part[tid] = nb;
    __syncthreads();
    for (int d = 1; d < kPlanThreadsPf; d <<= 1) {   // inclusive scan
      const long long v = tid >= d ? part[tid - d] : 0;
      __syncthreads();
      part[tid] += v;
      __syncthreads();
    }
    if (g < a.NG) {
      const long long first64 = carry + part[tid] - nb;
      int first = a.max_blocks;
      if (first64 + nb > a.max_blocks) {   // as above; every later group then fails this test too
        flag |= MARL_FLAG_BAD_GROUP;
        nb = 0;
      } else {
        first = (int)first64;
        atomicMax(&end_all, first + nb);
      }
      a.block_start[g] = first;
      // the group's work items, last row block (most keys) first
      const int qb = block_rows(nrows);
      for (int k = 0; k < nb; ++k) a.items[first + k] = make_int2(g, (nb - 1 - k) * qb);
    }
    __syncthreads();
    if (tid == kPlanThreadsPf - 1) carry += part[tid];
    __syncthreads();
  }
  if (flag) atomicOr(&flags_all, flag);
  __syncthreads();
  if (tid == 0) {
    a.block_start[a.NG] = end_all;   // the accepted groups' blocks are exactly [0, end_all)
    a.counters[kPfCursor] = 0;
    a.counters[kPfFlags] = flags_all;   // the attention kernel may add MARL_FLAG_BAD_PAGE
  }
}

__device__ __forceinline__ void prefill_item(const PrefillArgs& a, const int g, const int row_begin,
                                             const int kvh, PrefillLds& lds, int& bad_page) {
  constexpr int kLoads = 1024 / (kNW * 64);     // 16-byte loads per thread and step (16 KB per step)
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i = lane & 15, j = lane >> 4;
  int unused = 0;
  const int ntok = group_tokens(a, g, unused);
  const int nrows = ntok * a.R;
  const int qrow0 = a.q_start[g];
  const int pos0 = a.q_pos0[g];
  const int32_t* table_row = a.prefix_table + (size_t)g * a.max_pp;
  const float sc = fmaxf(fabsf(a.scale) * 1.44269504088896340736f, 1e-30f);
  const uint32_t sign_flip = a.scale < 0.f ? 0x80008000u : 0u;
  const int rows_here = min(block_rows(nrows), nrows - row_begin);
  // keys this block needs: 0 .. position of its last row
  const int tok_end = pos0 + (row_begin + rows_here - 1) / a.R + 1;

  // this wave's tiles: wave, wave + kNW, ...; tile_lo / tile_hi: fewest / most keys any of its rows sees
  int row_index[kMT], limit[kMT], tile_lo[kMT], tile_hi[kMT];
  u32x4 qreg[kMT][4];
#pragma unroll
  for (int qt = 0; qt < kMT; ++qt) {
    const int r0 = (qt * kNW + wave) * 16;            // first row of the tile within the block
    const int rho = row_begin + r0 + i;
    tile_lo[qt] = tile_hi[qt] = 0;                    // tile without rows: never computed
    if (r0 < rows_here) {
      tile_lo[qt] = pos0 + (row_begin + r0) / a.R + 1;
      tile_hi[qt] = pos0 + (row_begin + min(r0 + 15, rows_here - 1)) / a.R + 1;
    }
    int idx = -1;
    limit[qt] = 1;
    if (r0 + i < rows_here) {
      idx = (qrow0 + rho / a.R) * a.Hq + kvh * a.R + rho % a.R;
      limit[qt] = pos0 + rho / a.R + 1;
    }
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
  f32x4 acc[kMT][8];
  float m_run[kMT], l_run[kMT];
#pragma unroll
  for (int qt = 0; qt < kMT; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) acc[qt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int nsteps = (tok_end + kBlockTok - 1) / kBlockTok;
  const size_t page_bytes = (size_t)a.Hkv * (kPage * kD * 2);

  // Page ids of step n (wave-uniform scalar loads).  A step past the end repeats the last one:
  // its loads fetch valid bytes that nobody uses, so the loop needs no conditional loads and
  // every wait knows how many younger loads are in flight.
  auto load_ids = [&](int n, int& p0, int& p1) {
    const int t = min(n, nsteps - 1) * kBlockTok;
    p0 = ld_uniform(table_row + (t >> 4));
    p1 = (t + kPage < tok_end) ? ld_uniform(table_row + (t >> 4) + 1) : p0;
    if ((unsigned)p0 >= (unsigned)a.num_pages) { p0 = 0; bad_page = 1; }
    if ((unsigned)p1 >= (unsigned)a.num_pages) { p1 = 0; bad_page = 1; }
  };
  // A step is 1024 16-byte vectors: K of page 0, K of page 1, V of page 0, V of page 1 (256
  // each, contiguous in memory); thread tid fetches vectors tid + k * threads, so which of the
  // four regions a load belongs to is the same for a whole wave: the page's base address is
  // scalar arithmetic and a lane adds only its fixed 32-bit offset.  K lands in LDS as 32 token
  // rows of 256 B with the 16-byte chunk index XOR-ed with a key of the row, V as
  // [page][channel][2 halves of 8 slots] with the unit index XOR-ed with (unit >> 3) & 1, so
  // that the 8 lanes of one operand read hit 8 different bank groups.
  // global_load_lds_dwordx4 moves the vectors from global memory straight into
  // LDS (the 64 lanes of a wave fill 1 KB in lane order, no registers in between).  Wave `wave`
  // fills, for k < kLoads, the 64 slots from slot w0 of region k * kNW/4 + wave/4; the XOR
  // swizzle (an involution inside a key row / a pair of value units) is applied on the source
  // side: the lane that fills slot s fetches vector swz(s).
  static_assert(kNW % 4 == 0, "a wave's 64 vectors must lie in one 256-vector region");
  const int w0 = (wave & 3) * 64;
  uint32_t src_off[kLoads];
  int region[kLoads];
#pragma unroll
  for (int k = 0; k < kLoads; ++k) {
    region[k] = k * (kNW / 4) + (wave >> 2);
    const int s_pos = w0 + lane;
    const int slot = s_pos >> 4;
    // swizzle key of K row tau = 16 * (region & 1) + slot: bits 0, 1, 3, 4 of tau (the 16 rows one
    // operand read touches differ in exactly those bits, so its 16 lanes hit 16 different bank groups)
    const int key = ((region[k] & 1) << 3) | ((slot >> 3) << 2) | (slot & 3);
    const int src = (region[k] >> 1) ? (s_pos ^ ((s_pos >> 3) & 1))
                                     : ((slot << 4) | ((s_pos & 15) ^ key));
    src_off[k] = (uint32_t)kvh * (kPage * kD * 2) + (uint32_t)src * 16;
  }
  auto issue = [&](int p0, int p1, char* buf) {
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const char* base = reinterpret_cast<const char*>((region[k] >> 1) ? a.v_pages : a.k_pages) +
                         (size_t)((region[k] & 1) ? p1 : p0) * page_bytes;
      char* dst = buf + region[k] * 4096 + w0 * 16;   // wave-uniform; lane l lands at dst + 16 l
      __builtin_amdgcn_global_load_lds(
          reinterpret_cast<const __attribute__((address_space(1))) void*>(reinterpret_cast<uintptr_t>(base + src_off[k])),
          reinterpret_cast<__attribute__((address_space(3))) void*>((uint32_t)reinterpret_cast<uintptr_t>(dst)),
          16, 0, 0);
    }
  };
  const int k_rd = (8 * (i >> 2) + (i & 3)) * 256;
  const int v_rd = 2 * kBlockTok * kD + (j >> 1) * 4096;

  constexpr float kPfRescaleSlack = 8.0f;   // log2 units
  auto compute_edge = [&](int n, const char* buf) {
    const int t0 = n * kBlockTok;
    const bool ragged = t0 + kBlockTok > tok_end;   // workgroup-uniform; only the last step
    u32x4 pb[kMT];   // set and used only for the tiles this step touches
    u32x4 kr[2][4];
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        kr[T][kk] = *reinterpret_cast<const u32x4*>(buf + k_rd + T * 4 * 256 + (((4 * kk + j) ^ i) << 4));
#pragma unroll
    for (int qt = 0; qt < kMT; ++qt) {
      if (t0 < tile_hi[qt]) {   // wave-uniform: some row of the tile sees a token of this step
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          s0 = mfma_16x16x32(kr[0][kk], qreg[qt][kk], s0);
          s1 = mfma_16x16x32(kr[1][kk], qreg[qt][kk], s1);
        }
        if (t0 + kBlockTok > tile_lo[qt]) {   // wave-uniform: the causal edge crosses this step
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (t0 + 8 * j + e >= limit[qt]) s0[e] = -INFINITY;
            if (t0 + 8 * j + 4 + e >= limit[qt]) s1[e] = -INFINITY;
          }
        }
        float mx = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                         fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
        mx = rows_allreduce_max(mx);
        // every row sees token 0, so after step 0 the reference maximum is finite and a fully masked
        // row of a later step gives alpha = 1, p = 0; the reference moves only when the row's maximum
        // exceeds it by more than 2^kPfRescaleSlack (as in the loop before the edge)
        const float m_new = mx * sc > m_run[qt] + kPfRescaleSlack ? mx * sc : m_run[qt];
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
    u32x4 vr[8];
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) {
      const int u = 2 * (16 * ct + i) + (j & 1);
      vr[ct] = *reinterpret_cast<const u32x4*>(buf + v_rd + ((u ^ ((i >> 2) & 1)) << 4));
    }
    if (ragged) {
      // value slots past the block's last key may hold anything (NaN included): zero them
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const int tok = t0 + 8 * j + 2 * d;
        const uint32_t mask = (tok < tok_end ? 0x0000ffffu : 0u) | (tok + 1 < tok_end ? 0xffff0000u : 0u);
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) vr[ct][d] &= mask;
      }
    }
#pragma unroll
    for (int qt = 0; qt < kMT; ++qt)
      if (t0 < tile_hi[qt]) {
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) acc[qt][ct] = mfma_16x16x32(vr[ct], pb[qt], acc[qt][ct]);
      }
  };


  // A step that every row of the wave's tiles sees in full (no causal edge, not ragged): the
  // same arithmetic as compute_edge without masks, tile tests and per-tile branches: all score
  // products, the row maxima, ONE test whether any row's reference maximum has to move (rare after
  // the first steps; the accumulators are rescaled in that branch only), then per tile the exponentials
  // and that tile's output products.  About 150 vector-ALU instructions per step instead of 250.
  auto compute_full = [&](int, const char* buf) {
    u32x4 kr[2][4];
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        kr[T][kk] = *reinterpret_cast<const u32x4*>(buf + k_rd + T * 4 * 256 + (((4 * kk + j) ^ i) << 4));
    f32x4 s0[kMT], s1[kMT];
    float m_new[kMT];
#pragma unroll
    for (int qt = 0; qt < kMT; ++qt) {
      s0[qt] = f32x4{0.f, 0.f, 0.f, 0.f};
      s1[qt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s0[qt] = mfma_16x16x32(kr[0][kk], qreg[qt][kk], s0[qt]);
        s1[qt] = mfma_16x16x32(kr[1][kk], qreg[qt][kk], s1[qt]);
      }
    }
    // The reference maximum of a row moves only when the row's maximum exceeds it by more than
    // 2^kPfRescaleSlack (weights then stay below that).  With an exact running maximum one of a
    // wave's 48 rows sets a new record in most steps of a long prompt; with the slack the test below
    // fails in nearly every step after the first few, and then neither the maxima of the rows (a
    // reduction over four lanes each) nor new references nor rescaled accumulators are needed.
    bool moved = false;
    float mx[kMT];
#pragma unroll
    for (int qt = 0; qt < kMT; ++qt) {
      mx[qt] = fmaxf(fmaxf(fmaxf(s0[qt][0], s0[qt][1]), fmaxf(s0[qt][2], s0[qt][3])),
                     fmaxf(fmaxf(s1[qt][0], s1[qt][1]), fmaxf(s1[qt][2], s1[qt][3]))) * sc;   // this lane's 8 tokens
      m_new[qt] = m_run[qt];
      moved |= mx[qt] > m_run[qt] + kPfRescaleSlack;
    }
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {   // wave-uniform
#pragma unroll
      for (int qt = 0; qt < kMT; ++qt) {
        const float row_mx = rows_allreduce_max(mx[qt]);
        if (row_mx > m_run[qt] + kPfRescaleSlack) m_new[qt] = row_mx;
        const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_new[qt]);   // 1 where the row did not move
        l_run[qt] *= alpha;
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) acc[qt][ct] *= alpha;
      }
    }
    u32x4 vr[8];
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) {
      const int u = 2 * (16 * ct + i) + (j & 1);
      vr[ct] = *reinterpret_cast<const u32x4*>(buf + v_rd + ((u ^ ((i >> 2) & 1)) << 4));
    }
#pragma unroll
    for (int qt = 0; qt < kMT; ++qt) {
      m_run[qt] = m_new[qt];
      float p[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[qt][e], sc, -m_new[qt]));
        p[4 + e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[qt][e], sc, -m_new[qt]));
      }
      l_run[qt] += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
      const u32x4 pb = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) acc[qt][ct] = mfma_16x16x32(vr[ct], pb, acc[qt][ct]);
    }
  };

  // ring of kPfStages LDS buffers: per iteration wait until this wave's part of step n has landed
  // (all but the youngest kPfStages-2 steps' loads), a bare workgroup barrier (everybody's part
  // has landed and everybody has finished reading buffer (n-1) % kPfStages; a fence would wait
  // for every outstanding load), then the loads of step n+kPfStages-1 go into that buffer
  int p0, p1;
#pragma unroll
  for (int s0 = 0; s0 < kPfStages - 1; ++s0) {
    load_ids(s0, p0, p1);
    issue(p0, p1, lds.buf[s0]);
  }
  load_ids(kPfStages - 1, p0, p1);
  auto ring_step = [&](int n, auto&& comp) {
    __builtin_amdgcn_s_waitcnt(pf_vmcnt_imm((kPfStages - 2) * kLoads));
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue(p0, p1, lds.buf[(n + kPfStages - 1) % kPfStages]);
    load_ids(n + kPfStages, p0, p1);
    comp(n, lds.buf[n % kPfStages]);
  };
  // Two loops (their register allocations do not mix): a wave that owns kMT tiles of this block
  // runs the steps before the causal edge of its first tile (tile_lo grows with the tile) in the
  // mask-free code, all other steps in the general code.  Every wave passes the same number of
  // barriers.
  bool all_tiles = true;
#pragma unroll
  for (int qt = 0; qt < kMT; ++qt) all_tiles = all_tiles && (qt * kNW + wave) * 16 < rows_here;
  const int n_full = all_tiles ? min(tile_lo[0] / kBlockTok, nsteps) : 0;
  int n = 0;
  for (; n < n_full; ++n) ring_step(n, compute_full);
  for (; n < nsteps; ++n) ring_step(n, compute_edge);
  __builtin_amdgcn_s_waitcnt(pf_vmcnt_imm(0));
  __syncthreads();
  // lane (i, j) holds channels 16*ct + 4*j .. +3 of q-row i
#pragma unroll
  for (int qt = 0; qt < kMT; ++qt) {
    const float l = rows_allreduce_sum(l_run[qt]);
    if (row_index[qt] >= 0) {
      const float inv = 1.0f / l;   // l >= 1: the row's own maximum contributes exp2(0)
      if (a.out_dtype == MARL_OUT_F32) {
        float* dst = reinterpret_cast<float*>(a.out) + (size_t)row_index[qt] * kD + 4 * j;
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) *reinterpret_cast<f32x4*>(dst + 16 * ct) = acc[qt][ct] * inv;
      } else {
        uint16_t* dst = reinterpret_cast<uint16_t*>(a.out) + (size_t)row_index[qt] * kD + 4 * j;
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) {
          const f32x4 r = acc[qt][ct] * inv;
          *reinterpret_cast<uint2*>(dst + 16 * ct) = make_uint2(pack_bf16(r[0], r[1]), pack_bf16(r[2], r[3]));
        }
      }
    }
  }
}

__global__ __launch_bounds__(kPfThreads)
__attribute__((amdgpu_waves_per_eu(MARL_PREFILL_WAVES_PER_EU, MARL_PREFILL_WAVES_PER_EU)))
void prefill_kernel(PrefillArgs a) {
  __shared__ PrefillLds lds;
  __shared__ int next_item;
  const int n_work = a.block_start[a.NG] * a.Hkv;
  int bad_page = 0;
  // The first item is the block index; later ones come from the counter, drawn when the
  // workgroup is free (drawing the next index while an item runs measured 2-5 % slower).
  int qi = blockIdx.x;
  while (qi < n_work) {
    const int2 it = a.items[qi / a.Hkv];
    prefill_item(a, it.x, it.y, qi % a.Hkv, lds, bad_page);
    // prefill_item ends with a workgroup barrier after its last LDS use
    if (threadIdx.x == 0) next_item = gridDim.x + atomicAdd(&a.counters[kPfCursor], 1);
    __syncthreads();
    qi = next_item;
    __syncthreads();
  }
  if (bad_page) atomicOr(&a.counters[kPfFlags], MARL_FLAG_BAD_PAGE);
}

// Scatter of a prompt chunk's keys and values into the group's pages.  One workgroup of 128
// threads per (group, KV head, column of the group's table row); a column the chunk does not
// touch exits at once.  The key rows of a page are contiguous (4 KB): 16-byte copies.  Values
// are stored channel-major, so thread c collects channel c of the page's 16 tokens and writes
// its 32 bytes with two stores when the chunk covers the whole page, else slot by slot.
__global__ __launch_bounds__(kD) void kv_write_prompt_kernel(PrefillArgs a) {
  const int col = blockIdx.x % a.max_pp;
  const int gk = blockIdx.x / a.max_pp;
  const int g = gk / a.Hkv, kvh = gk % a.Hkv;
  const int c = threadIdx.x;
  int flag = 0;
  const int n = group_tokens(a, g, flag);
  const int pos0 = a.q_pos0[g];
  const int lo = max(pos0, col * kPage), hi = min(pos0 + n, (col + 1) * kPage);   // positions to write
  if (col == 0 && kvh == 0 && c == 0 && flag && a.flags) atomicOr(a.flags, flag);
  if (flag & MARL_FLAG_BAD_GROUP) return;
  if (lo >= hi) return;
  const int page = a.prefix_table[(size_t)g * a.max_pp + col];
  if ((unsigned)page >= (unsigned)a.num_pages) {
    if (kvh == 0 && c == 0 && a.flags) atomicOr(a.flags, MARL_FLAG_BAD_PAGE);
    return;
  }
  const size_t blk = ((size_t)page * a.Hkv + kvh) * (kPage * kD);                 // elements
  const size_t tok0 = (size_t)a.q_start[g] + (col * kPage - pos0);                // token of slot 0 (may be "negative")
  const size_t row_stride = (size_t)a.Hkv * kD;
  // keys: 16 slots x 16 chunks of 16 bytes, two per thread
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int v = c + k * kD;
    const int slot = v >> 4, chunk = v & 15;
    const int pos = col * kPage + slot;
    if (pos >= lo && pos < hi)
      *reinterpret_cast<u32x4*>(a.k_pages_w + blk + (size_t)slot * kD + chunk * 8) =
          *reinterpret_cast<const u32x4*>(a.k_new + (tok0 + slot) * row_stride + (size_t)kvh * kD + chunk * 8);
  }
  // values: channel c of every slot
  uint16_t vals[kPage];
#pragma unroll
  for (int slot = 0; slot < kPage; ++slot) {
    const int pos = col * kPage + slot;
    vals[slot] = (pos >= lo && pos < hi) ? a.v_new[(tok0 + slot) * row_stride + (size_t)kvh * kD + c] : (uint16_t)0;
  }
  uint16_t* vdst = a.v_pages_w + blk + (size_t)c * kPage;
  if (hi - lo == kPage) {
    u32x4 w0, w1;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      w0[d] = (uint32_t)vals[2 * d] | ((uint32_t)vals[2 * d + 1] << 16);
      w1[d] = (uint32_t)vals[8 + 2 * d] | ((uint32_t)vals[8 + 2 * d + 1] << 16);
    }
    *reinterpret_cast<u32x4*>(vdst) = w0;
    *reinterpret_cast<u32x4*>(vdst + 8) = w1;
  } else {
#pragma unroll
    for (int slot = 0; slot < kPage; ++slot) {
      const int pos = col * kPage + slot;
      if (pos >= lo && pos < hi) vdst[slot] = vals[slot];
    }
  }
}

}  // namespace

int prefill_rows_per_block() { return kQB; }

int prefill_blocks_per_cu() {
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, prefill_kernel, kPfThreads, 0) != hipSuccess || n < 1) n = 1;
  return n;
}

hipError_t launch_prefill(const PrefillArgs& a, int grid, hipStream_t st) {
  hipLaunchKernelGGL(prefill_plan_kernel, dim3(1), dim3(kPlanThreadsPf), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(prefill_kernel, dim3(grid), dim3(kPfThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_kv_write_prompt(const PrefillArgs& a, hipStream_t st) {
  if (a.NT == 0 || a.NG == 0) return hipSuccess;
  hipLaunchKernelGGL(kv_write_prompt_kernel, dim3((unsigned)a.NG * a.Hkv * a.max_pp), dim3(kD), 0, st, a);
  return hipGetLastError();
}

}  // namespace marl
