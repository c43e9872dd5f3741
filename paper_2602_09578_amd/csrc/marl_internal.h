// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "marl_decode.h"

namespace marl {

constexpr int kPage = 16;        // tokens per page
constexpr int kD = 128;          // head dimension
constexpr int kBlockTok = 32;    // tokens one MFMA step of a wave covers (two pages)
constexpr int kRowsPerQBlock = 128;       // query rows one prefix work item covers (4-wave kernel)
constexpr int kRowsPerQBlockWide = 256;   // ... in the 8-wave kernel
// suffix items up to this many tokens are handled by one wave (build-time tuning knob)
#ifndef MARL_SHORT_TOKENS
#define MARL_SHORT_TOKENS 128
#endif
constexpr int kShortTokens = MARL_SHORT_TOKENS;
constexpr int kAttnThreads = 256;  // 4 waves per workgroup
constexpr int kPlanThreads = 1024;
constexpr int kNumClasses = 2048;  // upper bound on cost classes (chunk / 32)

// Everything the attention kernels need; passed by value.
struct AttnArgs {
  const uint16_t* q;
  const uint16_t* k_pages;
  const uint16_t* v_pages;
  const int32_t* prefix_table;
  const int32_t* suffix_table;
  const int32_t* prefix_lens;
  const int32_t* suffix_lens;
  const int32_t* group_of_seq;
  int32_t* counters;
  int32_t* group_count;
  int32_t* group_start;
  int32_t* seq_rank;
  int32_t* group_tmp;
  int32_t* group_seqs;
  int32_t* seq_chunks;   // per sequence: prefix chunk count | suffix chunk count << 16
  int4* suffix_items;
  int4* prefix_items;
  float2* partial_ml;
  float* partial_o;
  void* out;
  int32_t NS, NG, Hq, Hkv, R;
  int32_t num_pages, max_pp, max_sp;
  int32_t Cs, Cp, NCs, NCp;
  int32_t qblock_rows;   // kRowsPerQBlock or kRowsPerQBlockWide
  int32_t out_dtype;
  float scale;
};

hipError_t launch_plan(const AttnArgs& a, hipStream_t st);
hipError_t launch_prefix(const AttnArgs& a, int grid, hipStream_t st);
hipError_t launch_suffix(const AttnArgs& a, int grid, hipStream_t st);
hipError_t launch_merge(const AttnArgs& a, hipStream_t st);
int prefix_blocks_per_cu(bool wide);
int suffix_blocks_per_cu();

struct KvAppendArgs {
  const uint16_t* k_new;
  const uint16_t* v_new;
  uint16_t* k_pages;
  uint16_t* v_pages;
  const int32_t* suffix_table;
  int32_t* suffix_lens;
  int32_t* flags;   // may be null
  int32_t NS, Hkv, num_pages, max_sp;
};
struct KvCopyArgs {
  uint16_t* k_pages;
  uint16_t* v_pages;
  const int32_t* src;
  const int32_t* dst;
  int32_t* flags;   // may be null
  int32_t n, Hkv, num_pages;
};
hipError_t launch_kv_append(const KvAppendArgs& a, hipStream_t st);
hipError_t launch_kv_copy_pages(const KvCopyArgs& a, hipStream_t st);

struct PackArgs {
  const marl_pack_entry* entries;   // device
  char* packed;
  int32_t n;
  int32_t total_chunks;
  int32_t unpack;   // 0: tensors -> packed, 1: packed -> tensors
};
hipError_t launch_pack(const PackArgs& a, int grid, hipStream_t st);

struct LogprobArgs {
  const uint16_t* logits;
  const int32_t* tokens;
  float* out;
  float2* partials;   // [rows][slices] (max, sum) in base-2 units; unused when slices == 1
  int32_t rows, vocab, slices, slice_len;
  float inv_temp_log2e;   // log2(e) / T
};
hipError_t launch_logprobs(const LogprobArgs& a, hipStream_t st);
hipError_t launch_logprobs_finish(const LogprobArgs& a, hipStream_t st);

struct SampleArgs {
  const uint16_t* logits;
  const float* uniforms;
  int32_t* out_tokens;
  float* out_logprobs;
  float2* partials;      // [rows][num_chunks] (max, sum) of each 4096-logit chunk, base-2 units
  int32_t rows, vocab, num_chunks, chunks_per_wave, groups_per_row;
  float inv_temp_log2e;
};
int sample_num_chunks(int vocab);
hipError_t launch_sample(const SampleArgs& a, hipStream_t st);

struct TopPArgs {
  const uint16_t* logits;
  const float* uniforms;
  int32_t* out_tokens;
  float* out_logprobs;
  int32_t rows, vocab;
  float inv_temp_log2e, top_p;
};
int top_p_max_vocab();
hipError_t launch_sample_top_p(const TopPArgs& a, hipStream_t st);

struct PrefillArgs {
  const uint16_t* q;            // [NT][Hq][128]
  const uint16_t* k_pages;
  const uint16_t* v_pages;
  const int32_t* prefix_table;  // [NG][max_pp]
  const int32_t* q_start;       // [NG + 1]
  const int32_t* q_pos0;        // [NG]
  void* out;                    // [NT][Hq][128]
  int32_t* counters;            // workspace header
  int32_t* block_start;         // [NG + 1] running number of row blocks
  int2* items;                  // [blocks] (group, first row of the block)
  // the prompt scatter only:
  const uint16_t* k_new;        // [NT][Hkv][128]
  const uint16_t* v_new;
  uint16_t* k_pages_w;
  uint16_t* v_pages_w;
  int32_t* flags;
  int32_t NT, NG, Hq, Hkv, R, num_pages, max_pp, out_dtype, max_blocks;
  float scale;
};
int prefill_rows_per_block();
int prefill_blocks_per_cu();
hipError_t launch_prefill(const PrefillArgs& a, int grid, hipStream_t st);
hipError_t launch_kv_write_prompt(const PrefillArgs& a, hipStream_t st);

struct GrpoArgs {
  const float* rewards;        // [num_seqs]
  const int32_t* group_start;  // [num_groups + 1]
  const int32_t* group_seqs;   // member lists, group after group
  float* out;                  // [num_seqs]
  int32_t num_groups;
  float eps;
};
hipError_t launch_grpo_advantages(const GrpoArgs& a, hipStream_t st);

}  // namespace marl
