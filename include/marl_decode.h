/*
 * marl_decode.h — C ABI of the MI355X (gfx950) rollout-decode library.
 *
 * The library computes the two data-parallel operations that one decode step of multi-agent
 * RL rollout spends its time in: single-token attention over a paged KV cache whose prompts
 * are each expanded into several samples sharing the prompt's prefix, and the per-token
 * log-probability that RL training consumes.  The paper motivates both (rollout is
 * memory-bound on KV caches: Section 4.1; several samples per prompt: Section 5.1 and the
 * parallelism settings of Section 8.1; skewed agent load: Section 2.2, Observation #2; GRPO
 * training: Section 8.1) but delegates them to a black-box inference backend (Section 7), so
 * the operations are the textbook ones, stated with every entry point below.
 *
 * Conventions for every entry point
 *   - Pointers named "device" are GPU addresses owned by the caller; the library never
 *     allocates, frees or keeps them.  `stream` is a hipStream_t (NULL = default stream).
 *   - Calls only enqueue work on `stream` and return; nothing synchronises with the host.
 *   - Return value: MARL_OK (0) or a negative marl_status.  Arguments are validated on the
 *     host before any HIP call, so argument errors are reported without touching the GPU.
 *     Contents of device arrays cannot be validated without a sync; instead the kernels
 *     clamp what they read (lengths to the table extents, page ids to [0, num_pages),
 *     group ids outside [0, num_groups) mean "no prefix") so bad contents never cause an
 *     out-of-range access, and record a flag readable with marl_attn_read_flags().
 *   - bf16 means the upper 16 bits of an IEEE float32; conversions round to nearest even.
 */
#ifndef MARL_DECODE_H
#define MARL_DECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum marl_status {
  MARL_OK = 0,
  MARL_INVALID_ARG = -1,   /* null pointer, negative count, Hq % Hkv != 0, non-finite scalar */
  MARL_UNSUPPORTED = -2,   /* head_dim != 128, page_size != 16, unknown out_dtype, bad chunk */
  MARL_WORKSPACE_TOO_SMALL = -3,
  MARL_HIP_ERROR = -4,     /* a launch failed; marl_last_hip_error() has the text */
  MARL_OUT_OF_MEMORY = -5  /* a host allocation of the host-side helpers (balancer, page pool) failed */
} marl_status;

enum { MARL_OUT_BF16 = 0, MARL_OUT_F32 = 1 };

/* Shape of one marl_decode_attn call (host memory). */
typedef struct marl_attn_shape {
  int32_t num_seqs;          /* NS >= 0 */
  int32_t num_groups;        /* NG >= 0: shared-prefix groups (prompts) */
  int32_t num_q_heads;       /* Hq */
  int32_t num_kv_heads;      /* Hkv, Hq % Hkv == 0, Hq / Hkv <= 16 */
  int32_t head_dim;          /* must be 128 */
  int32_t page_size;         /* must be 16 */
  int32_t num_pages;         /* extent of k_pages / v_pages along dim 0, >= 1 */
  int32_t max_prefix_pages;  /* row stride of prefix_block_table, >= 0 */
  int32_t max_suffix_pages;  /* row stride of suffix_block_table, >= 0 */
  int32_t out_dtype;         /* MARL_OUT_BF16 or MARL_OUT_F32 */
  int32_t suffix_chunk_tokens; /* 0 = library default; else a multiple of 32 in [32, 65536] */
  int32_t prefix_chunk_tokens; /* 0 = library default; else a multiple of 32 in [32, 65536] */
} marl_attn_shape;

/* How the library lays out its workspace for a shape (host-only; for sizing and for tests
 * that read the work list back).  All offsets are in bytes from the workspace start. */
typedef struct marl_attn_plan_layout {
  int32_t suffix_chunk_tokens;   /* Cs actually used */
  int32_t prefix_chunk_tokens;   /* Cp actually used */
  int32_t suffix_slots;          /* NCs = max(1, ceil(max_suffix_pages*16 / Cs)) */
  int32_t prefix_slots;          /* NCp = max(1, ceil(max_prefix_pages*16 / Cp)) */
  int32_t rows_per_qblock;       /* query rows one prefix work item covers: 256 if the average
                                    group, ceil(NS/NG)*(Hq/Hkv) rows, exceeds 128, else 128 */
  int32_t max_suffix_items;      /* NS * NCs */
  int32_t max_prefix_items;      /* (NG + NS*(Hq/Hkv)/rows_per_qblock + 1) * NCp */
  int32_t reserved;
  size_t counters_off;           /* int32[64]: see MARL_CTR_* */
  size_t group_count_off;        /* int32[NG]   sequences per group */
  size_t group_start_off;        /* int32[NG+1] exclusive scan of group_count */
  size_t seq_rank_off;           /* int32[NS]   scratch */
  size_t group_tmp_off;          /* int32[NS]   scratch */
  size_t group_seqs_off;         /* int32[NS]   sequence ids grouped by group (CSR values) */
  size_t seq_chunks_off;         /* int32[NS]   prefix chunks | suffix chunks << 16 of each sequence */
  size_t suffix_items_off;       /* int32[max_suffix_items][4] {seq, tok_begin, tok_end, 0} */
  size_t prefix_items_off;       /* int32[max_prefix_items][4] {group, tok_begin, tok_end, row_begin} */
  size_t partial_ml_off;         /* float[NS][Hq][NCp+NCs][2]  (max, sum) per partial */
  size_t partial_o_off;          /* float[NS][Hq][NCp+NCs][128] unnormalised partial output */
  size_t total_bytes;
} marl_attn_plan_layout;

enum {
  MARL_CTR_NUM_SUFFIX_ITEMS = 0,
  MARL_CTR_NUM_PREFIX_ITEMS = 1,
  MARL_CTR_SUFFIX_CURSOR = 2,    /* work-queue cursors, zero after the plan kernel */
  MARL_CTR_PREFIX_CURSOR = 3,
  MARL_CTR_FLAGS = 4,            /* MARL_FLAG_* bits set by the kernels */
  MARL_CTR_NUM_LONG_SUFFIX_ITEMS = 5, /* suffix items of more than 128 tokens: they head the list */
  MARL_CTR_SHORT_CURSOR = 6,     /* work-queue cursor of the remaining (short) suffix items */
  MARL_CTR_NUM_SHORT_PARTIAL_ITEMS = 7 /* suffix items of at most 128 tokens that belong to sequences with
                                     several suffix chunks (the only short items that become partials) */
};
enum {
  MARL_FLAG_BAD_GROUP = 1,       /* a group_of_seq entry was outside [0, NG) */
  MARL_FLAG_LEN_CLAMPED = 2,     /* a length was negative or exceeded its table row */
  MARL_FLAG_BAD_PAGE = 4         /* a block-table entry of a valid token was outside [0, num_pages) */
};

/* Fills *layout for *shape.  Host-only, no GPU needed.
 * Chunking rule when the shape gives 0:  Cs starts at 8192 and is halved while
 * NS*Hkv*ceil(max_suffix_tokens/Cs) < 2048 and Cs > 256;  Cp starts at 8192 and is halved
 * while NG*Hkv*Q*ceil(max_prefix_tokens/Cp) < W and Cp > 256, where
 * Q = max(1, ceil(ceil(NS/NG)*(Hq/Hkv) / rows_per_qblock)) estimates the query-row blocks of
 * a group and W = 512 (256 when rows_per_qblock is 256). */
int marl_attn_plan_layout_for(const marl_attn_shape* shape, marl_attn_plan_layout* layout);

/* *bytes = layout.total_bytes (an upper bound that depends on the shape only). Host-only. */
int marl_workspace_bytes(const marl_attn_shape* shape, size_t* bytes);

/*
 * Batched single-token attention over a paged KV cache with shared prefixes.
 *
 * For sequence s with group g = group_of_seq[s] and query head h (KV head kh = h / (Hq/Hkv)),
 * the logical tokens are the P = prefix_lens[g] prefix tokens of the group followed by the
 * S = suffix_lens[s] tokens the sequence generated itself (the current token included: the
 * call only reads the cache).  Prefix token j is at page prefix_block_table[g][j/16], slot
 * j%16; suffix token j' at page suffix_block_table[s][j'/16], slot j'%16.  With
 * x_j = scale * <q[s,h,:], K_j>, the result is out[s,h,:] = sum_j softmax(x)_j V_j, and zeros
 * when P + S == 0.
 *
 * Device arrays:
 *   q                   bf16  [NS, Hq, 128]
 *   k_pages             bf16  [num_pages, Hkv, 16 slots, 128]   (a token's key is contiguous)
 *   v_pages             bf16  [num_pages, Hkv, 128, 16 slots]   (a channel's 16 slots are contiguous)
 *   prefix_block_table  int32 [NG, max_prefix_pages]   entries past a row's pages are ignored (-1 by convention)
 *   suffix_block_table  int32 [NS, max_suffix_pages]
 *   prefix_lens         int32 [NG]  tokens
 *   suffix_lens         int32 [NS]  tokens
 *   group_of_seq        int32 [NS]  in [0, NG); a group's sequences may appear in any order
 *   out                 bf16 or float32 [NS, Hq, 128] per shape->out_dtype
 *   workspace           at least marl_workspace_bytes() bytes, 256-byte aligned; contents on
 *                       entry are irrelevant, contents on exit are the work list and partials
 * q, k_pages, v_pages and out must be 16-byte aligned (MARL_INVALID_ARG otherwise): they are
 * accessed as 16-byte vectors.
 * Unused slots of a partly filled page and pages no table names are never read into a result
 * (they may hold anything, NaN included).  The values the call does use must be finite: q, and
 * the keys and values of every token the lengths address.  With a NaN or an infinity among them
 * the affected rows are unspecified (the attention kernels are compiled on the assumption that
 * no NaN enters their floating-point arithmetic); the same holds for marl_prefill_attn.
 * Calls that share a workspace must be ordered on one stream.
 *
 * Work: a plan kernel builds the group->sequences CSR and two work lists (prefix items per
 * group, suffix items per sequence, each at most a chunk of tokens, longest first); a
 * prefix kernel streams each group's prefix KV once for all of the group's query rows; a
 * suffix kernel streams each sequence's own KV in items of more than 128 tokens; a merge kernel
 * combines the per-chunk (max, sum, output) partials in a fixed order, so results are
 * bit-identical across runs.  A sequence whose own tokens form a single item never writes a
 * suffix partial: the kernel that processes the item (the suffix kernel, or for items of at most
 * 128 tokens the first phase of the merge kernel, one item per wave) applies the merge formula to
 * the group's prefix partials and its own result and writes the output rows.  Short items of
 * sequences with several suffix chunks are taken by the prefix kernel's workgroups before they
 * start on the prefix items.
 */
int marl_decode_attn(const marl_attn_shape* shape, void* workspace, size_t workspace_bytes,
                     const void* q, const void* k_pages, const void* v_pages,
                     const int32_t* prefix_block_table, const int32_t* suffix_block_table,
                     const int32_t* prefix_lens, const int32_t* suffix_lens,
                     const int32_t* group_of_seq, float scale, void* out, void* stream);

/* Runs only the plan kernel of marl_decode_attn (same arguments' meaning); after it, the
 * workspace holds the CSR, the work lists and the counters described by the layout. */
int marl_attn_plan(const marl_attn_shape* shape, void* workspace, size_t workspace_bytes,
                   const int32_t* prefix_lens, const int32_t* suffix_lens,
                   const int32_t* group_of_seq, void* stream);

/* Copies the MARL_FLAG_* word of a workspace to *flags_host.  Synchronises `stream`. */
int marl_attn_read_flags(const void* workspace, int32_t* flags_host, void* stream);

/*
 * marl_decode_attn for callers that cannot allocate device memory or hold a workspace of their
 * own: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operation, same kernels and bit-identical results as marl_decode_attn; the workspace is a
 * fixed array of MARL_STATIC_WORKSPACE_BYTES that is part of the library's code object (every GPU
 * the library runs on holds one copy from the first use there until the process ends).  The call
 * allocates nothing and frees nothing; its first call on a device looks the array's address up.
 *   - A shape whose marl_workspace_bytes() exceeds MARL_STATIC_WORKSPACE_BYTES is rejected with
 *     MARL_WORKSPACE_TOO_SMALL on the host, before any HIP call (shrink the batch, or use
 *     marl_decode_attn with a workspace of the caller's).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race; order them on one stream.  The array keeps the last call's
 *     work list and partials; the plan kernel clears the counters it needs at zero, nothing else
 *     needs clearing.
 *   - flags: device int32*, may be NULL; after the call's work it holds the MARL_FLAG_* word of
 *     this call (what marl_attn_read_flags reads from a caller's workspace), copied on `stream`
 *     without synchronising.  Must be 4-byte aligned.
 *   - Per-kernel event timing (marl_profile_begin) never covers this entry point.
 * The device that is current at the call must be the one that owns `stream` and the operands.
 */
#define MARL_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
int marl_decode_attn_static(const marl_attn_shape* shape,
                            const void* q, const void* k_pages, const void* v_pages,
                            const int32_t* prefix_block_table, const int32_t* suffix_block_table,
                            const int32_t* prefix_lens, const int32_t* suffix_lens,
                            const int32_t* group_of_seq, float scale, void* out, int32_t* flags,
                            void* stream);

/*
 * KV-cache maintenance for the decode loop (what happens before marl_decode_attn in a decode
 * iteration).  Both are pure data movement; results are bit-exact.
 *
 * marl_kv_append: for every sequence s, with pos = suffix_lens[s], stores the new token's key
 * k_new[s, kh, :] at k_pages[page, kh, pos % 16, :] and its value v_new[s, kh, c] at
 * v_pages[page, kh, c, pos % 16], page = suffix_block_table[s][pos / 16], then sets
 * suffix_lens[s] = pos + 1.  The caller must have put a page into the table row when pos is a
 * multiple of 16.  A sequence whose table row is full (pos >= max_suffix_pages * 16) or whose
 * page id is outside [0, num_pages) is left untouched (length included) and, if `flags` is not
 * NULL, MARL_FLAG_LEN_CLAMPED / MARL_FLAG_BAD_PAGE is OR-ed into *flags (device int32).
 * Only num_seqs, num_kv_heads, head_dim, page_size, num_pages and max_suffix_pages of the
 * shape are used.  Device arrays: k_new, v_new bf16 [NS, Hkv, 128]; the rest as in
 * marl_decode_attn (k_pages, v_pages and suffix_lens are written).  k_new, v_new, k_pages and
 * v_pages must be 16-byte aligned (MARL_INVALID_ARG otherwise).
 *
 * marl_kv_copy_pages: for i < n copies physical page src[i] to page dst[i] (all KV heads, K
 * and V), the device half of forking a sample from another one (the host allocates dst and
 * edits the block tables).  src, dst: device int32 [n]; a dst must not appear twice or as a
 * src of the same call.  Pairs with an id outside [0, num_pages) are skipped and flagged.
 */
int marl_kv_append(const marl_attn_shape* shape, const void* k_new, const void* v_new,
                   void* k_pages, void* v_pages, const int32_t* suffix_block_table,
                   int32_t* suffix_lens, int32_t* flags, void* stream);
int marl_kv_copy_pages(const marl_attn_shape* shape, void* k_pages, void* v_pages,
                       const int32_t* src, const int32_t* dst, int32_t n, int32_t* flags,
                       void* stream);

/*
 * Per-row log-probability of one chosen token:
 *   out[r] = logits[r, tokens[r]] / T - log( sum_v exp(logits[r, v] / T) )
 * Device arrays: logits bf16 [rows, vocab] (row stride = vocab elements), tokens int32
 * [rows], out float32 [rows].  A token id outside [0, vocab) gives NaN for that row.
 * temperature must be finite and > 0.  workspace: marl_logprobs_workspace_bytes() bytes
 * (may be 0, then workspace may be NULL), 256-byte aligned.
 */
int marl_logprobs_workspace_bytes(int32_t rows, int32_t vocab, size_t* bytes);
int marl_token_logprobs(const void* logits, const int32_t* tokens, float temperature, float* out,
                        int32_t rows, int32_t vocab, void* workspace, size_t workspace_bytes,
                        void* stream);

/*
 * Draws one token per row from softmax(logits / T) by inverse CDF and returns its
 * log-probability, with one streaming pass over the logits (plus 8 KB per row):
 *   p_v = softmax(logits[r, :] / T)_v,  token[r] = min { t : sum_{v <= t} p_v > uniforms[r] },
 *   logprob[r] = log p_{token[r]}.
 * uniforms: device float32 [rows] in [0, 1), supplied by the caller (the library draws no
 * random numbers).  If rounding leaves no such t, the last token with non-zero probability is
 * returned.  The sums run in float32, so for a uniform within ~1e-6 of a CDF step the
 * neighbouring token may be returned.  A row without any finite logit gives token -1 and NaN.
 * out_tokens int32 [rows], out_logprobs float32 [rows]; workspace of
 * marl_sample_workspace_bytes() bytes, 8-byte aligned.  Other arguments as marl_token_logprobs.
 */
int marl_sample_workspace_bytes(int32_t rows, int32_t vocab, size_t* bytes);
int marl_sample_tokens(const void* logits, const float* uniforms, float temperature,
                       int32_t* out_tokens, float* out_logprobs, int32_t rows, int32_t vocab,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Top-p (nucleus) variant of marl_sample_tokens.  With p = softmax(logits[r, :] / T): rank the
 * tokens by probability (equal probabilities: lower index first); the nucleus is the shortest
 * head of that ranking whose total probability is >= top_p; the token is drawn from the
 * nucleus by inverse CDF in index order,
 *   token[r] = min { t in nucleus : sum_{v <= t, v in nucleus} p_v > uniforms[r] * p(nucleus) },
 * and logprob[r] = log p_token (of the untruncated distribution).  top_p in (0, 1]; top_p = 1
 * keeps every token.  bf16 logits take at most 65536 values, so the kernel finds the nucleus
 * with an exact count per value instead of a sort; float32 sums decide which value is the
 * threshold and which token passes u, so within ~1e-6 (relative) of such a boundary the
 * neighbouring choice may be returned.  A row without a finite logit, or with +inf / NaN,
 * gives token -1 and NaN.  No workspace.  vocab <= 8388608.  Other arguments as
 * marl_sample_tokens.
 */
int marl_sample_tokens_top_p(const void* logits, const float* uniforms, float temperature,
                             float top_p, int32_t* out_tokens, float* out_logprobs, int32_t rows,
                             int32_t vocab, void* stream);

/*
 * Prefill (prompt) attention: the step that creates a prompt's KV prefix, which all samples of
 * that prompt then share (the paper's Parallel Sampling, Section 5.1; the computation itself is
 * textbook causal attention, the paper gives no formula).  Group g brings
 * n_g = q_start[g+1] - q_start[g] query tokens, rows q_start[g] .. of q, at positions
 * q_pos0[g] .. q_pos0[g] + n_g - 1 of its prompt (q_pos0 > 0: the earlier positions were
 * prefilled before).  The keys and values of positions 0 .. q_pos0[g] + n_g - 1 must already be
 * in the pages listed in prefix_block_table[g] (marl_kv_write_prompt puts a chunk there).
 *   out[t, h, :] = softmax_j( scale * <q[t, h, :], K[j, h / R, :]> ) V[j, h / R, :],
 *   j = 0 .. position of t (inclusive),  R = num_q_heads / num_kv_heads.
 * Device arrays: q bf16 [num_tokens, Hq, 128]; k_pages / v_pages / prefix_block_table as in
 * marl_decode_attn; q_start int32 [num_groups + 1] (non-decreasing, within [0, num_tokens]);
 * q_pos0 int32 [num_groups]; out bf16 or float32 [num_tokens, Hq, 128].  Rows of q that no
 * group covers keep whatever out held.  A group whose tokens do not fit its table row is cut
 * short (MARL_FLAG_LEN_CLAMPED), an inconsistent q_start / q_pos0 entry drops the group
 * (MARL_FLAG_BAD_GROUP), a page id out of range reads page 0 (MARL_FLAG_BAD_PAGE); read the
 * flags with marl_attn_read_flags on this call's workspace.
 * workspace: marl_prefill_workspace_bytes() bytes, 256-byte aligned, used from the start of the
 * call's work until its end on the stream.
 */
typedef struct {
  int32_t num_tokens;        /* NT: query tokens of all groups together */
  int32_t num_groups;        /* NG */
  int32_t num_q_heads;       /* Hq */
  int32_t num_kv_heads;      /* Hkv, divides Hq, Hq / Hkv <= 16 */
  int32_t head_dim;          /* 128 */
  int32_t page_size;         /* 16 */
  int32_t num_pages;         /* extent of k_pages / v_pages */
  int32_t max_prefix_pages;  /* row stride of prefix_block_table */
  int32_t out_dtype;         /* MARL_OUT_BF16 or MARL_OUT_F32 */
  int32_t reserved;          /* 0 */
} marl_prefill_shape;

int marl_prefill_workspace_bytes(const marl_prefill_shape* shape, size_t* bytes);
int marl_prefill_attn(const marl_prefill_shape* shape, void* workspace, size_t workspace_bytes,
                      const void* q, const void* k_pages, const void* v_pages,
                      const int32_t* prefix_block_table, const int32_t* q_start,
                      const int32_t* q_pos0, float scale, void* out, void* stream);

/*
 * Scatter of prompt keys / values into the pages: token q_start[g] + tau of k_new / v_new
 * (bf16 [num_tokens, Hkv, 128]) goes to position q_pos0[g] + tau of group g, i.e. page
 * prefix_block_table[g][pos / 16], slot pos % 16 (K [page][kv_head][slot][128],
 * V [page][kv_head][128][slot]).  Skipped and flagged in *flags (device int32, may be NULL;
 * OR-ed, the caller zeroes it): the tokens of a group that do not fit its table row
 * (MARL_FLAG_LEN_CLAMPED), a group with an inconsistent q_start / q_pos0 entry
 * (MARL_FLAG_BAD_GROUP), a page id out of range (MARL_FLAG_BAD_PAGE).  Bit-exact data movement.
 * k_new, k_pages and v_pages must be 16-byte aligned (MARL_INVALID_ARG otherwise): keys are
 * copied, and whole value pages stored, as 16-byte vectors.
 */
int marl_kv_write_prompt(const marl_prefill_shape* shape, const void* k_new, const void* v_new,
                         void* k_pages, void* v_pages, const int32_t* prefix_block_table,
                         const int32_t* q_start, const int32_t* q_pos0, int32_t* flags,
                         void* stream);

/*
 * Group-normalised advantages of GRPO (Shao et al. 2024; the paper trains every agent with
 * GRPO, Section 8.1).  For each group g (the samples of one prompt) with members
 * group_seqs[group_start[g] .. group_start[g+1]):
 *   mean_g = average reward of the members,  std_g = sqrt(average squared deviation),
 *   out[s] = (rewards[s] - mean_g) / (std_g + eps)   for every member s.
 * A member whose deviation is exactly 0 gets 0 (so a group of equal rewards gives zeros also
 * with eps = 0).  Sequences that belong to no group keep whatever out held.
 * Device arrays: rewards float32 [num_seqs], group_start int32 [num_groups + 1] (non-
 * decreasing, group_start[0] >= 0), group_seqs int32 (sequence ids in [0, num_seqs), each at
 * most once), out float32 [num_seqs].  The plan of marl_decode_attn leaves exactly these two
 * index arrays in its workspace (group_start_off, group_seqs_off of the plan layout).
 * eps must be finite and >= 0.  Contents of the index arrays are not validated.
 */
int marl_grpo_advantages(const float* rewards, const int32_t* group_start,
                         const int32_t* group_seqs, int32_t num_groups, float eps, float* out,
                         void* stream);

/*
 * Hierarchical load balancing of rollout requests (Section 5.2 of the paper), as a host-side,
 * step-driven simulation that yields the per-step batch composition of every inference
 * instance (the sequences one marl_decode_attn call of that instance would cover).  All
 * pointers are HOST pointers; nothing here touches the GPU.  A handle is not thread-safe.
 *
 * Model.  Agents own inference instances (global ids 0.., handed out agent after agent).  An
 * instance holds a FIFO list of unfinished requests; its load is the length of that list; the
 * first slots_per_instance of them run (one token per step), the rest wait.
 *   submit: the request goes to the agent's active instance with the smallest load (ties: the
 *     smallest instance id), found with a min-heap (intra-agent balancing).
 *   step:  (1) instances whose migration has finished join their new agent with an empty list;
 *     (2) every active instance emits one token for each running request; requests that reach
 *     their length complete (done_step = the step counter before it is advanced) and leave;
 *     (3) the step counter advances; if it is a multiple of poll_interval, the agents' waiting
 *     queues q_a (sum over active instances of max(0, load - slots)) are compared: receiver =
 *     the longest queue (ties: smallest agent id), donor = the shortest queue (ties: most active
 *     instances, then smallest id).  If q_receiver - q_donor > delta, then
 *     min(ceil(difference / slots_per_instance), donor's active instances - 1) instances move:
 *     each time the donor's least-loaded instance (ties: smallest id) is detached, its
 *     requests are re-submitted in order to the donor's remaining instances (progress kept),
 *     and it joins the receiver migration_delay steps later (inter-agent balancing).
 * Readings of the paper, which states the rules only in prose: "queue length" is the number of
 * waiting (not running) requests; the number of instances moved is the queue difference in
 * units of one instance's slots (with slots_per_instance = 1 this is the paper's "difference in
 * queue lengths"); a moved instance serves only requests submitted after it joins; its old
 * requests are re-queued on the donor.  The paper sets delta = 5 (Section 8.1).
 */
typedef struct marl_balancer marl_balancer;
typedef struct {
  int32_t num_agents;
  int32_t delta;               /* disparity threshold, >= 0 */
  int32_t slots_per_instance;  /* requests an instance decodes concurrently, >= 1 */
  int32_t poll_interval;       /* steps between inter-agent polls, >= 1 */
  int32_t migration_delay;     /* steps a moved instance is offline, >= 0 */
} marl_balancer_config;
typedef struct {
  int64_t now;                 /* steps taken */
  int64_t submitted, completed;
  int64_t migrations;          /* instances moved so far */
} marl_balancer_stats;
/* instances_per_agent: [num_agents], each >= 1.  *out receives the handle. */
int marl_balancer_create(const marl_balancer_config* cfg, const int32_t* instances_per_agent,
                         marl_balancer** out);
void marl_balancer_destroy(marl_balancer* b);
/* request_id >= 0 and unused so far, gen_len >= 1 tokens; *instance (may be NULL) receives the
 * chosen instance. */
int marl_balancer_submit(marl_balancer* b, int32_t agent, int32_t request_id, int32_t gen_len,
                         int32_t* instance);
int marl_balancer_step(marl_balancer* b, marl_balancer_stats* stats /* may be NULL */);
/* any of the output pointers may be NULL */
int marl_balancer_agent_state(const marl_balancer* b, int32_t agent, int32_t* active_instances,
                              int64_t* waiting_requests, int64_t* assigned_requests);
/* The requests the instance will decode in the next step, in list order, with the tokens each
 * has generated so far.  *owner = its agent, or -1 while it migrates.  *count is always set;
 * MARL_WORKSPACE_TOO_SMALL if it exceeds capacity (then nothing else is written). */
int marl_balancer_instance_batch(const marl_balancer* b, int32_t instance, int32_t* owner,
                                 int32_t* request_ids, int32_t* generated, int32_t capacity,
                                 int32_t* count);
/* *instance = where the request is now (-1 once complete), *done_step = -1 while unfinished */
int marl_balancer_request_state(const marl_balancer* b, int32_t request_id, int32_t* instance,
                                int32_t* generated, int64_t* done_step);

/*
 * Page pool: the host-side bookkeeping of the paged KV cache (which physical pages are free,
 * how many block-table rows refer to a page), with copy-on-write for samples that share pages.
 * The paper's rollout engines keep the shared prompt once and let the samples of a prompt
 * diverge (Parallel Sampling, Section 5.1); it leaves the mechanism to the inference backend,
 * so the rules are stated here.  Host-only (no GPU call, no device memory); the caller owns
 * the block tables as HOST int32 arrays, mirrors them to the device, and runs the copies this
 * object asks for with marl_kv_copy_pages before the next marl_kv_append.
 *
 *   state   every page is free or has a reference count >= 1 (= the number of table entries,
 *           over all rows the caller holds, that contain it).
 *   alloc   takes n free pages, count 1 each; the free pages form a stack that initially pops
 *           0, 1, 2, ... and receives released pages on top (last released, first reused).
 *           If fewer than n pages are free nothing is taken: MARL_WORKSPACE_TOO_SMALL.
 *   retain / release   +1 / -1 on each listed page; a page whose count reaches 0 is free again.
 *           An id outside [0, num_pages), a free page, or (release) more releases in one call
 *           than the page has references: MARL_INVALID_ARG and nothing is changed.
 *   fork    the child row gets the ceil(len / 16) page ids of the parent row, each retained:
 *           parent and child share every page, the partly filled last one included.
 *   prepare_append   makes position `len` of a row writable for marl_kv_append and reports at
 *           most one page copy: if len is a multiple of 16 a fresh page is put into
 *           row[len / 16]; otherwise, if row[len / 16] is shared (count > 1), a fresh page
 *           replaces it in the row, the old one is released, and (*copy_src, *copy_dst) =
 *           (old, fresh) must be copied on the device before the append (copy-on-write: the
 *           other holders keep the old page unchanged); otherwise nothing happens.  Without a
 *           copy both are -1.  len >= max_pages * 16: MARL_INVALID_ARG; no free page:
 *           MARL_WORKSPACE_TOO_SMALL (nothing changed).
 *   drop    releases the ceil(len / 16) pages of a row (a finished sample).
 */
typedef struct marl_page_pool marl_page_pool;
int marl_page_pool_create(int32_t num_pages, marl_page_pool** out);
void marl_page_pool_destroy(marl_page_pool* p);
int marl_page_pool_alloc(marl_page_pool* p, int32_t n, int32_t* pages_out);
int marl_page_pool_retain(marl_page_pool* p, const int32_t* pages, int32_t n);
int marl_page_pool_release(marl_page_pool* p, const int32_t* pages, int32_t n);
int marl_page_pool_fork(marl_page_pool* p, const int32_t* parent_row, int32_t len, int32_t* child_row);
int marl_page_pool_prepare_append(marl_page_pool* p, int32_t* row, int32_t max_pages, int32_t len,
                                  int32_t* copy_src, int32_t* copy_dst);
int marl_page_pool_drop(marl_page_pool* p, const int32_t* row, int32_t len);
/* *refcount = 0 for a free page; *free_pages = number of free pages (either may be NULL) */
int marl_page_pool_query(const marl_page_pool* p, int32_t page, int32_t* refcount, int32_t* free_pages);

/*
 * Weight synchronisation as ONE copy (the paper's Discussion, "Hardware-Aware Abstraction":
 * updating a rollout engine parameter by parameter is dominated by the control plane, so the
 * weights are aggregated into a single contiguous buffer and synchronised with O(1) operations
 * instead of O(number of parameters)).  marl_pack_tensors gathers n tensors into one
 * contiguous device buffer with a single kernel launch; marl_unpack_tensors scatters such a
 * buffer back into n tensors.  Pure data movement, bit-exact.
 *
 * The caller describes the tensors in a table of marl_pack_entry that lives in DEVICE memory
 * (it is read by the kernel; build it once per model and keep it):
 *   ptr          device address of the tensor's first byte (any alignment; 16-byte aligned
 *                tensors at 16-byte aligned offsets are moved with 16-byte accesses)
 *   offset       where the tensor's bytes start in the packed buffer
 *   bytes        size of the tensor
 *   first_chunk  number of MARL_PACK_CHUNK_BYTES pieces of all earlier entries:
 *                first_chunk[0] = 0, first_chunk[i+1] = first_chunk[i] + ceil(bytes[i] / chunk)
 * marl_pack_plan fills offset (tensors in table order, each start rounded up to 256 bytes) and
 * first_chunk of a HOST copy of the table from its ptr/bytes fields and returns the packed size
 * and the total chunk count, which the two device calls take as arguments.
 * Tensors and packed ranges must not overlap each other.  Errors: MARL_INVALID_ARG for null
 * pointers with n > 0, negative counts, or a plan whose totals do not fit (more than 2^31 - 1
 * chunks).  n = 0 is a no-op.
 */
#define MARL_PACK_CHUNK_BYTES 262144
typedef struct {
  void* ptr;
  uint64_t offset;
  uint64_t bytes;
  uint64_t first_chunk;
} marl_pack_entry;
int marl_pack_plan(marl_pack_entry* entries_host, int32_t n, uint64_t* packed_bytes, int64_t* total_chunks);
int marl_pack_tensors(const marl_pack_entry* entries, int32_t n, int64_t total_chunks, void* packed,
                      void* stream);
int marl_unpack_tensors(const marl_pack_entry* entries, int32_t n, int64_t total_chunks,
                        const void* packed, void* stream);

/*
 * Per-kernel timing of marl_decode_attn / marl_token_logprobs calls (for benchmarks).
 * After marl_profile_begin(max_calls) every call records HIP events around each of its
 * kernels on the call's stream (no synchronisation).  marl_profile_end() synchronises the
 * device, writes the average duration in milliseconds of each stage over the recorded
 * calls (MARL_STAGE_* indices; stages that never ran stay 0), the number of recorded
 * attention calls and log-prob calls, and switches recording off.
 */
enum {
  MARL_STAGE_PLAN = 0, MARL_STAGE_PREFIX = 1, MARL_STAGE_SUFFIX = 2, MARL_STAGE_MERGE = 3,
  MARL_STAGE_LOGPROB = 4, MARL_STAGE_LOGPROB_FINISH = 5, MARL_NUM_STAGES = 6
};
int marl_profile_begin(int32_t max_calls);
int marl_profile_end(float stage_ms[MARL_NUM_STAGES], int32_t* attn_calls, int32_t* logprob_calls);

const char* marl_status_string(int status);
const char* marl_last_hip_error(void);
int marl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MARL_DECODE_H */
