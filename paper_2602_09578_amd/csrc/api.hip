// C ABI of the library: argument validation (before any HIP call), workspace layout,
// kernel launches, optional per-kernel event timing.  See include/marl_decode.h.
#include <math.h>
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "marl_internal.h"

// Workspace of marl_decode_attn_static, the entry point for callers that cannot allocate.
// One array per GPU, part of the library's code object: the device keeps it from the moment the
// library is loaded there until the process ends.  In host code the array's name is only a handle
// for hipGetSymbolAddress; kernels and copies get the address that call returns, per device.
static __device__ __align__(256) unsigned char scratch[MARL_STATIC_WORKSPACE_BYTES];

namespace {

thread_local std::string g_last_hip_error;

int hip_fail(hipError_t e, const char* what) {
  g_last_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  return MARL_HIP_ERROR;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
// device arrays that the kernels read and write as 16-byte vectors
bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }
long ceil_div(long a, long b) { return (a + b - 1) / b; }

int check_shape(const marl_attn_shape* s) {
  if (!s) return MARL_INVALID_ARG;
  if (s->num_seqs < 0 || s->num_groups < 0 || s->num_q_heads <= 0 || s->num_kv_heads <= 0 ||
      s->num_pages < 1 || s->max_prefix_pages < 0 || s->max_suffix_pages < 0)
    return MARL_INVALID_ARG;
  if (s->num_q_heads % s->num_kv_heads != 0) return MARL_INVALID_ARG;
  if (s->head_dim != marl::kD || s->page_size != marl::kPage) return MARL_UNSUPPORTED;
  if (s->num_q_heads / s->num_kv_heads > 16) return MARL_UNSUPPORTED;
  if (s->out_dtype != MARL_OUT_BF16 && s->out_dtype != MARL_OUT_F32) return MARL_UNSUPPORTED;
  const int32_t chunks[2] = {s->suffix_chunk_tokens, s->prefix_chunk_tokens};
  for (int32_t c : chunks)
    if (c != 0 && (c < 32 || c > 65536 || c % 32 != 0)) return MARL_UNSUPPORTED;
  // index arithmetic in the kernels is 32-bit for rows and tokens
  if ((long)s->num_seqs * s->num_q_heads >= (1L << 31)) return MARL_UNSUPPORTED;
  if ((long)s->max_prefix_pages * marl::kPage >= (1L << 30) ||
      (long)s->max_suffix_pages * marl::kPage >= (1L << 30))
    return MARL_UNSUPPORTED;
  return MARL_OK;
}

int make_layout(const marl_attn_shape* s, marl_attn_plan_layout* L) {
  const int rc = check_shape(s);
  if (rc != MARL_OK) return rc;
  if (!L) return MARL_INVALID_ARG;
  memset(L, 0, sizeof *L);
  const long NS = s->num_seqs, NG = s->num_groups, Hkv = s->num_kv_heads, Hq = s->num_q_heads;
  const long mst = (long)s->max_suffix_pages * marl::kPage, mpt = (long)s->max_prefix_pages * marl::kPage;
  // Groups with more than 128 query rows (judged by the average group) use the 8-wave prefix
  // kernel with blocks of 256 rows, so that their prefix KV is streamed once, not twice.
  const long rows = NG > 0 ? ceil_div(NS, NG) * (Hq / Hkv) : 0;   // query rows of an average group
  const long qb = rows > marl::kRowsPerQBlock ? marl::kRowsPerQBlockWide : marl::kRowsPerQBlock;
  // Default chunks: as large as possible (every work item costs a fixed few microseconds and
  // one partial per query row) while the shape still promises enough items to fill the GPU.
  long Cs = s->suffix_chunk_tokens;
  if (Cs == 0) {
    Cs = 8192;
    while (NS * Hkv * ceil_div(mst, Cs) < 2048 && Cs > 256) Cs /= 2;
  }
  long Cp = s->prefix_chunk_tokens;
  if (Cp == 0) {
    const long qblocks = rows > qb ? ceil_div(rows, qb) : 1;
    Cp = 8192;
    const long want = qb == marl::kRowsPerQBlockWide ? 256 : 512;   // about one item per resident workgroup
    while (NG * Hkv * qblocks * ceil_div(mpt, Cp) < want && Cp > 256) Cp /= 2;
  }
  const long NCs = ceil_div(mst, Cs) > 1 ? ceil_div(mst, Cs) : 1;
  const long NCp = ceil_div(mpt, Cp) > 1 ? ceil_div(mpt, Cp) : 1;
  const long R = Hq / Hkv;
  const long max_s_items = NS * NCs;
  const long max_p_items = (NG + NS * R / qb + 1) * NCp;
  if (max_s_items >= (1L << 28) || max_p_items >= (1L << 28)) return MARL_UNSUPPORTED;
  if (NCs >= (1L << 15) || NCp >= (1L << 15)) return MARL_UNSUPPORTED;   // packed into 16 bits each
  L->suffix_chunk_tokens = (int32_t)Cs;
  L->prefix_chunk_tokens = (int32_t)Cp;
  L->suffix_slots = (int32_t)NCs;
  L->prefix_slots = (int32_t)NCp;
  L->rows_per_qblock = (int32_t)qb;
  L->max_suffix_items = (int32_t)max_s_items;
  L->max_prefix_items = (int32_t)max_p_items;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off = align_up(off + bytes, 256); return o; };
  L->counters_off = take(64 * sizeof(int32_t));
  L->group_count_off = take((size_t)NG * 4);
  L->group_start_off = take((size_t)(NG + 1) * 4);
  L->seq_rank_off = take((size_t)NS * 4);
  L->group_tmp_off = take((size_t)NS * 4);
  L->group_seqs_off = take((size_t)NS * 4);
  L->seq_chunks_off = take((size_t)NS * 4);
  L->suffix_items_off = take((size_t)max_s_items * 16);
  L->prefix_items_off = take((size_t)max_p_items * 16);
  L->partial_ml_off = take((size_t)NS * Hq * (NCp + NCs) * 8);
  L->partial_o_off = take((size_t)NS * Hq * (NCp + NCs) * marl::kD * 4);
  L->total_bytes = off;
  return MARL_OK;
}

// ---- per-kernel event timing ---------------------------------------------------------------
struct Profile {
  std::mutex mu;
  bool on = false;
  int max_calls = 0;
  struct Span { hipEvent_t a, b; int stage; };
  std::vector<Span> spans;
  int attn_calls = 0, lp_calls = 0;
} g_prof;

struct StageTimer {
  hipStream_t st;
  bool on;
  explicit StageTimer(hipStream_t s, bool enabled) : st(s), on(enabled) {}
  template <class F>
  hipError_t run(int stage, F&& launch) {
    if (!on) return launch();
    Profile::Span sp{nullptr, nullptr, stage};
    if (hipEventCreate(&sp.a) != hipSuccess || hipEventCreate(&sp.b) != hipSuccess) return launch();
    (void)hipEventRecord(sp.a, st);
    const hipError_t e = launch();
    (void)hipEventRecord(sp.b, st);
    g_prof.spans.push_back(sp);
    return e;
  }
};

int g_num_cus = 0, g_prefix_bpc = 0, g_prefix_wide_bpc = 0, g_suffix_bpc = 0;

std::once_flag g_dev_once;
hipError_t g_dev_err = hipSuccess;

void query_device() {
  int dev = 0;
  g_dev_err = hipGetDevice(&dev);
  if (g_dev_err != hipSuccess) return;
  hipDeviceProp_t p;
  g_dev_err = hipGetDeviceProperties(&p, dev);
  if (g_dev_err != hipSuccess) return;
  g_num_cus = p.multiProcessorCount;
  g_prefix_bpc = marl::prefix_blocks_per_cu(false);
  g_prefix_wide_bpc = marl::prefix_blocks_per_cu(true);
  g_suffix_bpc = marl::suffix_blocks_per_cu();
}

// Points the workspace arrays of `a` into `ws` as the layout says.
void point_workspace(const marl_attn_plan_layout& L, void* ws, marl::AttnArgs& a) {
  char* w = static_cast<char*>(ws);
  a.counters = reinterpret_cast<int32_t*>(w + L.counters_off);
  a.group_count = reinterpret_cast<int32_t*>(w + L.group_count_off);
  a.group_start = reinterpret_cast<int32_t*>(w + L.group_start_off);
  a.seq_rank = reinterpret_cast<int32_t*>(w + L.seq_rank_off);
  a.group_tmp = reinterpret_cast<int32_t*>(w + L.group_tmp_off);
  a.group_seqs = reinterpret_cast<int32_t*>(w + L.group_seqs_off);
  a.seq_chunks = reinterpret_cast<int32_t*>(w + L.seq_chunks_off);
  a.suffix_items = reinterpret_cast<int4*>(w + L.suffix_items_off);
  a.prefix_items = reinterpret_cast<int4*>(w + L.prefix_items_off);
  a.partial_ml = reinterpret_cast<float2*>(w + L.partial_ml_off);
  a.partial_o = reinterpret_cast<float*>(w + L.partial_o_off);
}

// The shape-derived fields of `a` (everything but pointers).
void fill_shape_args(const marl_attn_shape* s, const marl_attn_plan_layout& L, marl::AttnArgs& a) {
  memset(&a, 0, sizeof a);
  a.NS = s->num_seqs;
  a.NG = s->num_groups;
  a.Hq = s->num_q_heads;
  a.Hkv = s->num_kv_heads;
  a.R = a.Hq / a.Hkv;
  a.num_pages = s->num_pages;
  a.max_pp = s->max_prefix_pages;
  a.max_sp = s->max_suffix_pages;
  a.Cs = L.suffix_chunk_tokens;
  a.Cp = L.prefix_chunk_tokens;
  a.NCs = L.suffix_slots;
  a.NCp = L.prefix_slots;
  a.qblock_rows = L.rows_per_qblock;
  a.out_dtype = s->out_dtype;
}

int fill_args(const marl_attn_shape* s, void* ws, size_t ws_bytes, marl::AttnArgs& a) {
  marl_attn_plan_layout L;
  const int rc = make_layout(s, &L);
  if (rc != MARL_OK) return rc;
  if (!ws) return MARL_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return MARL_INVALID_ARG;
  if (ws_bytes < L.total_bytes) return MARL_WORKSPACE_TOO_SMALL;
  fill_shape_args(s, L, a);
  point_workspace(L, ws, a);
  return MARL_OK;
}

// Validates the operands of a decode-attention call (host-only) and stores them in `a`, whose
// shape fields are already set.
int take_attn_operands(marl::AttnArgs& a, const void* q, const void* k_pages, const void* v_pages,
                       const int32_t* prefix_block_table, const int32_t* suffix_block_table,
                       const int32_t* prefix_lens, const int32_t* suffix_lens,
                       const int32_t* group_of_seq, float scale, void* out) {
  if (!isfinite(scale)) return MARL_INVALID_ARG;
  if (a.NS > 0 && (!q || !out || !suffix_lens || !group_of_seq || !k_pages || !v_pages)) return MARL_INVALID_ARG;
  if (a.NS > 0 && a.max_sp > 0 && !suffix_block_table) return MARL_INVALID_ARG;
  if (a.NG > 0 && (!prefix_lens || (a.max_pp > 0 && !prefix_block_table))) return MARL_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_pages) || !aligned16(v_pages) || !aligned16(out)) return MARL_INVALID_ARG;
  a.q = static_cast<const uint16_t*>(q);
  a.k_pages = static_cast<const uint16_t*>(k_pages);
  a.v_pages = static_cast<const uint16_t*>(v_pages);
  a.prefix_table = prefix_block_table;
  a.suffix_table = suffix_block_table;
  a.prefix_lens = prefix_lens;
  a.suffix_lens = suffix_lens;
  a.group_of_seq = group_of_seq;
  a.scale = scale;
  a.out = out;
  return MARL_OK;
}

// Enqueues the kernels of one decode-attention call.  `may_time`: the call takes part in the
// per-kernel event timing when that is switched on (events are created then).
int enqueue_decode_attn(const marl::AttnArgs& a, hipStream_t st, bool may_time) {
  std::call_once(g_dev_once, query_device);
  if (g_dev_err != hipSuccess) return hip_fail(g_dev_err, "device query");

  std::unique_lock<std::mutex> lock(g_prof.mu, std::defer_lock);
  bool timed = false;
  if (may_time && g_prof.on) {
    lock.lock();
    timed = g_prof.on && g_prof.attn_calls < g_prof.max_calls;
    if (timed) ++g_prof.attn_calls; else lock.unlock();
  }
  StageTimer T(st, timed);
  hipError_t e;
  if ((e = T.run(MARL_STAGE_PLAN, [&] { return marl::launch_plan(a, st); })) != hipSuccess)
    return hip_fail(e, "plan kernel");
  {  // always launched: its workgroups also process the short suffix items
    if ((e = T.run(MARL_STAGE_PREFIX, [&] { return marl::launch_prefix(a, g_num_cus * (a.qblock_rows == marl::kRowsPerQBlockWide ? g_prefix_wide_bpc : g_prefix_bpc), st); })) != hipSuccess)
      return hip_fail(e, "prefix kernel");
  }
  // the suffix kernel takes the items of more than kShortTokens tokens: none can exist when
  // neither a table row nor a chunk holds that many
  if ((long)a.max_sp * marl::kPage > marl::kShortTokens && a.Cs > marl::kShortTokens) {
    if ((e = T.run(MARL_STAGE_SUFFIX, [&] { return marl::launch_suffix(a, g_num_cus * g_suffix_bpc, st); })) != hipSuccess)
      return hip_fail(e, "suffix kernel");
  }
  if ((e = T.run(MARL_STAGE_MERGE, [&] { return marl::launch_merge(a, st); })) != hipSuccess)
    return hip_fail(e, "merge kernel");
  return MARL_OK;
}

// ---- workspace for callers that cannot allocate (the array itself is at the top of this file) ----
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Plain one-word store, for a flag word that no kernel of an empty call would write.
__global__ void store_word_kernel(int32_t* dst, int32_t value) { *dst = value; }

int static_scratch_of_current_device(void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return MARL_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!p || reinterpret_cast<uintptr_t>(p) % 256 != 0) {
      g_last_hip_error = "hipGetSymbolAddress(scratch): unusable address";
      return MARL_HIP_ERROR;
    }
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return MARL_OK;
}

}  // namespace

extern "C" {

int marl_version(void) { return 1; }

const char* marl_status_string(int status) {
  switch (status) {
    case MARL_OK: return "ok";
    case MARL_INVALID_ARG: return "invalid argument";
    case MARL_UNSUPPORTED: return "unsupported shape or option";
    case MARL_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MARL_HIP_ERROR: return "HIP error";
    case MARL_OUT_OF_MEMORY: return "out of host memory";
    default: return "unknown status";
  }
}

const char* marl_last_hip_error(void) { return g_last_hip_error.c_str(); }

int marl_attn_plan_layout_for(const marl_attn_shape* shape, marl_attn_plan_layout* layout) {
  return make_layout(shape, layout);
}

int marl_workspace_bytes(const marl_attn_shape* shape, size_t* bytes) {
  if (!bytes) return MARL_INVALID_ARG;
  marl_attn_plan_layout L;
  const int rc = make_layout(shape, &L);
  if (rc != MARL_OK) return rc;
  *bytes = L.total_bytes;
  return MARL_OK;
}

int marl_attn_plan(const marl_attn_shape* shape, void* workspace, size_t workspace_bytes,
                   const int32_t* prefix_lens, const int32_t* suffix_lens,
                   const int32_t* group_of_seq, void* stream) {
  marl::AttnArgs a;
  const int rc = fill_args(shape, workspace, workspace_bytes, a);
  if (rc != MARL_OK) return rc;
  if ((a.NG > 0 && !prefix_lens) || (a.NS > 0 && (!suffix_lens || !group_of_seq))) return MARL_INVALID_ARG;
  a.prefix_lens = prefix_lens;
  a.suffix_lens = suffix_lens;
  a.group_of_seq = group_of_seq;
  const hipError_t e = marl::launch_plan(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MARL_OK : hip_fail(e, "plan kernel");
}

int marl_decode_attn(const marl_attn_shape* shape, void* workspace, size_t workspace_bytes,
                     const void* q, const void* k_pages, const void* v_pages,
                     const int32_t* prefix_block_table, const int32_t* suffix_block_table,
                     const int32_t* prefix_lens, const int32_t* suffix_lens,
                     const int32_t* group_of_seq, float scale, void* out, void* stream) {
  marl::AttnArgs a;
  int rc = fill_args(shape, workspace, workspace_bytes, a);
  if (rc != MARL_OK) return rc;
  rc = take_attn_operands(a, q, k_pages, v_pages, prefix_block_table, suffix_block_table, prefix_lens,
                          suffix_lens, group_of_seq, scale, out);
  if (rc != MARL_OK) return rc;
  if (a.NS == 0) return MARL_OK;
  return enqueue_decode_attn(a, static_cast<hipStream_t>(stream), /*may_time=*/true);
}

int marl_decode_attn_static(const marl_attn_shape* shape,
                            const void* q, const void* k_pages, const void* v_pages,
                            const int32_t* prefix_block_table, const int32_t* suffix_block_table,
                            const int32_t* prefix_lens, const int32_t* suffix_lens,
                            const int32_t* group_of_seq, float scale, void* out, int32_t* flags,
                            void* stream) {
  // host-only checks first: the shape, its workspace need against the fixed capacity, the operands
  marl_attn_plan_layout L;
  int rc = make_layout(shape, &L);
  if (rc != MARL_OK) return rc;
  if (L.total_bytes > MARL_STATIC_WORKSPACE_BYTES) return MARL_WORKSPACE_TOO_SMALL;
  marl::AttnArgs a;
  fill_shape_args(shape, L, a);
  rc = take_attn_operands(a, q, k_pages, v_pages, prefix_block_table, suffix_block_table, prefix_lens,
                          suffix_lens, group_of_seq, scale, out);
  if (rc != MARL_OK) return rc;
  if (reinterpret_cast<uintptr_t>(flags) % 4 != 0) return MARL_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (a.NS == 0) {
    if (flags) {   // no kernel of the call runs, so none could have set a flag
      hipLaunchKernelGGL(store_word_kernel, dim3(1), dim3(1), 0, st, flags, 0);
      const hipError_t e = hipGetLastError();
      if (e != hipSuccess) return hip_fail(e, "flag store kernel");
    }
    return MARL_OK;
  }
  void* ws = nullptr;
  rc = static_scratch_of_current_device(&ws);
  if (rc != MARL_OK) return rc;
  point_workspace(L, ws, a);   // the plan kernel clears the counters and flags it finds there
  rc = enqueue_decode_attn(a, st, /*may_time=*/false);
  if (rc != MARL_OK) return rc;
  if (flags) {
    const hipError_t e = hipMemcpyAsync(flags, a.counters + MARL_CTR_FLAGS, sizeof(int32_t),
                                        hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) return hip_fail(e, "copy flags");
  }
  return MARL_OK;
}

int marl_attn_read_flags(const void* workspace, int32_t* flags_host, void* stream) {
  if (!workspace || !flags_host) return MARL_INVALID_ARG;
  const int32_t* ctr = static_cast<const int32_t*>(workspace);   // counters sit at offset 0
  hipError_t e = hipMemcpyAsync(flags_host, ctr + MARL_CTR_FLAGS, sizeof(int32_t), hipMemcpyDeviceToHost,
                                static_cast<hipStream_t>(stream));
  if (e == hipSuccess) e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MARL_OK : hip_fail(e, "read flags");
}

// ---- KV-cache maintenance ---------------------------------------------------------------------
int marl_kv_append(const marl_attn_shape* shape, const void* k_new, const void* v_new,
                   void* k_pages, void* v_pages, const int32_t* suffix_block_table,
                   int32_t* suffix_lens, int32_t* flags, void* stream) {
  const int rc = check_shape(shape);
  if (rc != MARL_OK) return rc;
  if (shape->num_seqs == 0) return MARL_OK;
  if (!k_new || !v_new || !k_pages || !v_pages || !suffix_block_table || !suffix_lens) return MARL_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_pages) || !aligned16(v_pages)) return MARL_INVALID_ARG;
  if (shape->max_suffix_pages < 1) return MARL_INVALID_ARG;
  marl::KvAppendArgs a;
  a.k_new = static_cast<const uint16_t*>(k_new);
  a.v_new = static_cast<const uint16_t*>(v_new);
  a.k_pages = static_cast<uint16_t*>(k_pages);
  a.v_pages = static_cast<uint16_t*>(v_pages);
  a.suffix_table = suffix_block_table;
  a.suffix_lens = suffix_lens;
  a.flags = flags;
  a.NS = shape->num_seqs;
  a.Hkv = shape->num_kv_heads;
  a.num_pages = shape->num_pages;
  a.max_sp = shape->max_suffix_pages;
  const hipError_t e = marl::launch_kv_append(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MARL_OK : hip_fail(e, "kv append kernel");
}

int marl_kv_copy_pages(const marl_attn_shape* shape, void* k_pages, void* v_pages,
                       const int32_t* src, const int32_t* dst, int32_t n, int32_t* flags,
                       void* stream) {
  const int rc = check_shape(shape);
  if (rc != MARL_OK) return rc;
  if (n < 0 || n >= (1 << 30)) return MARL_INVALID_ARG;
  if (n == 0) return MARL_OK;
  if (!k_pages || !v_pages || !src || !dst) return MARL_INVALID_ARG;
  if (!aligned16(k_pages) || !aligned16(v_pages)) return MARL_INVALID_ARG;
  marl::KvCopyArgs a;
  a.k_pages = static_cast<uint16_t*>(k_pages);
  a.v_pages = static_cast<uint16_t*>(v_pages);
  a.src = src;
  a.dst = dst;
  a.flags = flags;
  a.n = n;
  a.Hkv = shape->num_kv_heads;
  a.num_pages = shape->num_pages;
  const hipError_t e = marl::launch_kv_copy_pages(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MARL_OK : hip_fail(e, "kv copy kernel");
}

// ---- log-probabilities ------------------------------------------------------------------------
static int logprob_split(int32_t rows, int32_t vocab, int32_t* slices, int32_t* slice_len) {
  if (rows < 0 || vocab < 1) return MARL_INVALID_ARG;
  long want = rows > 0 ? (1024 + rows - 1) / rows : 1;     // aim for >= 1024 workgroups (of 1024 threads)
  long len = (vocab + want - 1) / want;
  if (len < 8192) len = 8192;                              // but keep slices worth a workgroup
  len = (len + 2047) / 2048 * 2048;
  *slice_len = (int32_t)(len > vocab ? ((long)vocab + 7) / 8 * 8 : len);
  *slices = (int32_t)(((long)vocab + *slice_len - 1) / *slice_len);
  return MARL_OK;
}

int marl_logprobs_workspace_bytes(int32_t rows, int32_t vocab, size_t* bytes) {
  if (!bytes) return MARL_INVALID_ARG;
  int32_t slices, slice_len;
  const int rc = logprob_split(rows, vocab, &slices, &slice_len);
  if (rc != MARL_OK) return rc;
  *bytes = slices > 1 ? (size_t)rows * slices * sizeof(float2) : 0;
  return MARL_OK;
}

int marl_token_logprobs(const void* logits, const int32_t* tokens, float temperature, float* out,
                        int32_t rows, int32_t vocab, void* workspace, size_t workspace_bytes,
                        void* stream) {
  marl::LogprobArgs a;
  memset(&a, 0, sizeof a);
  const int rc = logprob_split(rows, vocab, &a.slices, &a.slice_len);
  if (rc != MARL_OK) return rc;
  if (!isfinite(temperature) || !(temperature > 0.f)) return MARL_INVALID_ARG;
  if ((long)rows * a.slices >= (1L << 31)) return MARL_UNSUPPORTED;
  if (rows == 0) return MARL_OK;
  if (!logits || !tokens || !out) return MARL_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(logits) % 2 != 0) return MARL_INVALID_ARG;
  const size_t need = a.slices > 1 ? (size_t)rows * a.slices * sizeof(float2) : 0;
  if (need > 0) {
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 8 != 0) return MARL_INVALID_ARG;
    if (workspace_bytes < need) return MARL_WORKSPACE_TOO_SMALL;
  }
  a.logits = static_cast<const uint16_t*>(logits);
  a.tokens = tokens;
  a.out = out;
  a.partials = static_cast<float2*>(workspace);
  a.rows = rows;
  a.vocab = vocab;
  a.inv_temp_log2e = 1.44269504088896340736f / temperature;
  hipStream_t st = static_cast<hipStream_t>(stream);

  std::unique_lock<std::mutex> lock(g_prof.mu, std::defer_lock);
  bool timed = false;
  if (g_prof.on) {
    lock.lock();
    timed = g_prof.on && g_prof.lp_calls < g_prof.max_calls;
    if (timed) ++g_prof.lp_calls; else lock.unlock();
  }
  StageTimer T(st, timed);
  hipError_t e;
  if ((e = T.run(MARL_STAGE_LOGPROB, [&] { return marl::launch_logprobs(a, st); })) != hipSuccess)
    return hip_fail(e, "logprob kernel");
  if (a.slices > 1) {
    if ((e = T.run(MARL_STAGE_LOGPROB_FINISH, [&] { return marl::launch_logprobs_finish(a, st); })) != hipSuccess)
      return hip_fail(e, "logprob finish kernel");
  }
  return MARL_OK;
}

// ---- sampling -----------------------------------------------------------------------------------
int marl_sample_workspace_bytes(int32_t rows, int32_t vocab, size_t* bytes) {
  if (!bytes || rows < 0 || vocab < 1) return MARL_INVALID_ARG;
  *bytes = (size_t)rows * marl::sample_num_chunks(vocab) * sizeof(float2);
  return MARL_OK;
}

int marl_sample_tokens(const void* logits, const float* uniforms, float temperature,
                       int32_t* out_tokens, float* out_logprobs, int32_t rows, int32_t vocab,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (rows < 0 || vocab < 1) return MARL_INVALID_ARG;
  if (!isfinite(temperature) || !(temperature > 0.f)) return MARL_INVALID_ARG;
  if (rows == 0) return MARL_OK;
  if (!logits || !uniforms || !out_tokens || !out_logprobs || !workspace) return MARL_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(logits) % 2 != 0 || reinterpret_cast<uintptr_t>(workspace) % 8 != 0)
    return MARL_INVALID_ARG;
  marl::SampleArgs a;
  memset(&a, 0, sizeof a);
  a.num_chunks = marl::sample_num_chunks(vocab);
  if (workspace_bytes < (size_t)rows * a.num_chunks * sizeof(float2)) return MARL_WORKSPACE_TOO_SMALL;
  // a workgroup (4 waves) covers 4 * chunks_per_wave chunks of a row; aim for >= 2048 workgroups
  const long want_groups = rows >= 2048 ? 1 : (2048 + rows - 1) / rows;
  long cpw = (a.num_chunks + 4 * want_groups - 1) / (4 * want_groups);
  if (cpw < 1) cpw = 1;
  a.chunks_per_wave = (int32_t)cpw;
  a.groups_per_row = (int32_t)((a.num_chunks + 4 * cpw - 1) / (4 * cpw));
  if ((long)rows * a.groups_per_row >= (1L << 31)) return MARL_UNSUPPORTED;
  a.logits = static_cast<const uint16_t*>(logits);
  a.uniforms = uniforms;
  a.out_tokens = out_tokens;
  a.out_logprobs = out_logprobs;
  a.partials = static_cast<float2*>(workspace);
  a.rows = rows;
  a.vocab = vocab;
  a.inv_temp_log2e = 1.44269504088896340736f / temperature;
  const hipError_t e = marl::launch_sample(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MARL_OK : hip_fail(e, "sampling kernels");
}

int marl_sample_tokens_top_p(const void* logits, const float* uniforms, float temperature,
                             float top_p, int32_t* out_tokens, float* out_logprobs, int32_t rows,
                             int32_t vocab, void* stream) {
  if (rows < 0 || vocab < 1) return MARL_INVALID_ARG;
  if (!isfinite(temperature) || !(temperature > 0.f)) return MARL_INVALID_ARG;
  if (!(top_p > 0.f) || !(top_p <= 1.f)) return MARL_INVALID_ARG;
  if (vocab > marl::top_p_max_vocab()) return MARL_UNSUPPORTED;
  if (rows == 0) return MARL_OK;
  if (!logits || !uniforms || !out_tokens || !out_logprobs) return MARL_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(logits) % 2 != 0) return MARL_INVALID_ARG;
  marl::TopPArgs a;
  a.logits = static_cast<const uint16_t*>(logits);
  a.uniforms = uniforms;
  a.out_tokens = out_tokens;
  a.out_logprobs = out_logprobs;
  a.rows = rows;
  a.vocab = vocab;
  a.inv_temp_log2e = 1.44269504088896340736f / temperature;
  a.top_p = top_p;
  const hipError_t e = marl::launch_sample_top_p(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MARL_OK : hip_fail(e, "top-p sampling kernel");
}

// ---- prefill ------------------------------------------------------------------------------------
namespace {
int check_prefill_shape(const marl_prefill_shape* s) {
  if (!s) return MARL_INVALID_ARG;
  if (s->num_tokens < 0 || s->num_groups < 0 || s->num_q_heads <= 0 || s->num_kv_heads <= 0 ||
      s->num_pages < 1 || s->max_prefix_pages < 0)
    return MARL_INVALID_ARG;
  if (s->num_q_heads % s->num_kv_heads != 0) return MARL_INVALID_ARG;
  if (s->head_dim != marl::kD || s->page_size != marl::kPage) return MARL_UNSUPPORTED;
  if (s->num_q_heads / s->num_kv_heads > 16) return MARL_UNSUPPORTED;
  if (s->out_dtype != MARL_OUT_BF16 && s->out_dtype != MARL_OUT_F32) return MARL_UNSUPPORTED;
  if ((long)s->num_tokens * s->num_q_heads >= (1L << 31)) return MARL_UNSUPPORTED;   // 32-bit row indices
  if ((long)s->max_prefix_pages * marl::kPage >= (1L << 30)) return MARL_UNSUPPORTED;
  return MARL_OK;
}
constexpr size_t kPrefillHeaderBytes = 256;   // counters
size_t prefill_start_bytes(const marl_prefill_shape* s) {
  return align_up(((size_t)s->num_groups + 1) * sizeof(int32_t), 256);
}
long prefill_max_blocks(const marl_prefill_shape* s) {   // row blocks of all groups, upper bound
  const long R = s->num_q_heads / s->num_kv_heads;
  return (long)s->num_tokens * R / marl::prefill_rows_per_block() + s->num_groups;
}
size_t prefill_ws_bytes(const marl_prefill_shape* s) {
  return kPrefillHeaderBytes + prefill_start_bytes(s) + align_up((size_t)prefill_max_blocks(s) * sizeof(int2), 256);
}
void fill_prefill_args(const marl_prefill_shape* s, marl::PrefillArgs& a) {
  memset(&a, 0, sizeof a);
  a.NT = s->num_tokens;
  a.NG = s->num_groups;
  a.Hq = s->num_q_heads;
  a.Hkv = s->num_kv_heads;
  a.R = a.Hq / a.Hkv;
  a.num_pages = s->num_pages;
  a.max_pp = s->max_prefix_pages;
  a.out_dtype = s->out_dtype;
}
}  // namespace

int marl_prefill_workspace_bytes(const marl_prefill_shape* shape, size_t* bytes) {
  const int rc = check_prefill_shape(shape);
  if (rc != MARL_OK) return rc;
  if (!bytes) return MARL_INVALID_ARG;
  *bytes = prefill_ws_bytes(shape);
  return MARL_OK;
}

int marl_prefill_attn(const marl_prefill_shape* shape, void* workspace, size_t workspace_bytes,
                      const void* q, const void* k_pages, const void* v_pages,
                      const int32_t* prefix_block_table, const int32_t* q_start,
                      const int32_t* q_pos0, float scale, void* out, void* stream) {
  const int rc = check_prefill_shape(shape);
  if (rc != MARL_OK) return rc;
  if (!isfinite(scale)) return MARL_INVALID_ARG;
  if (shape->num_tokens == 0 || shape->num_groups == 0) return MARL_OK;
  if (!workspace || !q || !k_pages || !v_pages || !prefix_block_table || !q_start || !q_pos0 || !out)
    return MARL_INVALID_ARG;
  if (shape->max_prefix_pages < 1) return MARL_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0 || reinterpret_cast<uintptr_t>(q) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(k_pages) % 16 != 0 || reinterpret_cast<uintptr_t>(v_pages) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(out) % 16 != 0)
    return MARL_INVALID_ARG;
  if (workspace_bytes < prefill_ws_bytes(shape)) return MARL_WORKSPACE_TOO_SMALL;
  marl::PrefillArgs a;
  fill_prefill_args(shape, a);
  a.q = static_cast<const uint16_t*>(q);
  a.k_pages = static_cast<const uint16_t*>(k_pages);
  a.v_pages = static_cast<const uint16_t*>(v_pages);
  a.prefix_table = prefix_block_table;
  a.q_start = q_start;
  a.q_pos0 = q_pos0;
  a.out = out;
  a.counters = static_cast<int32_t*>(workspace);
  a.block_start = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + kPrefillHeaderBytes);
  a.items = reinterpret_cast<int2*>(static_cast<char*>(workspace) + kPrefillHeaderBytes + prefill_start_bytes(shape));
  if (prefill_max_blocks(shape) >= (1L << 28)) return MARL_UNSUPPORTED;
  a.max_blocks = (int32_t)prefill_max_blocks(shape);
  a.scale = scale;
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return hip_fail(e, "device query");
  // no more workgroups than the shape can have row blocks
  const long max_items = prefill_max_blocks(shape) * a.Hkv;
  long grid = (long)cus * marl::prefill_blocks_per_cu();
  if (grid > max_items) grid = max_items;
  if (grid < 1) grid = 1;
  e = marl::launch_prefill(a, (int)grid, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MARL_OK : hip_fail(e, "prefill kernels");
}

int marl_kv_write_prompt(const marl_prefill_shape* shape, const void* k_new, const void* v_new,
                         void* k_pages, void* v_pages, const int32_t* prefix_block_table,
                         const int32_t* q_start, const int32_t* q_pos0, int32_t* flags,
                         void* stream) {
  const int rc = check_prefill_shape(shape);
  if (rc != MARL_OK) return rc;
  if (shape->num_tokens == 0 || shape->num_groups == 0) return MARL_OK;
  if (!k_new || !v_new || !k_pages || !v_pages || !prefix_block_table || !q_start || !q_pos0)
    return MARL_INVALID_ARG;
  if (shape->max_prefix_pages < 1) return MARL_INVALID_ARG;
  // one workgroup per (group, KV head, table column)
  if ((long)shape->num_groups * shape->num_kv_heads * shape->max_prefix_pages >= (1L << 31)) return MARL_UNSUPPORTED;
  // keys are copied, and whole value pages stored, as 16-byte vectors
  if (!aligned16(k_new) || !aligned16(k_pages) || !aligned16(v_pages)) return MARL_INVALID_ARG;
  marl::PrefillArgs a;
  fill_prefill_args(shape, a);
  a.k_new = static_cast<const uint16_t*>(k_new);
  a.v_new = static_cast<const uint16_t*>(v_new);
  a.k_pages_w = static_cast<uint16_t*>(k_pages);
  a.v_pages_w = static_cast<uint16_t*>(v_pages);
  a.prefix_table = prefix_block_table;
  a.q_start = q_start;
  a.q_pos0 = q_pos0;
  a.flags = flags;
  const hipError_t e = marl::launch_kv_write_prompt(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MARL_OK : hip_fail(e, "prompt scatter kernel");
}

// ---- GRPO advantages ----------------------------------------------------------------------------
int marl_grpo_advantages(const float* rewards, const int32_t* group_start, const int32_t* group_seqs,
                         int32_t num_groups, float eps, float* out, void* stream) {
  if (num_groups < 0 || !isfinite(eps) || eps < 0.f) return MARL_INVALID_ARG;
  if (num_groups == 0) return MARL_OK;
  if (!rewards || !group_start || !group_seqs || !out) return MARL_INVALID_ARG;
  marl::GrpoArgs a;
  a.rewards = rewards;
  a.group_start = group_start;
  a.group_seqs = group_seqs;
  a.out = out;
  a.num_groups = num_groups;
  a.eps = eps;
  const hipError_t e = marl::launch_grpo_advantages(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MARL_OK : hip_fail(e, "advantage kernel");
}

// ---- weight synchronisation as one copy ------------------------------------------------------
int marl_pack_plan(marl_pack_entry* entries, int32_t n, uint64_t* packed_bytes, int64_t* total_chunks) {
  if (n < 0 || !packed_bytes || !total_chunks || (n > 0 && !entries)) return MARL_INVALID_ARG;
  uint64_t off = 0, chunks = 0;
  for (int32_t i = 0; i < n; ++i) {
    if (entries[i].bytes > 0 && !entries[i].ptr) return MARL_INVALID_ARG;
    off = (off + 255) & ~(uint64_t)255;
    entries[i].offset = off;
    entries[i].first_chunk = chunks;
    if (entries[i].bytes > (uint64_t)1 << 46) return MARL_INVALID_ARG;
    off += entries[i].bytes;
    chunks += (entries[i].bytes + MARL_PACK_CHUNK_BYTES - 1) / MARL_PACK_CHUNK_BYTES;
    if (chunks > 0x7fffffffull) return MARL_INVALID_ARG;
  }
  *packed_bytes = off;
  *total_chunks = (int64_t)chunks;
  return MARL_OK;
}

#ifndef MARL_PACK_BLOCKS_PER_CU
#define MARL_PACK_BLOCKS_PER_CU 2
#endif
namespace {
int pack_call(const marl_pack_entry* entries, int32_t n, int64_t total_chunks, void* packed, int unpack,
              void* stream) {
  if (n < 0 || total_chunks < 0 || total_chunks > 0x7fffffffll) return MARL_INVALID_ARG;
  if (n == 0 || total_chunks == 0) return MARL_OK;
  if (!entries || !packed) return MARL_INVALID_ARG;
  std::call_once(g_dev_once, query_device);
  if (g_dev_err != hipSuccess) return hip_fail(g_dev_err, "device query");
  marl::PackArgs a;
  a.entries = entries;
  a.packed = static_cast<char*>(packed);
  a.n = n;
  a.total_chunks = (int32_t)total_chunks;
  a.unpack = unpack;
  const hipError_t e = marl::launch_pack(a, g_num_cus * MARL_PACK_BLOCKS_PER_CU, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? MARL_OK : hip_fail(e, "pack kernel");
}
}  // namespace

int marl_pack_tensors(const marl_pack_entry* entries, int32_t n, int64_t total_chunks, void* packed,
                      void* stream) {
  return pack_call(entries, n, total_chunks, packed, 0, stream);
}
int marl_unpack_tensors(const marl_pack_entry* entries, int32_t n, int64_t total_chunks,
                        const void* packed, void* stream) {
  return pack_call(entries, n, total_chunks, const_cast<void*>(packed), 1, stream);
}

// ---- profiling ----------------------------------------------------------------------------------
int marl_profile_begin(int32_t max_calls) {
  if (max_calls < 1 || max_calls > (1 << 20)) return MARL_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  for (auto& sp : g_prof.spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
  g_prof.spans.clear();
  g_prof.attn_calls = g_prof.lp_calls = 0;
  g_prof.max_calls = max_calls;
  g_prof.on = true;
  return MARL_OK;
}

int marl_profile_end(float stage_ms[MARL_NUM_STAGES], int32_t* attn_calls, int32_t* logprob_calls) {
  if (!stage_ms) return MARL_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  g_prof.on = false;
  for (int i = 0; i < MARL_NUM_STAGES; ++i) stage_ms[i] = 0.f;
  int rc = MARL_OK;
  if (!g_prof.spans.empty()) {
    const hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) rc = hip_fail(e, "profile sync");
  }
  double sum[MARL_NUM_STAGES] = {0};
  for (auto& sp : g_prof.spans) {
    float ms = 0.f;
    if (rc == MARL_OK && hipEventElapsedTime(&ms, sp.a, sp.b) == hipSuccess) sum[sp.stage] += ms;
    (void)hipEventDestroy(sp.a);
    (void)hipEventDestroy(sp.b);
  }
  g_prof.spans.clear();
  for (int i = 0; i < MARL_NUM_STAGES; ++i) {
    const int n = i <= MARL_STAGE_MERGE ? g_prof.attn_calls : g_prof.lp_calls;
    stage_ms[i] = n > 0 ? (float)(sum[i] / n) : 0.f;
  }
  if (attn_calls) *attn_calls = g_prof.attn_calls;
  if (logprob_calls) *logprob_calls = g_prof.lp_calls;
  return rc;
}

}  // extern "C"
