// C-ABI layer of libpe (see include/pe.h): argument validation on the host, then kernel launches on
// the caller's stream.  Nothing here allocates, frees or synchronises.
#include "../../include/pe.h"

#include <atomic>
#include <mutex>

#include "pe_launch.h"

// Split partials of pe_paged_decode_static: one copy per GPU, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[PE_STATIC_SCRATCH_BYTES];

namespace {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// The decode workgroup shapes that are built (waves*100 + register buffers*10 + wave-loads per tile).
bool decode_shape_built(int shape) { return shape == 422 || shape == 424 || shape == 432 || shape == 822; }

// PE_OK if the descriptor names a shape the kernels are built for.
int check_desc(const pe_cache_desc* d) {
  if (d == nullptr) return PE_ERR_INVALID_ARG;
  if (d->dtype != PE_F32 && d->dtype != PE_BF16) return PE_ERR_UNSUPPORTED;
  if (d->num_seqs < 1 || d->num_kv_heads < 1 || d->num_q_heads < 1 || d->max_blocks < 1 || d->num_phys_blocks < 1)
    return PE_ERR_INVALID_ARG;
  if (d->num_q_heads % d->num_kv_heads != 0) return PE_ERR_INVALID_ARG;
  if (d->num_q_heads / d->num_kv_heads > 8) return PE_ERR_UNSUPPORTED;
  if (d->head_dim != 64 && d->head_dim != 128) return PE_ERR_UNSUPPORTED;
  if (d->block_size != 16 && d->block_size != 32 && d->block_size != 64 && d->block_size != 128)
    return PE_ERR_UNSUPPORTED;
  if (d->layout != PE_LAYOUT_PER_HEAD && d->layout != PE_LAYOUT_SHARED) return PE_ERR_UNSUPPORTED;
  if (d->num_phys_blocks > 0x7fffffffLL) return PE_ERR_UNSUPPORTED;
  if ((int64_t)d->num_seqs * d->num_kv_heads > 0x7fffffffLL / 64) return PE_ERR_UNSUPPORTED;
  if (d->decode_splits < 0 || d->decode_splits > 256) return PE_ERR_INVALID_ARG;
  if (d->decode_flat_order != 0 && d->decode_flat_order != 1) return PE_ERR_INVALID_ARG;
  if (d->decode_shape != 0) {
    if (!decode_shape_built(d->decode_shape)) return PE_ERR_UNSUPPORTED;
    const bool tunable = d->dtype == PE_BF16 && d->head_dim == 128 && d->num_q_heads / d->num_kv_heads == 4 &&
                         d->layout == PE_LAYOUT_PER_HEAD;
    if (d->decode_shape != 422 && !tunable) return PE_ERR_UNSUPPORTED;
  }
  return PE_OK;
}

// Compute units of the current device, asked of the HIP runtime once per device.  Without a device (or on an
// error) the count of an MI355X is assumed; the sticky error state of the runtime is left clean.
int compute_units() {
  constexpr int kMaxDevices = 64, kDefault = 256;
  static std::atomic<int> cached[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return kDefault;
  }
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
    (void)hipGetLastError();
    return kDefault;
  }
  cached[dev].store(n, std::memory_order_relaxed);
  return n;
}

// Number of splits of a row in the attention calls.  The kernel streams best with ONE four-wave workgroup per
// compute unit (each wave keeps a tile in flight while it consumes another; more resident workgroups only
// add prologue, epilogue and merge work), so rows are split just enough to cover the compute units of the
// device, and never into splits shorter than 256 tokens.
int decode_splits(const pe_cache_desc* d) {
  if (d->decode_splits > 0) return d->decode_splits;
  const int64_t rows = (int64_t)d->num_seqs * d->num_kv_heads;
  const int64_t cus = compute_units();
  int64_t splits = (cus + rows - 1) / rows;
  const int64_t max_tokens = (int64_t)d->max_blocks * d->block_size;
  const int64_t max_by_len = max_tokens / 256 > 1 ? max_tokens / 256 : 1;
  if (splits > max_by_len) splits = max_by_len;
  if (splits > 64) splits = 64;
  if (splits < 1) splits = 1;
  return (int)splits;
}

int check_workspace(const void* ws, size_t have, size_t need) {
  if (need == 0) return PE_OK;
  if (ws == nullptr || have < need || !aligned(ws, 256)) return PE_ERR_WORKSPACE;
  return PE_OK;
}

bool finite(float x) { return x == x && x - x == 0.f; }

// The part of the attention launch description that follows from the descriptor alone.
pe::DecodeArgs decode_args(const pe_cache_desc* desc, int splits) {
  pe::DecodeArgs a;
  a.num_seqs = desc->num_seqs;
  a.num_kv_heads = desc->num_kv_heads;
  a.num_q_heads = desc->num_q_heads;
  a.head_dim = desc->head_dim;
  a.block_size = desc->block_size;
  a.max_blocks = desc->max_blocks;
  a.splits = splits;
  a.xcd_map = desc->decode_flat_order ? 0 : 1;
  const int shape = desc->decode_shape != 0 ? desc->decode_shape : 422;
  a.waves = shape / 100;
  a.depth = shape / 10 % 10;
  a.loads = shape % 10;
  a.is_bf16 = desc->dtype == PE_BF16;
  a.shared = desc->layout == PE_LAYOUT_SHARED;
  return a;
}

}  // namespace

extern "C" {

int pe_version(void) { return 300; }  // 0.3.0: per-descriptor launch shape replaces the process-wide options

const char* pe_status_string(int status) {
  switch (status) {
    case PE_OK: return "ok";
    case PE_ERR_INVALID_ARG: return "invalid argument";
    case PE_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case PE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case PE_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

int pe_decode_splits(const pe_cache_desc* desc) { return check_desc(desc) == PE_OK ? decode_splits(desc) : 0; }

size_t pe_workspace_bytes(int op, const pe_cache_desc* desc, int64_t total_tokens) {
  if (check_desc(desc) != PE_OK) return 0;
  switch (op) {
    case PE_OP_PAGED_DECODE:
      return pe::decode_partials_bytes(desc->num_seqs, desc->num_q_heads, desc->head_dim, decode_splits(desc));
    case PE_OP_APPEND_PAGED_DECODE:
      return pe::decode_partials_bytes(desc->num_seqs, desc->num_q_heads, desc->head_dim, decode_splits(desc));
    case PE_OP_PREFILL_PRUNE:
      if (total_tokens < 0) return 0;
      return pe::prune_workspace_bytes(desc->num_seqs, desc->num_kv_heads, total_tokens,
                                       desc->layout == PE_LAYOUT_SHARED);
    default:
      return 0;
  }
}

namespace {
int score_blocks_impl(const pe_cache_desc* desc, const void* k_pool, const void* v_pool, const int32_t* block_table,
                      const int32_t* seq_lens, float* scores_out, int recent, void* stream, int budget = 0);
}

int pe_score_blocks(const pe_cache_desc* desc, const void* k_pool, const void* v_pool, const int32_t* block_table,
                    const int32_t* seq_lens, float* scores_out, void* workspace, size_t workspace_bytes,
                    void* stream) {
  (void)workspace;
  (void)workspace_bytes;
  return score_blocks_impl(desc, k_pool, v_pool, block_table, seq_lens, scores_out, 0, stream);
}

int pe_score_recent_blocks(const pe_cache_desc* desc, const void* k_pool, const void* v_pool,
                           const int32_t* block_table, const int32_t* seq_lens, int32_t recent,
                           float* scores_inout, void* stream) {
  if (recent < 1) return PE_ERR_INVALID_ARG;
  return score_blocks_impl(desc, k_pool, v_pool, block_table, seq_lens, scores_inout, recent, stream);
}

int pe_score_triggered_blocks(const pe_cache_desc* desc, const void* k_pool, const void* v_pool,
                              const int32_t* block_table, const int32_t* seq_lens, int32_t budget_tokens,
                              float* scores_inout, void* stream) {
  if (desc == nullptr) return PE_ERR_INVALID_ARG;
  if (budget_tokens <= 0 || desc->block_size <= 0 || budget_tokens % desc->block_size != 0) return PE_ERR_INVALID_ARG;
  return score_blocks_impl(desc, k_pool, v_pool, block_table, seq_lens, scores_inout, 0, stream, budget_tokens);
}

namespace {
int score_blocks_impl(const pe_cache_desc* desc, const void* k_pool, const void* v_pool, const int32_t* block_table,
                      const int32_t* seq_lens, float* scores_out, int recent, void* stream, int budget) {
  const int st = check_desc(desc);
  if (st != PE_OK) return st;
  if (!k_pool || !v_pool || !block_table || !seq_lens || !scores_out) return PE_ERR_INVALID_ARG;
  if (!aligned(k_pool, 16) || !aligned(v_pool, 16)) return PE_ERR_INVALID_ARG;
  pe::ScoreArgs a;
  a.k_pool = k_pool;
  a.v_pool = v_pool;
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.scores = scores_out;
  a.num_seqs = desc->num_seqs;
  a.num_kv_heads = desc->num_kv_heads;
  a.head_dim = desc->head_dim;
  a.block_size = desc->block_size;
  a.max_blocks = desc->max_blocks;
  a.is_bf16 = desc->dtype == PE_BF16;
  a.shared = desc->layout == PE_LAYOUT_SHARED;
  a.recent = recent;
  a.budget = budget;
  return pe::launch_score_blocks(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PE_OK : PE_ERR_HIP;
}
}  // namespace

int pe_prefill_prune(const pe_cache_desc* desc, const void* k_in, const void* v_in, const int32_t* cu_seqlens,
                     int64_t total_tokens, int32_t max_seqlen, int32_t budget_tokens, void* k_pool, void* v_pool,
                     const int32_t* block_table, int32_t* seq_lens_out, int32_t* kept_idx_out, void* workspace,
                     size_t workspace_bytes, void* stream) {
  const int st = check_desc(desc);
  if (st != PE_OK) return st;
  if (!cu_seqlens || !k_pool || !v_pool || !block_table || !seq_lens_out) return PE_ERR_INVALID_ARG;
  if (total_tokens < 0 || total_tokens > 0x7fffffffLL || max_seqlen < 0 || max_seqlen > total_tokens)
    return PE_ERR_INVALID_ARG;
  if (total_tokens > 0 && (!k_in || !v_in)) return PE_ERR_INVALID_ARG;
  if (budget_tokens <= 0 || budget_tokens % desc->block_size != 0) return PE_ERR_INVALID_ARG;
  {  // the longest pruned row must fit a table row: the gather indexes block_table[...][pos / B]
    const int64_t keep = max_seqlen < budget_tokens ? max_seqlen : budget_tokens;
    if ((keep + desc->block_size - 1) / desc->block_size > desc->max_blocks) return PE_ERR_INVALID_ARG;
  }
  if (!aligned(k_pool, 16) || !aligned(v_pool, 16) || !aligned(k_in, 16) || !aligned(v_in, 16))
    return PE_ERR_INVALID_ARG;
  const int ws = check_workspace(workspace, workspace_bytes,
                                 pe::prune_workspace_bytes(desc->num_seqs, desc->num_kv_heads, total_tokens,
                                                           desc->layout == PE_LAYOUT_SHARED));
  if (ws != PE_OK) return ws;
  pe::PruneArgs a;
  a.k_in = k_in;
  a.v_in = v_in;
  a.cu_seqlens = cu_seqlens;
  a.k_pool = k_pool;
  a.v_pool = v_pool;
  a.block_table = block_table;
  a.seq_lens_out = seq_lens_out;
  a.kept_idx_out = kept_idx_out;
  a.workspace = workspace;
  a.total_tokens = total_tokens;
  a.max_seqlen = max_seqlen;
  a.budget = budget_tokens;
  a.num_seqs = desc->num_seqs;
  a.num_kv_heads = desc->num_kv_heads;
  a.head_dim = desc->head_dim;
  a.block_size = desc->block_size;
  a.max_blocks = desc->max_blocks;
  a.is_bf16 = desc->dtype == PE_BF16;
  a.shared = desc->layout == PE_LAYOUT_SHARED;
  return pe::launch_prefill_prune(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PE_OK : PE_ERR_HIP;
}

namespace {
int evict_blocks_impl(const pe_cache_desc* desc, const float* scores, float* scores_mut, int32_t* block_table,
                      int32_t* seq_lens, int32_t budget_tokens, int32_t* evicted_logical_out, int32_t* freed_phys_out,
                      void* stream, const pe_evict_opts* opts = nullptr);
}

int pe_evict_blocks_ex(const pe_cache_desc* desc, const pe_evict_opts* opts, float* scores, int32_t* block_table,
                       int32_t* seq_lens, int32_t budget_tokens, int32_t* evicted_logical_out,
                       int32_t* freed_phys_out, void* stream) {
  if (opts == nullptr) return PE_ERR_INVALID_ARG;
  if (opts->policy != PE_POLICY_LOWEST_SCORE && opts->policy != PE_POLICY_OLDEST) return PE_ERR_INVALID_ARG;
  if (opts->protect_first < 0 || opts->protect_last < 0) return PE_ERR_INVALID_ARG;
  if (opts->policy == PE_POLICY_LOWEST_SCORE && scores == nullptr) return PE_ERR_INVALID_ARG;
  if (opts->cached_scores && scores == nullptr) return PE_ERR_INVALID_ARG;
  return evict_blocks_impl(desc, scores, opts->cached_scores ? scores : nullptr, block_table, seq_lens, budget_tokens,
                           evicted_logical_out, freed_phys_out, stream, opts);
}

int pe_score_evict(const pe_cache_desc* desc, const void* k_pool, const void* v_pool, int32_t* block_table,
                   int32_t* seq_lens, int32_t budget_tokens, float* scores_out, int32_t* evicted_logical_out,
                   int32_t* freed_phys_out, void* stream) {
  const int st = check_desc(desc);
  if (st != PE_OK) return st;
  if (!k_pool || !v_pool || !block_table || !seq_lens || !evicted_logical_out || !freed_phys_out)
    return PE_ERR_INVALID_ARG;
  if (!aligned(k_pool, 16) || !aligned(v_pool, 16)) return PE_ERR_INVALID_ARG;
  if (budget_tokens <= 0 || budget_tokens % desc->block_size != 0) return PE_ERR_INVALID_ARG;
  if (desc->layout != PE_LAYOUT_PER_HEAD) return PE_ERR_UNSUPPORTED;  // needs every head's score before the argmin
  pe::ScoreEvictArgs a;
  a.k_pool = k_pool;
  a.v_pool = v_pool;
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.scores_out = scores_out;
  a.evicted_logical = evicted_logical_out;
  a.freed_phys = freed_phys_out;
  a.num_seqs = desc->num_seqs;
  a.num_kv_heads = desc->num_kv_heads;
  a.head_dim = desc->head_dim;
  a.block_size = desc->block_size;
  a.max_blocks = desc->max_blocks;
  a.budget = budget_tokens;
  a.is_bf16 = desc->dtype == PE_BF16;
  return pe::launch_score_evict(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PE_OK : PE_ERR_HIP;
}

int pe_evict_blocks(const pe_cache_desc* desc, const float* scores, int32_t* block_table, int32_t* seq_lens,
                    int32_t budget_tokens, int32_t* evicted_logical_out, int32_t* freed_phys_out, void* stream) {
  return evict_blocks_impl(desc, scores, nullptr, block_table, seq_lens, budget_tokens, evicted_logical_out,
                           freed_phys_out, stream);
}

int pe_evict_blocks_cached(const pe_cache_desc* desc, float* scores_inout, int32_t* block_table, int32_t* seq_lens,
                           int32_t budget_tokens, int32_t* evicted_logical_out, int32_t* freed_phys_out,
                           void* stream) {
  return evict_blocks_impl(desc, scores_inout, scores_inout, block_table, seq_lens, budget_tokens,
                           evicted_logical_out, freed_phys_out, stream);
}

namespace {
int evict_blocks_impl(const pe_cache_desc* desc, const float* scores, float* scores_mut, int32_t* block_table,
                      int32_t* seq_lens, int32_t budget_tokens, int32_t* evicted_logical_out, int32_t* freed_phys_out,
                      void* stream, const pe_evict_opts* opts) {
  const int st = check_desc(desc);
  if (st != PE_OK) return st;
  if ((!scores && !(opts && opts->policy == PE_POLICY_OLDEST)) || !block_table || !seq_lens || !evicted_logical_out || !freed_phys_out) return PE_ERR_INVALID_ARG;
  if (budget_tokens <= 0 || budget_tokens % desc->block_size != 0) return PE_ERR_INVALID_ARG;
  pe::EvictArgs a;
  a.scores = scores;
  a.scores_mut = scores_mut;
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.evicted_logical = evicted_logical_out;
  a.freed_phys = freed_phys_out;
  a.num_seqs = desc->num_seqs;
  a.num_kv_heads = desc->num_kv_heads;
  a.block_size = desc->block_size;
  a.max_blocks = desc->max_blocks;
  a.budget = budget_tokens;
  a.shared = desc->layout == PE_LAYOUT_SHARED;
  if (opts != nullptr) {
    a.policy = opts->policy;
    a.protect_first = opts->protect_first;
    a.protect_last = opts->protect_last;
    a.share_heads = opts->share_heads != 0;
  }
  return pe::launch_evict_blocks(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PE_OK : PE_ERR_HIP;
}
}  // namespace

int pe_paged_decode(const pe_cache_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                    const int32_t* block_table, const int32_t* seq_lens, float softmax_scale, void* out,
                    void* workspace, size_t workspace_bytes, void* stream) {
  const int st = check_desc(desc);
  if (st != PE_OK) return st;
  if (!q || !k_pool || !v_pool || !block_table || !seq_lens || !out) return PE_ERR_INVALID_ARG;
  if (!aligned(k_pool, 16) || !aligned(v_pool, 16) || !aligned(q, 16)) return PE_ERR_INVALID_ARG;
  if (!finite(softmax_scale)) return PE_ERR_INVALID_ARG;
  const int splits = decode_splits(desc);
  const int ws = check_workspace(
      workspace, workspace_bytes,
      pe::decode_partials_bytes(desc->num_seqs, desc->num_q_heads, desc->head_dim, splits));
  if (ws != PE_OK) return ws;
  pe::DecodeArgs a = decode_args(desc, splits);
  a.q = q;
  a.k_pool = k_pool;
  a.v_pool = v_pool;
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.out = out;
  a.partials = static_cast<float*>(workspace);
  a.scale = softmax_scale;
  return pe::launch_paged_decode(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PE_OK : PE_ERR_HIP;
}

namespace {
// Device address of `scratch` on the current device, looked up once per device (every GPU holds its own copy of
// the array at its own address).
int static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return PE_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return PE_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return PE_ERR_HIP;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return PE_OK;
}
}  // namespace

int pe_paged_decode_static(const pe_cache_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                           const int32_t* block_table, const int32_t* seq_lens, float softmax_scale, void* out,
                           void* stream) {
  const int st = check_desc(desc);
  if (st != PE_OK) return st;
  if (!q || !k_pool || !v_pool || !block_table || !seq_lens || !out) return PE_ERR_INVALID_ARG;
  if (!aligned(k_pool, 16) || !aligned(v_pool, 16) || !aligned(q, 16)) return PE_ERR_INVALID_ARG;
  if (!finite(softmax_scale)) return PE_ERR_INVALID_ARG;
  const int splits = decode_splits(desc);
  const size_t need = pe::decode_partials_bytes(desc->num_seqs, desc->num_q_heads, desc->head_dim, splits);
  if (need > (size_t)PE_STATIC_SCRATCH_BYTES) return PE_ERR_WORKSPACE;  // the partials would not fit the array
  void* partials = nullptr;
  if (need > 0) {
    const int sc = static_scratch(&partials);
    if (sc != PE_OK) return sc;
  }
  pe::DecodeArgs a = decode_args(desc, splits);
  a.q = q;
  a.k_pool = k_pool;
  a.v_pool = v_pool;
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.out = out;
  // every (row, split, head) record the merge reads is written by the attention kernel of the same call (empty
  // splits write (acc, m, l) = (0, -inf, 0)), so what an earlier call left in the array never shows
  a.partials = static_cast<float*>(partials);
  a.scale = softmax_scale;
  return pe::launch_paged_decode(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PE_OK : PE_ERR_HIP;
}

int pe_append_paged_decode(const pe_cache_desc* desc, const void* new_k, const void* new_v, const void* q,
                           void* k_pool, void* v_pool, int32_t* block_table, const int32_t* seq_lens,
                           int32_t* seq_lens_out, int32_t* freed_phys, const int32_t* spare, int32_t* spare_used,
                           int32_t n_spare, float softmax_scale, void* out, void* workspace, size_t workspace_bytes,
                           void* stream) {
  const int st = check_desc(desc);
  if (st != PE_OK) return st;
  if (!new_k || !new_v || !q || !k_pool || !v_pool || !block_table || !seq_lens || !seq_lens_out || !freed_phys ||
      !spare || !spare_used || !out)
    return PE_ERR_INVALID_ARG;
  if (seq_lens_out == seq_lens) return PE_ERR_INVALID_ARG;
  if (n_spare < 1) return PE_ERR_INVALID_ARG;
  if (!aligned(k_pool, 16) || !aligned(v_pool, 16) || !aligned(q, 16) || !aligned(new_k, 16) || !aligned(new_v, 16))
    return PE_ERR_INVALID_ARG;
  if (!finite(softmax_scale)) return PE_ERR_INVALID_ARG;
  const int splits = decode_splits(desc);
  const int ws = check_workspace(
      workspace, workspace_bytes,
      pe::decode_partials_bytes(desc->num_seqs, desc->num_q_heads, desc->head_dim, splits));
  if (ws != PE_OK) return ws;
  pe::DecodeArgs a = decode_args(desc, splits);
  a.q = q;
  a.k_pool = k_pool;
  a.v_pool = v_pool;
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.out = out;
  a.partials = static_cast<float*>(workspace);
  a.scale = softmax_scale;
  a.new_k = new_k;
  a.new_v = new_v;
  a.freed_phys = freed_phys;
  a.spare = spare;
  a.spare_used = spare_used;
  a.seq_lens_out = seq_lens_out;
  a.n_spare = n_spare;
  if (desc->layout == PE_LAYOUT_SHARED) {
    // One table row per sequence: the workgroups of a sequence's heads would race on its page bookkeeping
    // inside one launch, so the same effect is produced by two launches (append, then attention over the
    // new lengths).
    pe::AppendArgs ap;
    ap.new_k = new_k;
    ap.new_v = new_v;
    ap.k_pool = k_pool;
    ap.v_pool = v_pool;
    ap.block_table = block_table;
    ap.seq_lens = const_cast<int32_t*>(seq_lens);
    ap.seq_lens_out = seq_lens_out;
    ap.freed_phys = freed_phys;
    ap.spare = spare;
    ap.spare_used = spare_used;
    ap.n_spare = n_spare;
    ap.num_seqs = desc->num_seqs;
    ap.num_kv_heads = desc->num_kv_heads;
    ap.head_dim = desc->head_dim;
    ap.block_size = desc->block_size;
    ap.max_blocks = desc->max_blocks;
    ap.is_bf16 = desc->dtype == PE_BF16;
    ap.shared = true;
    if (pe::launch_append_kv(ap, static_cast<hipStream_t>(stream)) != hipSuccess) return PE_ERR_HIP;
    a.seq_lens = seq_lens_out;
    a.new_k = nullptr;
    a.new_v = nullptr;
  }
  return pe::launch_paged_decode(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PE_OK : PE_ERR_HIP;
}

int pe_append_paged_decode_layers(const pe_cache_desc* desc, int32_t num_layers, const void* new_k, const void* new_v,
                                  const void* q, void* k_pool, void* v_pool, int32_t* block_table,
                                  const int32_t* seq_lens, int32_t* seq_lens_out, int32_t* freed_phys,
                                  const int32_t* spare, int32_t* spare_used, int32_t n_spare, float softmax_scale,
                                  void* out, void* workspace, size_t workspace_bytes, void* stream) {
  const int st = check_desc(desc);
  if (st != PE_OK) return st;
  if (num_layers < 1 || n_spare < 1) return PE_ERR_INVALID_ARG;
  if (!new_k || !new_v || !q || !block_table || !seq_lens || !seq_lens_out || !freed_phys || !spare || !spare_used || !out)
    return PE_ERR_INVALID_ARG;
  const bool shared = desc->layout == PE_LAYOUT_SHARED;
  const size_t elem = desc->dtype == PE_BF16 ? 2 : 4;
  const int64_t S = desc->num_seqs;
  const int64_t rows = shared ? S : S * desc->num_kv_heads;  // table rows, spare lists, freed pages per layer
  const size_t kv_bytes = (size_t)S * desc->num_kv_heads * desc->head_dim * elem;
  const size_t q_bytes = (size_t)S * desc->num_q_heads * desc->head_dim * elem;
  for (int32_t l = 0; l < num_layers; ++l) {
    const int rc = pe_append_paged_decode(
        desc, static_cast<const char*>(new_k) + l * kv_bytes, static_cast<const char*>(new_v) + l * kv_bytes,
        static_cast<const char*>(q) + l * q_bytes, k_pool, v_pool, block_table + l * rows * desc->max_blocks,
        seq_lens + l * S, seq_lens_out + l * S, freed_phys + l * rows, spare + l * rows * n_spare, spare_used + l * rows,
        n_spare, softmax_scale, static_cast<char*>(out) + l * q_bytes, workspace, workspace_bytes, stream);
    if (rc != PE_OK) return rc;
  }
  return PE_OK;
}

int pe_append_kv(const pe_cache_desc* desc, const void* new_k, const void* new_v, void* k_pool, void* v_pool,
                 int32_t* block_table, int32_t* seq_lens, int32_t* freed_phys, const int32_t* spare,
                 int32_t* spare_used, int32_t n_spare, void* stream) {
  const int st = check_desc(desc);
  if (st != PE_OK) return st;
  if (!new_k || !new_v || !k_pool || !v_pool || !block_table || !seq_lens || !freed_phys || !spare || !spare_used)
    return PE_ERR_INVALID_ARG;
  if (n_spare < 1) return PE_ERR_INVALID_ARG;
  if (!aligned(k_pool, 16) || !aligned(v_pool, 16) || !aligned(new_k, 16) || !aligned(new_v, 16))
    return PE_ERR_INVALID_ARG;
  pe::AppendArgs a;
  a.new_k = new_k;
  a.new_v = new_v;
  a.k_pool = k_pool;
  a.v_pool = v_pool;
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.freed_phys = freed_phys;
  a.spare = spare;
  a.spare_used = spare_used;
  a.n_spare = n_spare;
  a.num_seqs = desc->num_seqs;
  a.num_kv_heads = desc->num_kv_heads;
  a.head_dim = desc->head_dim;
  a.block_size = desc->block_size;
  a.max_blocks = desc->max_blocks;
  a.is_bf16 = desc->dtype == PE_BF16;
  a.shared = desc->layout == PE_LAYOUT_SHARED;
  return pe::launch_append_kv(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PE_OK : PE_ERR_HIP;
}

}  // extern "C"
