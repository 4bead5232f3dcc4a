// Host-side launch interfaces between the C-ABI layer (pe_api.hip) and the kernel translation units.
// Arguments are already validated by the caller: shapes are supported, pointers are non-null.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace pe {

struct ScoreArgs {
  const void* k_pool;
  const void* v_pool;
  const int32_t* block_table;
  const int32_t* seq_lens;
  float* scores;
  int num_seqs, num_kv_heads, head_dim, block_size, max_blocks;
  bool is_bf16;
  int recent = 0;  // 0: score every page; n > 0: only the n most recently filled pages of each row
  bool shared = false;  // one table row per sequence, pages [B][Hk][D]
  int budget = 0;       // > 0: score only the sequences that trigger an eviction at this budget
};
hipError_t launch_score_blocks(const ScoreArgs& a, hipStream_t stream);

struct ScoreEvictArgs {
  const void* k_pool;
  const void* v_pool;
  int32_t* block_table;
  int32_t* seq_lens;
  float* scores_out;  // may be null
  int32_t* evicted_logical;
  int32_t* freed_phys;
  int num_seqs, num_kv_heads, head_dim, block_size, max_blocks, budget;
  bool is_bf16;
};
hipError_t launch_score_evict(const ScoreEvictArgs& a, hipStream_t stream);

struct EvictArgs {
  const float* scores;
  float* scores_mut = nullptr;  // when set (== scores): delete the evicted entry from the score row as well
  int32_t* block_table;
  int32_t* seq_lens;
  int32_t* evicted_logical;
  int32_t* freed_phys;
  int num_seqs, num_kv_heads, block_size, max_blocks, budget;
  int policy = 0, protect_first = 0, protect_last = 0, share_heads = 0;
  bool shared = false;  // one table row per sequence (implies share_heads); outputs are [S]
};
hipError_t launch_evict_blocks(const EvictArgs& a, hipStream_t stream);

struct AppendArgs {
  const void* new_k;
  const void* new_v;
  void* k_pool;
  void* v_pool;
  int32_t* block_table;
  int32_t* seq_lens;
  int32_t* freed_phys;
  const int32_t* spare;
  int32_t* spare_used;
  int n_spare, num_seqs, num_kv_heads, head_dim, block_size, max_blocks;
  bool is_bf16;
  bool shared = false;  // one table row, one spare list and one freed page per sequence
  int32_t* seq_lens_out = nullptr;  // when set, the new lengths go here and seq_lens is only read
};
hipError_t launch_append_kv(const AppendArgs& a, hipStream_t stream);

struct DecodeArgs {
  const void* q;
  const void* k_pool;
  const void* v_pool;
  const int32_t* block_table;
  const int32_t* seq_lens;
  void* out;
  float* partials;  // workspace: [rows][splits][G][D + 2] fp32 (unused when splits == 1)
  float scale;
  int num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, max_blocks;
  int splits;
  int xcd_map;
  int waves, depth;  // workgroup size in waves, register pipeline depth
  int loads = 2;     // wave-loads of K (and of V) per tile
  bool is_bf16;
  // fused append: all null / 0 for plain attention
  const void* new_k = nullptr;
  const void* new_v = nullptr;
  int32_t* freed_phys = nullptr;
  const int32_t* spare = nullptr;
  int32_t* spare_used = nullptr;
  int32_t* seq_lens_out = nullptr;
  int n_spare = 0;
  bool shared = false;  // one table row per sequence, pages [B][Hk][D]; plain attention only
};
hipError_t launch_paged_decode(const DecodeArgs& a, hipStream_t stream);
size_t decode_partials_bytes(int num_seqs, int num_q_heads, int head_dim, int splits);

struct PruneArgs {
  const void* k_in;
  const void* v_in;
  const int32_t* cu_seqlens;
  void* k_pool;
  void* v_pool;
  const int32_t* block_table;
  int32_t* seq_lens_out;
  int32_t* kept_idx_out;  // may be null
  void* workspace;
  int64_t total_tokens;
  int max_seqlen, budget;
  int num_seqs, num_kv_heads, head_dim, block_size, max_blocks;
  bool is_bf16;
  bool shared = false;  // one decision per sequence (head-mean token scores), pages [B][Hk][D]
};
hipError_t launch_prefill_prune(const PruneArgs& a, hipStream_t stream);
size_t prune_workspace_bytes(int num_seqs, int num_kv_heads, int64_t total_tokens, bool shared);

}  // namespace pe
