// Decode-time eviction (Alg. 3: "Evict One page with the lowest score", "Update the KV Cache Block
// Table") and the harness append step that follows it in a decode iteration.
//
// With a caller-kept score array (scores are immutable per full page) the evicted entry is deleted from
// the score row too, so that scores stay aligned with the table.
//
// evict: one workgroup per sequence, one wave per (sequence, KV head) row at a time.  The wave finds
// argmin_j (score_j, j) over the row's full pages with a lane-strided scan and a lexicographic
// wave reduction (ties: lowest logical index), then shifts the table entries behind the evicted one
// left by one, 64 entries per pass.  seq_lens[s] is read by every wave before the barrier and
// written once after it.
#include "pe_device.h"
#include "pe_evict_common.h"
#include "pe_launch.h"

namespace pe {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

template <int M>
__device__ __forceinline__ void min_step(float& sc, int& idx) {
  const float osc = lane_xor_f32<M>(sc);
  const int oidx = lane_xor_i32<M>(idx);
  if (osc < sc || (osc == sc && oidx < idx)) {
    sc = osc;
    idx = oidx;
  }
}

__global__ __launch_bounds__(kThreads) void evict_blocks_kernel(const float* scores, float* scores_mut,
                                                                int32_t* __restrict__ block_table,
                                                                int32_t* __restrict__ seq_lens,
                                                                int32_t* __restrict__ evicted_logical,
                                                                int32_t* __restrict__ freed_phys, int num_kv_heads,
                                                                int block_size, int max_blocks, int budget,
                                                                int policy, int protect_first, int protect_last,
                                                                int share_heads, int shared) {
  const int s = (int)blockIdx.x;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int len = seq_lens[s];
  const int n = len / block_size;
  // a length beyond the table row is a caller error: such a sequence is left alone
  const bool trigger = len > 0 && (len % block_size) == 0 && len >= budget && n <= max_blocks;
  // candidate pages lo .. hi-1: protection yields before the budget does (always one candidate)
  const int lo = protect_first < n - 1 ? protect_first : n - 1;
  const int hi = n - protect_last > lo + 1 ? n - protect_last : lo + 1;

  // One decision per sequence: every wave computes the same argmin over head-averaged scores (mean over
  // the KV heads in fp64, head order, one rounding to fp32) BEFORE any wave touches a score row.
  int j_shared = lo;
  if (trigger && policy == 0 && share_heads) {
    // the search starts from (+inf, lo): a NaN never compares lower, so a row whose candidates are all NaN (a
    // precondition violation: K/V must be finite) still ends with an index inside [lo, hi)
    float best = __builtin_inff();
    int best_j = lo;
    for (int j = lo + lane; j < hi; j += kWave) {
      double sum = 0.0;
      for (int g = 0; g < num_kv_heads; ++g) sum += (double)scores[((int64_t)s * num_kv_heads + g) * max_blocks + j];
      const float v = (float)(sum / (double)num_kv_heads);
      if (v < best || (v == best && j < best_j)) {
        best = v;
        best_j = j;
      }
    }
    min_step<1>(best, best_j);
    min_step<2>(best, best_j);
    min_step<4>(best, best_j);
    min_step<8>(best, best_j);
    min_step<16>(best, best_j);
    min_step<32>(best, best_j);
    j_shared = __builtin_amdgcn_readfirstlane(best_j);
  }
  if (share_heads) __syncthreads();

  if (shared) {
    // one table row per sequence: wave 0 moves it (and score row 0), the other waves only their score rows
    for (int h = wave; h < num_kv_heads; h += kWaves) {
      if (!trigger) {
        if (h == 0 && lane == 0) {
          evicted_logical[s] = -1;
          freed_phys[s] = -1;
        }
        continue;
      }
      float* sc_mut = scores_mut != nullptr ? scores_mut + ((int64_t)s * num_kv_heads + h) * max_blocks : nullptr;
      int32_t* bt = h == 0 ? block_table + (int64_t)s * max_blocks : nullptr;
      const int freed = compact_row(bt, sc_mut, j_shared, n, lane);
      if (h == 0 && lane == 0) {
        evicted_logical[s] = j_shared;
        freed_phys[s] = freed;
      }
    }
    __syncthreads();
    if (threadIdx.x == 0 && trigger) seq_lens[s] = len - block_size;
    return;
  }

  for (int h = wave; h < num_kv_heads; h += kWaves) {
    const int64_t row = (int64_t)s * num_kv_heads + h;
    if (!trigger) {
      if (lane == 0) {
        evicted_logical[row] = -1;
        freed_phys[row] = -1;
      }
      continue;
    }
    int32_t* bt = block_table + row * max_blocks;
    int jstar = j_shared;  // policy 1 (oldest unprotected page) and shared decisions are already known
    if (policy == 0 && !share_heads) {
      const float* sc_row = scores + row * max_blocks;
      float best = __builtin_inff();
      int best_j = lo;  // as above: the result stays inside [lo, hi) whatever the scores hold
      for (int j = lo + lane; j < hi; j += kWave) {
        const float v = sc_row[j];
        if (v < best || (v == best && j < best_j)) {
          best = v;
          best_j = j;
        }
      }
      min_step<1>(best, best_j);
      min_step<2>(best, best_j);
      min_step<4>(best, best_j);
      min_step<8>(best, best_j);
      min_step<16>(best, best_j);
      min_step<32>(best, best_j);
      jstar = __builtin_amdgcn_readfirstlane(best_j);
    }
    float* sc_mut = scores_mut != nullptr ? scores_mut + row * max_blocks : nullptr;
    const int freed = compact_row(bt, sc_mut, jstar, n, lane);
    if (lane == 0) {
      evicted_logical[row] = jstar;
      freed_phys[row] = freed;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0 && trigger) seq_lens[s] = len - block_size;
}

// Append: one workgroup per sequence.  Phase 1 links a new page into each row when the tail page is
// full; phase 2 copies the new K/V rows with 16-byte lane accesses.  The new length goes to seq_lens, or to
// seq_lens_out when that is given (seq_lens is then only read).
__global__ __launch_bounds__(kThreads) void append_kv_kernel(const uint4* __restrict__ new_k,
                                                             const uint4* __restrict__ new_v,
                                                             uint4* __restrict__ k_pool, uint4* __restrict__ v_pool,
                                                             int32_t* __restrict__ block_table,
                                                             int32_t* __restrict__ seq_lens,
                                                             int32_t* __restrict__ freed_phys,
                                                             const int32_t* __restrict__ spare,
                                                             int32_t* __restrict__ spare_used, int n_spare,
                                                             int num_kv_heads, int block_size, int max_blocks,
                                                             int VEC_PER_ROW, int32_t* __restrict__ seq_lens_out) {
  const int s = (int)blockIdx.x;
  const int len = seq_lens[s];
  const int slot = len % block_size;
  const int jb = len / block_size;
  if (len < 0 || jb >= max_blocks) return;  // caller precondition violated: leave everything untouched
  if (slot == 0) {
    for (int h = (int)threadIdx.x; h < num_kv_heads; h += kThreads) {
      const int64_t row = (int64_t)s * num_kv_heads + h;
      int32_t page = freed_phys[row];
      if (page >= 0) {
        freed_phys[row] = -1;
      } else {
        const int used = spare_used[row];
        page = used < n_spare ? spare[row * n_spare + used] : -1;
        spare_used[row] = used + 1;
      }
      block_table[row * max_blocks + jb] = page;
    }
  }
  __syncthreads();
  for (int idx = (int)threadIdx.x; idx < num_kv_heads * VEC_PER_ROW; idx += kThreads) {
    const int h = idx / VEC_PER_ROW, u = idx % VEC_PER_ROW;
    const int64_t row = (int64_t)s * num_kv_heads + h;
    const int32_t page = block_table[row * max_blocks + jb];
    if (page < 0) continue;  // spare list exhausted (precondition violated): drop the token
    const int64_t dst = ((int64_t)page * block_size + slot) * VEC_PER_ROW + u;
    k_pool[dst] = new_k[row * VEC_PER_ROW + u];
    v_pool[dst] = new_v[row * VEC_PER_ROW + u];
  }
  __syncthreads();
  if (threadIdx.x == 0) (seq_lens_out != nullptr ? seq_lens_out : seq_lens)[s] = len + 1;
}

}  // namespace

hipError_t launch_evict_blocks(const EvictArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(evict_blocks_kernel, dim3((unsigned)a.num_seqs), dim3(kThreads), 0, stream, a.scores,
                     a.scores_mut, a.block_table, a.seq_lens, a.evicted_logical, a.freed_phys, a.num_kv_heads, a.block_size,
                     a.max_blocks, a.budget, a.policy, a.protect_first, a.protect_last, (a.share_heads || a.shared) ? 1 : 0,
                     a.shared ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_append_kv(const AppendArgs& a, hipStream_t stream) {
  const int vec_per_head_row = a.head_dim * (a.is_bf16 ? 2 : 4) / 16;
  // shared: the sequence is one row of Hk * D elements with one table row, spare list and freed page
  const int rows_per_seq = a.shared ? 1 : a.num_kv_heads;
  const int vec_per_row = a.shared ? vec_per_head_row * a.num_kv_heads : vec_per_head_row;
  hipLaunchKernelGGL(append_kv_kernel, dim3((unsigned)a.num_seqs), dim3(kThreads), 0, stream, (const uint4*)a.new_k,
                     (const uint4*)a.new_v, (uint4*)a.k_pool, (uint4*)a.v_pool, a.block_table, a.seq_lens,
                     a.freed_phys, a.spare, a.spare_used, a.n_spare, rows_per_seq, a.block_size, a.max_blocks,
                     vec_per_row, a.seq_lens_out);
  return hipGetLastError();
}

}  // namespace pe
