// Block importance scores (Alg. 1, block mode; Alg. 3 "Compute Score of Page i"):
//   S_j = (1/B) * sum_{i in page j} ||V_i||_2 / ||K_i||_2
// One wave sweeps one page: every lane loads 16 bytes, consecutive lanes consecutive addresses, so a
// wave-load covers 1 KiB of the page.  Sums of squares are accumulated in fp64, reduced over the
// lanes of a token row, and the page mean is summed in slot order and rounded once to fp32.
//
// A page's score never changes once the page is full (its tokens are immutable), so a caller that
// keeps the score array alive may ask for the most recently filled pages only (`recent` > 0): the
// kernel then visits pages nfull - recent .. nfull - 1 of every row and leaves the other entries alone.
#include "pe_device.h"
#include "pe_evict_common.h"
#include "pe_launch.h"
#include "pe_norms.h"

namespace pe {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kPagesPerWave = 4;
constexpr int kPagesPerGroup = kWaves * kPagesPerWave;

// One page scored by one wave.
template <typename T, int D, int B>
struct PageScore {
  using G = RowGeom<T, D>;
  static constexpr int LPR = G::kLanesPerRow;
  static constexpr int TPL = G::kTokensPerLoad;
  static constexpr int NL = B / TPL;  // wave-loads per page
  static constexpr int NV = 2 * NL;   // per-lane partial sums: (K, V) x NL token rows
  static_assert(NV <= LPR, "reduce-scatter needs at least as many lanes per row as values");
  static constexpr int kVecPerPage = B * D / G::kPerVec;

  static __device__ __forceinline__ void issue(uint4 (&kb)[NL], uint4 (&vb)[NL], const T* k_pool, const T* v_pool,
                                               int phys, int lane) {
    const int64_t base = (int64_t)phys * kVecPerPage + lane;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      kb[i] = load_vec_stream(k_pool, base + i * kWave);
      vb[i] = load_vec_stream(v_pool, base + i * kWave);
    }
  }

  // The page's score (the same value in every lane): fp64 throughout, one rounding to fp32.
  static __device__ __forceinline__ float finish(const uint4 (&kb)[NL], const uint4 (&vb)[NL], int lane) {
    // value index = kv * NL + i  (kv: 0 = K, 1 = V; i = wave-load = token row i*TPL + lane/LPR)
    double part[NV];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      part[i] = sumsq_vec<T>(kb[i], 0.0);
      part[NL + i] = sumsq_vec<T>(vb[i], 0.0);
    }
    const double ratio = token_ratio_from_partials<NL, LPR>(part, lane);
    // page mean, summed in slot order t = 0 .. B-1; token t = i*TPL + g sits on lane g*LPR + 2*bitrev(i)
    double sum = 0.0;
#pragma unroll
    for (int t = 0; t < B; ++t) {
      constexpr int kBits = ilog2(NL);
      const int i = t / TPL, g = t % TPL;
      const int src = g * LPR + 2 * bit_reverse<kBits>(i);
      const int lo = __builtin_amdgcn_readlane(__double2loint(ratio), src);
      const int hi = __builtin_amdgcn_readlane(__double2hiint(ratio), src);
      sum += __hiloint2double(hi, lo);
    }
    return (float)(sum / (double)B);
  }
};

template <typename T, int D, int B>
__global__ __launch_bounds__(kThreads) void score_blocks_kernel(const T* __restrict__ k_pool,
                                                                const T* __restrict__ v_pool,
                                                                const int32_t* __restrict__ block_table,
                                                                const int32_t* __restrict__ seq_lens,
                                                                float* __restrict__ scores, int num_kv_heads,
                                                                int max_blocks, int groups_per_row, int recent) {
  using PS = PageScore<T, D, B>;
  constexpr int NL = PS::NL;

  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int row = (int)(blockIdx.x / groups_per_row);
  const int grp = (int)(blockIdx.x % groups_per_row);
  const int s = row / num_kv_heads;
  const int nfull_raw = seq_lens[s] / B;
  const int nfull = nfull_raw < max_blocks ? nfull_raw : max_blocks;  // never index past the table row
  const int32_t* bt = block_table + (int64_t)row * max_blocks;
  float* out = scores + (int64_t)row * max_blocks;
  // recent == 0: every entry of the row; else only the last `recent` full pages
  const int j_first = recent > 0 ? (nfull > recent ? nfull - recent : 0) : 0;
  const int j_end = recent > 0 ? nfull : max_blocks;
  const int j0 = j_first + grp * kPagesPerGroup + wave;

  uint4 kb[2][NL], vb[2][NL];
  if (j0 < nfull) PS::issue(kb[0], vb[0], k_pool, v_pool, bt[j0], lane);
#pragma unroll
  for (int it = 0; it < kPagesPerWave; ++it) {
    const int j = j0 + it * kWaves;
    if (it + 1 < kPagesPerWave && j + kWaves < nfull)
      PS::issue(kb[(it + 1) & 1], vb[(it + 1) & 1], k_pool, v_pool, bt[j + kWaves], lane);
    if (j >= j_end) break;
    if (j >= nfull) {
      if (lane == 0) out[j] = __builtin_inff();
      continue;
    }
    const float sc = PS::finish(kb[it & 1], vb[it & 1], lane);
    if (lane == 0) out[j] = sc;
  }
}

// Score and evict in one launch (Alg. 3, the whole "L % B == 0" branch): one workgroup per sequence, one wave
// per row at a time.  The wave sweeps the row's pages in logical order with a two-deep register pipeline,
// keeps the running minimum (a strictly lower score replaces it, so ties stay with the lowest index), then
// compacts the table row.  Scores are also written out when the caller wants them.
template <typename T, int D, int B>
__global__ __launch_bounds__(kThreads) void score_evict_kernel(const T* __restrict__ k_pool,
                                                               const T* __restrict__ v_pool,
                                                               int32_t* __restrict__ block_table,
                                                               int32_t* __restrict__ seq_lens,
                                                               float* __restrict__ scores_out,
                                                               int32_t* __restrict__ evicted_logical,
                                                               int32_t* __restrict__ freed_phys, int num_kv_heads,
                                                               int max_blocks, int budget) {
  using PS = PageScore<T, D, B>;
  constexpr int NL = PS::NL;
  const int s = (int)blockIdx.x;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int len = seq_lens[s];
  const int n = len / B;
  const bool trigger = len > 0 && (len % B) == 0 && len >= budget && n <= max_blocks;

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
    float* out = scores_out != nullptr ? scores_out + row * max_blocks : nullptr;
    uint4 kb[2][NL], vb[2][NL];
    float best = 0.f;
    int jstar = 0;
    PS::issue(kb[0], vb[0], k_pool, v_pool, bt[0], lane);
    for (int j = 0; j < n; j += 2) {
      // unconditional issues (the last ones re-read the row's last page) keep the load order known
      PS::issue(kb[1], vb[1], k_pool, v_pool, bt[j + 1 < n ? j + 1 : n - 1], lane);
      const float s0 = PS::finish(kb[0], vb[0], lane);
      if (j == 0 || s0 < best) {
        best = s0;
        jstar = j;
      }
      if (out != nullptr && lane == 0) out[j] = s0;
      PS::issue(kb[0], vb[0], k_pool, v_pool, bt[j + 2 < n ? j + 2 : n - 1], lane);
      if (j + 1 < n) {
        const float s1 = PS::finish(kb[1], vb[1], lane);
        if (s1 < best) {
          best = s1;
          jstar = j + 1;
        }
        if (out != nullptr && lane == 0) out[j + 1] = s1;
      }
    }
    if (out != nullptr)
      for (int j = n + lane; j < max_blocks; j += kWave) out[j] = __builtin_inff();
    __builtin_amdgcn_s_waitcnt(0);  // the trailing re-read of the last page has landed before the row moves
    const int freed = compact_row(bt, nullptr, jstar, n, lane);
    if (lane == 0) {
      evicted_logical[row] = jstar;
      freed_phys[row] = freed;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0 && trigger) seq_lens[s] = len - B;
}

template <typename T, int D, int B>
hipError_t launch(const ScoreArgs& a, hipStream_t stream) {
  const int span = a.recent > 0 ? (a.recent < a.max_blocks ? a.recent : a.max_blocks) : a.max_blocks;
  const int groups_per_row = (span + kPagesPerGroup - 1) / kPagesPerGroup;
  const int64_t rows = (int64_t)a.num_seqs * a.num_kv_heads;
  const int64_t grid = rows * groups_per_row;
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((score_blocks_kernel<T, D, B>), dim3((unsigned)grid), dim3(kThreads), 0, stream,
                     (const T*)a.k_pool, (const T*)a.v_pool, a.block_table, a.seq_lens, a.scores,
                     a.num_kv_heads, a.max_blocks, groups_per_row, a.recent);
  return hipGetLastError();
}

template <typename T, int D, int B>
hipError_t launch_fused(const ScoreEvictArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL((score_evict_kernel<T, D, B>), dim3((unsigned)a.num_seqs), dim3(kThreads), 0, stream,
                     (const T*)a.k_pool, (const T*)a.v_pool, a.block_table, a.seq_lens, a.scores_out,
                     a.evicted_logical, a.freed_phys, a.num_kv_heads, a.max_blocks, a.budget);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score_evict(const ScoreEvictArgs& a, hipStream_t stream) {
#define PE_CASE(TT, DD, BB) \
  if (a.head_dim == DD && a.block_size == BB) return launch_fused<TT, DD, BB>(a, stream)
  if (a.is_bf16) {
    PE_CASE(bf16_t, 64, 16);
    PE_CASE(bf16_t, 64, 32);
    PE_CASE(bf16_t, 128, 16);
    PE_CASE(bf16_t, 128, 32);
  } else {
    PE_CASE(float, 64, 16);
    PE_CASE(float, 64, 32);
    PE_CASE(float, 128, 16);
    PE_CASE(float, 128, 32);
  }
#undef PE_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_score_blocks(const ScoreArgs& a, hipStream_t stream) {
#define PE_CASE(TT, DD, BB) \
  if (a.head_dim == DD && a.block_size == BB) return launch<TT, DD, BB>(a, stream)
  if (a.is_bf16) {
    PE_CASE(bf16_t, 64, 16);
    PE_CASE(bf16_t, 64, 32);
    PE_CASE(bf16_t, 128, 16);
    PE_CASE(bf16_t, 128, 32);
  } else {
    PE_CASE(float, 64, 16);
    PE_CASE(float, 64, 32);
    PE_CASE(float, 128, 16);
    PE_CASE(float, 128, 32);
  }
#undef PE_CASE
  return hipErrorInvalidValue;
}

}  // namespace pe
