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
#include "pe_launch.h"
#include "pe_norms.h"

namespace pe {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kPagesPerWave = 4;
constexpr int kPagesPerGroup = kWaves * kPagesPerWave;

template <typename T, int D, int B>
__global__ __launch_bounds__(kThreads) void score_blocks_kernel(const T* __restrict__ k_pool,
                                                                const T* __restrict__ v_pool,
                                                                const int32_t* __restrict__ block_table,
                                                                const int32_t* __restrict__ seq_lens,
                                                                float* __restrict__ scores, int num_kv_heads,
                                                                int max_blocks, int groups_per_row, int recent) {
  using G = RowGeom<T, D>;
  constexpr int LPR = G::kLanesPerRow;
  constexpr int TPL = G::kTokensPerLoad;
  constexpr int NL = B / TPL;  // wave-loads per page
  constexpr int NV = 2 * NL;   // per-lane partial sums: (K, V) x NL token rows
  static_assert(NV <= LPR, "reduce-scatter needs at least as many lanes per row as values");
  constexpr int kVecPerPage = B * D / G::kPerVec;

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
  auto issue = [&](int buf, int j) {
    if (j < nfull) {
      const int64_t base = (int64_t)bt[j] * kVecPerPage + lane;
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        kb[buf][i] = load_vec_stream(k_pool, base + i * kWave);
        vb[buf][i] = load_vec_stream(v_pool, base + i * kWave);
      }
    }
  };

  issue(0, j0);
#pragma unroll
  for (int it = 0; it < kPagesPerWave; ++it) {
    const int j = j0 + it * kWaves;
    if (it + 1 < kPagesPerWave) issue((it + 1) & 1, j + kWaves);
    if (j >= j_end) break;
    if (j >= nfull) {
      if (lane == 0) out[j] = __builtin_inff();
      continue;
    }
    const int buf = it & 1;
    // value index = kv * NL + i  (kv: 0 = K, 1 = V; i = wave-load = token row i*TPL + lane/LPR)
    double part[NV];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      part[i] = sumsq_vec<T>(kb[buf][i], 0.0);
      part[NL + i] = sumsq_vec<T>(vb[buf][i], 0.0);
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
    if (lane == 0) out[j] = (float)(sum / (double)B);
  }
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

}  // namespace

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
