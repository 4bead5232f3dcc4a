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

// A chunk of CH token rows (a whole page, or 32 tokens of a larger one) scored by one wave.
template <typename T, int D, int CH>
struct ChunkScore {
  using G = RowGeom<T, D>;
  static constexpr int LPR = G::kLanesPerRow;
  static constexpr int TPL = G::kTokensPerLoad;
  static constexpr int NL = CH / TPL;  // wave-loads per chunk
  static constexpr int NV = 2 * NL;    // per-lane partial sums: (K, V) x NL token rows
  static_assert(NV <= LPR, "reduce-scatter needs at least as many lanes per row as values");
  static constexpr int kVecPerChunk = CH * D / G::kPerVec;

  // vec_base: index (in 16-byte units) of the chunk's first element; lane_vec: this lane's offset inside a
  // wave-load (the lane id when token rows are contiguous); load_stride: distance between wave-loads
  static __device__ __forceinline__ void issue(uint4 (&kb)[NL], uint4 (&vb)[NL], const T* k_pool, const T* v_pool,
                                               int64_t vec_base, int lane_vec, int load_stride = kWave) {
    const int64_t base = vec_base + lane_vec;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      kb[i] = load_vec_stream(k_pool, base + (int64_t)i * load_stride);
      vb[i] = load_vec_stream(v_pool, base + (int64_t)i * load_stride);
    }
  }

  // sum + the chunk's token ratios, added in slot order (the same value in every lane); fp64 throughout.
  static __device__ __forceinline__ double add_ratios(const uint4 (&kb)[NL], const uint4 (&vb)[NL], int lane,
                                                      double sum) {
    // value index = kv * NL + i  (kv: 0 = K, 1 = V; i = wave-load = token row i*TPL + lane/LPR)
    double part[NV];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      part[i] = sumsq_vec<T>(kb[i], 0.0);
      part[NL + i] = sumsq_vec<T>(vb[i], 0.0);
    }
    const double ratio = token_ratio_from_partials<NL, LPR>(part, lane);
    // token t = i*TPL + g sits on lane g*LPR + 2*bitrev(i)
#pragma unroll
    for (int t = 0; t < CH; ++t) {
      constexpr int kBits = ilog2(NL);
      const int i = t / TPL, g = t % TPL;
      const int src = g * LPR + 2 * bit_reverse<kBits>(i);
      const int lo = __builtin_amdgcn_readlane(__double2loint(ratio), src);
      const int hi = __builtin_amdgcn_readlane(__double2hiint(ratio), src);
      sum += __hiloint2double(hi, lo);
    }
    return sum;
  }
};

// Pages of more than 32 tokens are swept as chunks of 32; the page mean is still one sum in slot order.
template <typename T, int D, int B>
struct PageGeom {
  static constexpr int CH = B < 32 ? B : 32;
  static constexpr int NCH = B / CH;
  using CS = ChunkScore<T, D, CH>;
  static constexpr int64_t kVecPerPage = (int64_t)NCH * CS::kVecPerChunk;
  static __device__ __forceinline__ int64_t chunk_base(int phys, int c) {
    return (int64_t)phys * kVecPerPage + (int64_t)c * CS::kVecPerChunk;
  }
};

template <typename T, int D, int B>
__global__ __launch_bounds__(kThreads) void score_blocks_kernel(const T* __restrict__ k_pool,
                                                                const T* __restrict__ v_pool,
                                                                const int32_t* __restrict__ block_table,
                                                                const int32_t* __restrict__ seq_lens,
                                                                float* __restrict__ scores, int num_kv_heads,
                                                                int max_blocks, int groups_per_row, int recent,
                                                                int shared, int budget) {
  using PG = PageGeom<T, D, B>;
  using CS = typename PG::CS;
  constexpr int NL = CS::NL;
  constexpr int NCH = PG::NCH;
  constexpr int kUnits = kPagesPerWave * NCH;  // (page, chunk) units of one wave, in order

  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int row = (int)(blockIdx.x / groups_per_row);
  const int grp = (int)(blockIdx.x % groups_per_row);
  const int s = row / num_kv_heads;
  const int len = seq_lens[s];
  // budget > 0: only sequences that are about to evict (newest page just filled, at budget) are scored
  if (budget > 0 && !(len > 0 && len % B == 0 && len >= budget)) return;
  const int nfull_raw = len / B;
  const int nfull = nfull_raw < max_blocks ? nfull_raw : max_blocks;  // never index past the table row
  // shared: one table row per sequence and pages of [B][Hk][D]: the token rows of this head are Hk rows apart
  constexpr int LPR = CS::LPR;
  const int row_mul = shared ? num_kv_heads : 1;
  const int lane_vec = shared ? ((lane / LPR) * num_kv_heads + row % num_kv_heads) * LPR + lane % LPR : lane;
  const int load_stride = kWave * row_mul;
  const int32_t* bt = block_table + (int64_t)(shared ? s : row) * max_blocks;
  float* out = scores + (int64_t)row * max_blocks;
  // recent == 0: every entry of the row; else only the last `recent` full pages
  const int j_first = recent > 0 ? (nfull > recent ? nfull - recent : 0) : 0;
  const int j_end = recent > 0 ? nfull : max_blocks;
  const int j0 = j_first + grp * kPagesPerGroup + wave;

  uint4 kb[2][NL], vb[2][NL];
  if (j0 < nfull) CS::issue(kb[0], vb[0], k_pool, v_pool, PG::chunk_base(bt[j0], 0) * row_mul, lane_vec, load_stride);
  double sum = 0.0;
#pragma unroll
  for (int u = 0; u < kUnits; ++u) {
    const int j = j0 + (u / NCH) * kWaves;
    if (u + 1 < kUnits) {
      const int jn = j0 + ((u + 1) / NCH) * kWaves;
      if (jn < nfull)
        CS::issue(kb[(u + 1) & 1], vb[(u + 1) & 1], k_pool, v_pool, PG::chunk_base(bt[jn], (u + 1) % NCH) * row_mul,
                  lane_vec, load_stride);
    }
    if (j >= j_end) break;
    if (j >= nfull) {
      if (lane == 0 && u % NCH == 0) out[j] = __builtin_inff();
      continue;
    }
    sum = CS::add_ratios(kb[u & 1], vb[u & 1], lane, sum);
    if (u % NCH == NCH - 1) {
      if (lane == 0) out[j] = (float)(sum / (double)B);  // one rounding to fp32
      sum = 0.0;
    }
  }
}

// Score and evict in one pass over the pages (Alg. 3, the whole "L % B == 0" branch): one workgroup per ROW, so
// the launch fills the chip whether all sequences of a batch evict together or only a few do.  Wave w of the
// workgroup sweeps the row's pages w, w + 4, ... in logical order with a two-deep register pipeline and the same
// per-page arithmetic as the sweep above, and keeps its running minimum (a strictly lower score replaces it, so
// ties stay with the lowest index); the four minima are merged lexicographically by (score, index) and wave 0
// compacts the table row.  Scores are also written out when the caller wants them.  The kernel only READS
// seq_lens: every row of a sequence must see the length from before the eviction, so the lengths are updated by
// score_evict_lens_kernel, launched right behind it.
template <typename T, int D, int B>
__global__ __launch_bounds__(kThreads) void score_evict_kernel(const T* __restrict__ k_pool,
                                                               const T* __restrict__ v_pool,
                                                               int32_t* __restrict__ block_table,
                                                               const int32_t* __restrict__ seq_lens,
                                                               float* __restrict__ scores_out,
                                                               int32_t* __restrict__ evicted_logical,
                                                               int32_t* __restrict__ freed_phys, int num_kv_heads,
                                                               int max_blocks, int budget) {
  using PG = PageGeom<T, D, B>;
  using CS = typename PG::CS;
  constexpr int NL = CS::NL;
  constexpr int NCH = PG::NCH;
  __shared__ float sm_best[kWaves];
  __shared__ int sm_j[kWaves];
  const int64_t row = (int64_t)blockIdx.x;
  const int s = (int)(row / num_kv_heads);
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int len = seq_lens[s];
  const int n = len / B;
  const bool trigger = len > 0 && (len % B) == 0 && len >= budget && n <= max_blocks;
  if (!trigger) {  // workgroup-uniform
    if (threadIdx.x == 0) {
      evicted_logical[row] = -1;
      freed_phys[row] = -1;
    }
    return;
  }
  int32_t* bt = block_table + row * max_blocks;
  float* out = scores_out != nullptr ? scores_out + row * max_blocks : nullptr;
  uint4 kb[2][NL], vb[2][NL];
  float best = __builtin_inff();
  int jstar = 0x7fffffff;  // this wave has seen no page yet
  double sum = 0.0;
  // this wave's (page, chunk) units in logical order: unit u = page wave + (u / NCH) * kWaves, chunk u % NCH
  const int pages_mine = wave < n ? (n - wave + kWaves - 1) / kWaves : 0;
  const int units = pages_mine * NCH;
  const auto page_of = [&](int u) { return wave + (u / NCH) * kWaves; };
  // a page is complete after its last chunk: round once, compare, report
  auto page_done = [&](int u) {
    if (u % NCH != NCH - 1) return;
    const int j = page_of(u);
    const float sc = (float)(sum / (double)B);
    sum = 0.0;
    if (jstar == 0x7fffffff || sc < best) {
      best = sc;
      jstar = j;
    }
    if (out != nullptr && lane == 0) out[j] = sc;
  };
  // unconditional issues (those past the end re-read the wave's last unit) keep the load order known
  auto issue_unit = [&](int buf, int u) {
    const int uc = u < units ? u : units - 1;
    if (buf == 0)
      CS::issue(kb[0], vb[0], k_pool, v_pool, PG::chunk_base(bt[page_of(uc)], uc % NCH), lane);
    else
      CS::issue(kb[1], vb[1], k_pool, v_pool, PG::chunk_base(bt[page_of(uc)], uc % NCH), lane);
  };
  if (units > 0) {
    issue_unit(0, 0);
    for (int u = 0; u < units; u += 2) {
      issue_unit(1, u + 1);
      sum = CS::add_ratios(kb[0], vb[0], lane, sum);
      page_done(u);
      issue_unit(0, u + 2);
      if (u + 1 < units) {
        sum = CS::add_ratios(kb[1], vb[1], lane, sum);
        page_done(u + 1);
      }
    }
  }
  if (out != nullptr)
    for (int j = n + (int)threadIdx.x; j < max_blocks; j += kThreads) out[j] = __builtin_inff();
  __builtin_amdgcn_s_waitcnt(0);  // this wave's trailing re-reads (pages and table entries) have landed
  if (lane == 0) {
    sm_best[wave] = best;
    sm_j[wave] = jstar;
  }
  __syncthreads();  // every wave is done with the table row before wave 0 moves it
  if (wave == 0) {
    float bsc = sm_best[0];
    int bj = sm_j[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
      const float osc = sm_best[w];
      const int oj = sm_j[w];
      // a wave that saw no page carries index 0x7fffffff and never wins; a NaN score never compares lower
      if (oj != 0x7fffffff && (bj == 0x7fffffff || osc < bsc || (osc == bsc && oj < bj))) {
        bsc = osc;
        bj = oj;
      }
    }
    if (bj == 0x7fffffff || bj >= n) bj = 0;  // n >= 1 here, so wave 0 always holds page 0: defensive only
    const int freed = compact_row(bt, nullptr, bj, n, lane);
    if (lane == 0) {
      evicted_logical[row] = bj;
      freed_phys[row] = freed;
    }
  }
}

// The length update of pe_score_evict: one thread per sequence, the same trigger predicate on the old length.
__global__ __launch_bounds__(kThreads) void score_evict_lens_kernel(int32_t* __restrict__ seq_lens, int num_seqs,
                                                                    int block_size, int max_blocks, int budget) {
  const int s = (int)(blockIdx.x * kThreads + threadIdx.x);
  if (s >= num_seqs) return;
  const int len = seq_lens[s];
  const int n = len / block_size;
  if (len > 0 && (len % block_size) == 0 && len >= budget && n <= max_blocks) seq_lens[s] = len - block_size;
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
                     a.num_kv_heads, a.max_blocks, groups_per_row, a.recent, a.shared ? 1 : 0, a.budget);
  return hipGetLastError();
}

template <typename T, int D, int B>
hipError_t launch_fused(const ScoreEvictArgs& a, hipStream_t stream) {
  const int64_t rows = (int64_t)a.num_seqs * a.num_kv_heads;
  if (rows <= 0 || rows > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((score_evict_kernel<T, D, B>), dim3((unsigned)rows), dim3(kThreads), 0, stream,
                     (const T*)a.k_pool, (const T*)a.v_pool, a.block_table, a.seq_lens, a.scores_out,
                     a.evicted_logical, a.freed_phys, a.num_kv_heads, a.max_blocks, a.budget);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(score_evict_lens_kernel, dim3((unsigned)((a.num_seqs + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                     stream, a.seq_lens, a.num_seqs, a.block_size, a.max_blocks, a.budget);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score_evict(const ScoreEvictArgs& a, hipStream_t stream) {
#define PE_CASE(TT, DD, BB) \
  if (a.head_dim == DD && a.block_size == BB) return launch_fused<TT, DD, BB>(a, stream)
#define PE_CASES(TT, DD) \
  PE_CASE(TT, DD, 16);   \
  PE_CASE(TT, DD, 32);   \
  PE_CASE(TT, DD, 64);   \
  PE_CASE(TT, DD, 128)
  if (a.is_bf16) {
    PE_CASES(bf16_t, 64);
    PE_CASES(bf16_t, 128);
  } else {
    PE_CASES(float, 64);
    PE_CASES(float, 128);
  }
#undef PE_CASES
#undef PE_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_score_blocks(const ScoreArgs& a, hipStream_t stream) {
#define PE_CASE(TT, DD, BB) \
  if (a.head_dim == DD && a.block_size == BB) return launch<TT, DD, BB>(a, stream)
#define PE_CASES(TT, DD) \
  PE_CASE(TT, DD, 16);   \
  PE_CASE(TT, DD, 32);   \
  PE_CASE(TT, DD, 64);   \
  PE_CASE(TT, DD, 128)
  if (a.is_bf16) {
    PE_CASES(bf16_t, 64);
    PE_CASES(bf16_t, 128);
  } else {
    PE_CASES(float, 64);
    PE_CASES(float, 128);
  }
#undef PE_CASES
#undef PE_CASE
  return hipErrorInvalidValue;
}

}  // namespace pe
