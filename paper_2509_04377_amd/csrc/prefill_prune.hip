// Prefill token pruning (Alg. 2, the steps after the prompt's attention): score every prompt token,
// evict the E = max(0, L - C) tokens that come first under (score ascending, index ascending), and
// write the survivors, order kept, into the row's pages.
//
// Three kernels on one stream:
//   1. token_scores:  sweep of the packed K/V prompt; S_i = ||V_i||/||K_i|| in fp64, rounded once to
//                     fp32, stored per KV head as a contiguous run  scores[hk][token].
//   2. select:        per row, radix select (digits of 12, 10 and 10 bits, most significant first) on the
//                     fp32 bit patterns (scores are >= +0, so they order like unsigned integers) for the
//                     E-th smallest score T and the number q of tokens equal to T that must go; then, per
//                     chunk of 1024 tokens of the row, how many scores are > T and how many == T.
//   3. gather:        per row and chunk, an index-ordered scan turns those counts into the destination
//                     of every kept token; token rows are then copied with 16-byte lane accesses.
// A token is kept iff score > T, or score == T and at least q equal-score tokens precede it.
//
// Head-shared mode (one decision per sequence, pages [B][Hk][D]): after kernel 1 the per-head scores are
// averaged over the heads (head order, fp64, one rounding) into one more score row, and kernels 2-3 run on
// that row with the whole (token, all heads) record as the unit that is copied.
#include "pe_device.h"
#include "pe_launch.h"
#include "pe_norms.h"

namespace pe {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kChunk = 1024;  // tokens per chunk in the count pass and in the gather (4 per gather thread)
constexpr int kTokPerThread = kChunk / kThreads;
constexpr int kSweepLoads = 4;  // token sweep: wave-loads of K (and of V) per step
constexpr int kSweepIters = 2;  // and steps per wave (4 and 8: the same on 2 GB of prompt, 5 us slower on 1 GB: longer tail)

__host__ __device__ inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {
  float* scores;  // [Hk][total_tokens]; shared mode: one more row, the mean over heads
  uint32_t* sel;  // [rows][2]: threshold bits T, tie quota q
  int32_t* cnt;   // [Hk][chunk_slots][2]: (#score > T, #score == T) per chunk
  int64_t chunk_slots;
};

__host__ inline int64_t chunk_slots_for(int64_t total_tokens, int num_seqs) {
  return total_tokens / kChunk + num_seqs + 1;
}

__host__ inline Workspace carve(void* base, int num_seqs, int num_kv_heads, int64_t total_tokens, bool shared) {
  Workspace w;
  char* p = static_cast<char*>(base);
  w.scores = reinterpret_cast<float*>(p);
  p += align256(sizeof(float) * (size_t)(num_kv_heads + (shared ? 1 : 0)) * (size_t)total_tokens);
  w.sel = reinterpret_cast<uint32_t*>(p);
  p += align256(sizeof(uint32_t) * 2 * (size_t)num_seqs * num_kv_heads);
  w.cnt = reinterpret_cast<int32_t*>(p);
  w.chunk_slots = chunk_slots_for(total_tokens, num_seqs);
  return w;
}

// Chunk slot of (sequence s, local chunk c): sequences never overlap because
// floor((a+b)/n) + 1 >= floor(a/n) + ceil(b/n).
__device__ __forceinline__ int64_t chunk_slot(int cu_s, int s, int c) { return (int64_t)(cu_s / kChunk) + s + c; }

// ---- 1. token scores -------------------------------------------------------------------------------
// The packed prompt is a flat array of (token, head) rows of D elements.  A wave-load covers TPL rows;
// a wave handles kIters groups of NL wave-loads for K and for V, software-pipelined.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void token_scores_kernel(const T* __restrict__ k_in,
                                                                const T* __restrict__ v_in,
                                                                float* __restrict__ scores, int64_t total_rows,
                                                                int64_t total_tokens, int num_kv_heads) {
  using G = RowGeom<T, D>;
  constexpr int LPR = G::kLanesPerRow;
  constexpr int TPL = G::kTokensPerLoad;
  constexpr int NL = kSweepLoads;
  constexpr int kRowsPerStep = NL * TPL;
  constexpr int kIters = kSweepIters;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int grp = lane / LPR;
  constexpr int kRowsPerWave = kIters * kRowsPerStep;
  constexpr int kRowsPerGroup = kWaves * kRowsPerWave;
  __shared__ float sm_score[kRowsPerGroup];  // the workgroup's scores in row order, stored head by head at the end
  const int64_t group_row0 = (int64_t)blockIdx.x * kRowsPerGroup;
  const int64_t row0 = group_row0 + (int64_t)wave * kRowsPerWave;

  uint4 kb[2][NL], vb[2][NL];
  // loads are unconditional: a row past the end is read from the last row instead (its result is never
  // stored), so the compiler keeps the order of outstanding loads and the next group stays in flight
  const int64_t last_row = total_rows - 1;
  const int u = lane % LPR;
  auto issue = [&](int buf, int64_t base_row) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int64_t r = base_row + i * TPL + grp;
      const int64_t vec = (r < last_row ? r : last_row) * LPR + u;
      kb[buf][i] = load_vec_stream(k_in, vec);
      vb[buf][i] = load_vec_stream(v_in, vec);
    }
  };
  issue(0, row0);
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int64_t base_row = row0 + (int64_t)it * kRowsPerStep;
    if (it + 1 < kIters) issue((it + 1) & 1, base_row + kRowsPerStep);
    if (base_row >= total_rows) break;
    const int buf = it & 1;
    double part[2 * NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      part[i] = sumsq_vec<T>(kb[buf][i], 0.0);
      part[NL + i] = sumsq_vec<T>(vb[buf][i], 0.0);
    }
    const double ratio = token_ratio_from_partials<NL, LPR>(part, lane);
    // the lane at position 2*k of its row group (k < NL) stores the row of wave-load bit_reverse(k)
    const int uu = u;
    if ((uu & 1) == 0 && uu < 2 * NL) {
      const int i = bit_reverse<ilog2(NL)>(uu >> 1);
      const int64_t r = base_row + i * TPL + grp;
      if (r < total_rows) sm_score[(int)(r - group_row0)] = (float)ratio;
    }
  }
  // The group's rows are (token, head) pairs in token-major order; the score array is head-major.  Written
  // head by head, the tokens of one head are consecutive floats (a full 128-byte line for 32 tokens).
  __syncthreads();
  const int64_t group_end = group_row0 + kRowsPerGroup < total_rows ? group_row0 + kRowsPerGroup : total_rows;
  if (group_row0 >= group_end) return;
  const int64_t tok_lo = group_row0 / num_kv_heads;
  const int ntok = (int)((group_end - 1) / num_kv_heads - tok_lo) + 1;
  for (int p = (int)threadIdx.x; p < ntok * num_kv_heads; p += kThreads) {
    const int h = p / ntok;
    const int64_t tok = tok_lo + (p - h * ntok);
    const int64_t r = tok * num_kv_heads + h;
    // non-temporal: the scores are written once and read by another kernel (measured 330 us against 344 us per
    // 2.1 GB swept with plain stores; with no stores at all the sweep takes 316 us)
    if (r >= group_row0 && r < group_end)
      __builtin_nontemporal_store(sm_score[(int)(r - group_row0)], &scores[(int64_t)h * total_tokens + tok]);
  }
}

// ---- 1b. head-shared mode: mean over heads of the fp32 token scores -----------------------------------
__global__ __launch_bounds__(kThreads) void head_mean_kernel(const float* __restrict__ scores,
                                                             float* __restrict__ mean_out, int64_t total_tokens,
                                                             int num_kv_heads) {
  const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (t >= total_tokens) return;
  double sum = 0.0;
  for (int h = 0; h < num_kv_heads; ++h) sum += (double)scores[(int64_t)h * total_tokens + t];
  mean_out[t] = (float)(sum / (double)num_kv_heads);
}

// ---- 2. per-row radix select + per-chunk counts ------------------------------------------------------
// One workgroup of 1024 threads per row.  Radix select on the row's fp32 bit patterns, most significant digit
// first: 12 bits (sign, exponent, top three mantissa bits: scores of one row cluster in a few exponents, and a
// narrower first digit would pile every LDS atomic onto three or four bins), then 10 + 10 bits.  After a pass
// the digit that holds rank k is found with a workgroup-wide scan.  The first pass reads the whole row with
// 16-byte loads, eight in flight per thread.  The tokens that fall into the first digit's bin are then
// collected in LDS (a few percent of the row for any spread-out score distribution), so the second and third
// pass never touch memory; a row with more candidates than the LDS buffer holds (e.g. all scores equal) falls
// back to passes over memory.  With the threshold known the same workgroup counts, per chunk of 1024 tokens,
// how many scores are > T and how many == T (one wave per chunk): the gather turns these into destinations.
// A row is worked on by one compute unit, and one compute unit pulls about 45 GB/s from L2 however many loads
// it keeps in flight: that, not the histogram atomics, bounds a pass over a long row (a finer first digit of
// 16384 bins was measured and changed nothing).  Spreading a row over several workgroups needs a launch per
// stage (pivots, counting pass, exact selection, chunk counts), which costs most of what it saves at these
// row lengths.
constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSelBins = 4096;
constexpr int kSelUnroll = 8;
constexpr int kSelCand = 8192;  // candidates kept in LDS after the first pass (32 KiB)

// f(bits) for every element of bits[0 .. L): a scalar head up to 16-byte alignment, 16-byte loads with
// kSelUnroll in flight per thread, a scalar tail.  The order of visits is unspecified.
template <typename F>
__device__ __forceinline__ void visit_row(const uint32_t* bits, int L, int tid, F f) {
  int mis = (int)((4u - (uint32_t)((reinterpret_cast<uintptr_t>(bits) >> 2) & 3u)) & 3u);
  mis = mis < L ? mis : L;
  if (tid < mis) f(bits[tid]);
  const uint4* v = reinterpret_cast<const uint4*>(bits + mis);
  const int nvec = (L - mis) >> 2;
  for (int base = tid; base < nvec; base += kSelUnroll * kSelThreads) {
    uint4 r[kSelUnroll];
#pragma unroll
    for (int j = 0; j < kSelUnroll; ++j) {
      const int i = base + j * kSelThreads;
      r[j] = v[i < nvec ? i : nvec - 1];
    }
#pragma unroll
    for (int j = 0; j < kSelUnroll; ++j) {
      if (base + j * kSelThreads < nvec) {
        f(r[j].x);
        f(r[j].y);
        f(r[j].z);
        f(r[j].w);
      }
    }
  }
  const int tail0 = mis + nvec * 4;
  if (tail0 + tid < L) f(bits[tail0 + tid]);
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ scores,
                                                             const int32_t* __restrict__ cu_seqlens,
                                                             uint32_t* __restrict__ sel, int32_t* __restrict__ cnt,
                                                             int32_t* __restrict__ seq_lens_out,
                                                             int32_t* __restrict__ kept_idx_out, int64_t total_tokens,
                                                             int64_t chunk_slots, int num_kv_heads, int budget) {
  __shared__ uint32_t hist[kSelBins];
  __shared__ uint32_t cand[kSelCand];
  __shared__ uint32_t wave_tot[kSelWaves];
  __shared__ uint32_t sh_prefix, sh_k, sh_ncand;
  const int row = (int)blockIdx.x;
  const int s = row / num_kv_heads, h = row % num_kv_heads;
  const int t0 = cu_seqlens[s];
  const int L = cu_seqlens[s + 1] - t0;
  const int keep = L < budget ? L : budget;
  const int E = L - keep;
  const uint32_t* bits = reinterpret_cast<const uint32_t*>(scores) + (int64_t)h * total_tokens + t0;
  const int tid = (int)threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;

  if (h == 0 && tid == 0) seq_lens_out[s] = keep;
  if (kept_idx_out != nullptr)
    for (int i = keep + tid; i < budget; i += kSelThreads) kept_idx_out[(int64_t)row * budget + i] = -1;

  // E == 0, nothing to evict: T = +0.0, q = 0 keeps every token (scores are >= +0)
  uint32_t prefix = 0u, mask = 0u;
  uint32_t k = (uint32_t)(E > 0 ? E - 1 : 0);  // 0-based rank of the threshold element among the remaining ones
  bool in_lds = false;                         // the remaining candidates are cand[0 .. ncand)
  uint32_t ncand = 0u;
  if (E > 0) {
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
      const int shift = pass == 0 ? 20 : pass == 1 ? 10 : 0;
      const int nbins = pass == 0 ? kSelBins : 1024;
      constexpr int kMaxPerThread = kSelBins / kSelThreads;
      const int per_thread = nbins / kSelThreads;  // 4 or 1 consecutive bins per thread
      for (int i = tid; i < nbins; i += kSelThreads) hist[i] = 0u;
      __syncthreads();
      const uint32_t bmask = (uint32_t)(nbins - 1);
      if (in_lds) {
        for (uint32_t i = (uint32_t)tid; i < ncand; i += kSelThreads) {
          const uint32_t b = cand[i];
          if ((b & mask) == prefix) atomicAdd(&hist[(b >> shift) & bmask], 1u);
        }
      } else {
        visit_row(bits, L, tid, [&](uint32_t b) {
          if ((b & mask) == prefix) atomicAdd(&hist[(b >> shift) & bmask], 1u);
        });
      }
      __syncthreads();
      // workgroup-wide exclusive scan of the per-thread bin totals, in bin order
      uint32_t c[kMaxPerThread], tot = 0u;
#pragma unroll
      for (int j = 0; j < kMaxPerThread; ++j) {
        const int bin = tid * per_thread + j;
        c[j] = (j < per_thread && bin < nbins) ? hist[bin] : 0u;
        tot += c[j];
      }
      uint32_t incl = tot;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)incl, off, kWave);
        if (lane >= off) incl += o;
      }
      if (lane == kWave - 1) wave_tot[wave] = incl;
      __syncthreads();
      uint32_t before = incl - tot;
      for (int w = 0; w < wave; ++w) before += wave_tot[w];
      if (k >= before && k < before + tot) {  // exactly one thread: rank k falls into one of its bins
#pragma unroll
        for (int j = 0; j < kMaxPerThread; ++j) {
          if (k >= before && k < before + c[j]) {
            sh_prefix = prefix | ((uint32_t)(tid * per_thread + j) << shift);
            sh_k = k - before;
            sh_ncand = c[j];
          }
          before += c[j];
        }
      }
      __syncthreads();
      prefix = sh_prefix;
      k = sh_k;
      const uint32_t in_bin = sh_ncand;
      mask |= bmask << shift;
      __syncthreads();
      if (pass == 0 && in_bin <= (uint32_t)kSelCand) {
        // collect the tokens of the chosen bin in LDS (their order does not matter: only values are counted)
        if (tid == 0) sh_ncand = 0u;
        __syncthreads();
        visit_row(bits, L, tid, [&](uint32_t b) {
          if ((b & mask) == prefix) cand[atomicAdd(&sh_ncand, 1u)] = b;
        });
        __syncthreads();
        ncand = sh_ncand;  // == in_bin
        in_lds = true;
        __syncthreads();
      }
    }
  }
  const uint32_t T = prefix;                         // threshold score (bit pattern)
  if (tid == 0) {
    sel[2 * row] = T;
    sel[2 * row + 1] = E > 0 ? k + 1 : 0u;           // q: the first q tokens (index order) with score == T go
  }

  // per-chunk counts, one wave per chunk: 16 tokens per lane, all loads issued before the first compare
  const int nchunks = (L + kChunk - 1) / kChunk;
  int32_t* crow = cnt + ((int64_t)h * chunk_slots + chunk_slot(t0, s, 0)) * 2;
  for (int c = wave; c < nchunks; c += kSelWaves) {
    constexpr int kPerLane = kChunk / kWave;
    uint32_t b[kPerLane];
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) {
      const int i = c * kChunk + j * kWave + lane;
      b[j] = bits[i < L ? i : L - 1];
    }
    int gt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) {
      const bool in = c * kChunk + j * kWave + lane < L;
      gt += __popcll(__builtin_amdgcn_ballot_w64(in && b[j] > T));
      eq += __popcll(__builtin_amdgcn_ballot_w64(in && b[j] == T));
    }
    if (lane == 0) {
      crow[2 * c] = gt;
      crow[2 * c + 1] = eq;
    }
  }
}

__device__ __forceinline__ int block_sum(int v, int* sh /* [kWaves] */) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  const int wave = (int)(threadIdx.x / kWave);
  __syncthreads();
  if (lane_id() == 0) sh[wave] = v;
  __syncthreads();
  int t = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) t += sh[w];
  return t;
}

// ---- 3. gather ----------------------------------------------------------------------------------------
// VPR_T > 0: vectors per token row known at compile time; 0: taken from vpr_rt (head-shared mode, where a
// row is the K (or V) of all heads of a token).
template <int VPR_T>
__global__ __launch_bounds__(kThreads) void gather_kernel(const uint4* __restrict__ k_in, const uint4* __restrict__ v_in,
                                                          const float* __restrict__ scores,
                                                          const int32_t* __restrict__ cu_seqlens,
                                                          const uint32_t* __restrict__ sel,
                                                          const int32_t* __restrict__ cnt,
                                                          const int32_t* __restrict__ block_table,
                                                          uint4* __restrict__ k_pool, uint4* __restrict__ v_pool,
                                                          int32_t* __restrict__ kept_idx_out, int64_t total_tokens,
                                                          int64_t chunk_slots, int num_kv_heads, int chunks_per_row,
                                                          int block_size, int max_blocks, int budget, int vpr_rt) {
  __shared__ int sh[kWaves];
  __shared__ int wave_off[kWaves][2];
  __shared__ int32_t src_tok[kChunk];  // kept tokens of this chunk: in-sequence index
  __shared__ int32_t dst_pos[kChunk];  // and their position in the pruned row
  __shared__ int n_kept_sh;
  const int row = (int)(blockIdx.x / chunks_per_row);
  const int chunk = (int)(blockIdx.x % chunks_per_row);
  const int s = row / num_kv_heads, h = row % num_kv_heads;
  const int t0 = cu_seqlens[s];
  const int L = cu_seqlens[s + 1] - t0;
  if (chunk * kChunk >= L) return;
  const int tid = (int)threadIdx.x;
  const int lane = lane_id();
  const int wave = tid / kWave;
  const uint32_t T = sel[2 * row];
  const int q = (int)sel[2 * row + 1];

  // counts of all earlier chunks of this row
  int gt_before = 0, eq_before = 0;
  {
    const int32_t* c = cnt + ((int64_t)h * chunk_slots + chunk_slot(t0, s, 0)) * 2;
    for (int cc = tid; cc < chunk; cc += kThreads) {
      gt_before += c[2 * cc];
      eq_before += c[2 * cc + 1];
    }
    gt_before = block_sum(gt_before, sh);
    eq_before = block_sum(eq_before, sh);
  }

  // this thread's kTokPerThread consecutive tokens
  const uint32_t* bits = reinterpret_cast<const uint32_t*>(scores) + (int64_t)h * total_tokens + t0;
  const int i0 = chunk * kChunk + tid * kTokPerThread;
  uint32_t b[kTokPerThread];
  int n_gt = 0, n_eq = 0;
#pragma unroll
  for (int j = 0; j < kTokPerThread; ++j) {
    b[j] = (i0 + j < L) ? bits[i0 + j] : 0u;
    const bool in = i0 + j < L;
    n_gt += in && b[j] > T;
    n_eq += in && b[j] == T;
  }
  // exclusive scan of (n_gt, n_eq) over the 256 threads, in thread (= index) order
  int inc_gt = n_gt, inc_eq = n_eq;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int a = __shfl_up(inc_gt, off, kWave);
    const int c2 = __shfl_up(inc_eq, off, kWave);
    if (lane >= off) {
      inc_gt += a;
      inc_eq += c2;
    }
  }
  if (lane == kWave - 1) {
    wave_off[wave][0] = inc_gt;
    wave_off[wave][1] = inc_eq;
  }
  __syncthreads();
  int ex_gt = inc_gt - n_gt + gt_before, ex_eq = inc_eq - n_eq + eq_before;
  for (int w = 0; w < wave; ++w) {
    ex_gt += wave_off[w][0];
    ex_eq += wave_off[w][1];
  }
  // kept tokens before this chunk's start (needed to make dst relative positions dense in LDS)
  const int kept_before_chunk = gt_before + (eq_before > q ? eq_before - q : 0);
#pragma unroll
  for (int j = 0; j < kTokPerThread; ++j) {
    const bool in = i0 + j < L;
    const bool is_gt = in && b[j] > T;
    const bool is_eq = in && b[j] == T;
    const bool kept = is_gt || (is_eq && ex_eq >= q);
    if (kept) {
      const int pos = ex_gt + (ex_eq > q ? ex_eq - q : 0);  // kept tokens before this one in the row
      const int slot = pos - kept_before_chunk;
      src_tok[slot] = i0 + j;
      dst_pos[slot] = pos;
    }
    ex_gt += is_gt;
    ex_eq += is_eq;
  }
  if (tid == kThreads - 1) n_kept_sh = ex_gt + (ex_eq > q ? ex_eq - q : 0) - kept_before_chunk;
  __syncthreads();
  const int n_kept = n_kept_sh;

  // copy the kept rows: VEC_PER_ROW lanes per token row, K and V
  const int32_t* bt = block_table + (int64_t)row * max_blocks;
  if constexpr (VPR_T > 0) {
    constexpr int VEC_PER_ROW = VPR_T;
    constexpr int kRowsPerPass = kThreads / VEC_PER_ROW;
    const int u = tid % VEC_PER_ROW, r = tid / VEC_PER_ROW;
    for (int base = 0; base < n_kept; base += kRowsPerPass) {
      const int e = base + r;
      if (e < n_kept) {
        const int tok = src_tok[e], pos = dst_pos[e];
        const int64_t src = ((int64_t)(t0 + tok) * num_kv_heads + h) * VEC_PER_ROW + u;
        const int64_t dst = ((int64_t)bt[pos / block_size] * block_size + pos % block_size) * VEC_PER_ROW + u;
        k_pool[dst] = k_in[src];
        v_pool[dst] = v_in[src];
        if (kept_idx_out != nullptr && u == 0) kept_idx_out[(int64_t)row * budget + pos] = tok;
      }
    }
  } else {
    const int total_vecs = n_kept * vpr_rt;
    for (int f = tid; f < total_vecs; f += kThreads) {
      const int e = f / vpr_rt, u = f - e * vpr_rt;
      const int tok = src_tok[e], pos = dst_pos[e];
      const int64_t src = ((int64_t)(t0 + tok) * num_kv_heads + h) * vpr_rt + u;
      const int64_t dst = ((int64_t)bt[pos / block_size] * block_size + pos % block_size) * vpr_rt + u;
      k_pool[dst] = k_in[src];
      v_pool[dst] = v_in[src];
      if (kept_idx_out != nullptr && u == 0) kept_idx_out[(int64_t)row * budget + pos] = tok;
    }
  }
}

template <typename T, int D>
hipError_t launch(const PruneArgs& a, hipStream_t stream) {
  using G = RowGeom<T, D>;
  const Workspace w = carve(a.workspace, a.num_seqs, a.num_kv_heads, a.total_tokens, a.shared);
  const int64_t total_rows = a.total_tokens * a.num_kv_heads;
  hipError_t e;
  if (total_rows > 0) {
    const int64_t rows_per_group = (int64_t)kWaves * kSweepIters * kSweepLoads * G::kTokensPerLoad;
    const int64_t grid = (total_rows + rows_per_group - 1) / rows_per_group;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((token_scores_kernel<T, D>), dim3((unsigned)grid), dim3(kThreads), 0, stream,
                       (const T*)a.k_in, (const T*)a.v_in, w.scores, total_rows, a.total_tokens, a.num_kv_heads);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  // what kernels 2-3 see: per-head rows, or (shared) one row per sequence whose score is the head mean and
  // whose record is the token's K (or V) of all heads
  const int heads = a.shared ? 1 : a.num_kv_heads;
  const float* sel_scores = w.scores;
  if (a.shared) {
    float* mean = w.scores + (size_t)a.num_kv_heads * (size_t)a.total_tokens;
    if (a.total_tokens > 0) {
      const int64_t grid = (a.total_tokens + kThreads - 1) / kThreads;
      hipLaunchKernelGGL(head_mean_kernel, dim3((unsigned)grid), dim3(kThreads), 0, stream, w.scores, mean,
                         a.total_tokens, a.num_kv_heads);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    sel_scores = mean;
  }
  const int rows = a.num_seqs * heads;
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)rows), dim3(kSelThreads), 0, stream, sel_scores, a.cu_seqlens,
                     w.sel, w.cnt, a.seq_lens_out, a.kept_idx_out, a.total_tokens, w.chunk_slots, heads, a.budget);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const int chunks_per_row = (a.max_seqlen + kChunk - 1) / kChunk;
  if (chunks_per_row == 0) return hipSuccess;
  const int64_t grid2 = (int64_t)rows * chunks_per_row;
  if (grid2 > 0x7fffffffLL) return hipErrorInvalidValue;
  constexpr int VPR = G::kLanesPerRow;
  if (a.shared) {
    hipLaunchKernelGGL((gather_kernel<0>), dim3((unsigned)grid2), dim3(kThreads), 0, stream, (const uint4*)a.k_in,
                       (const uint4*)a.v_in, sel_scores, a.cu_seqlens, w.sel, w.cnt, a.block_table, (uint4*)a.k_pool,
                       (uint4*)a.v_pool, a.kept_idx_out, a.total_tokens, w.chunk_slots, heads, chunks_per_row,
                       a.block_size, a.max_blocks, a.budget, VPR * a.num_kv_heads);
  } else {
    hipLaunchKernelGGL((gather_kernel<VPR>), dim3((unsigned)grid2), dim3(kThreads), 0, stream, (const uint4*)a.k_in,
                       (const uint4*)a.v_in, sel_scores, a.cu_seqlens, w.sel, w.cnt, a.block_table, (uint4*)a.k_pool,
                       (uint4*)a.v_pool, a.kept_idx_out, a.total_tokens, w.chunk_slots, heads, chunks_per_row,
                       a.block_size, a.max_blocks, a.budget, VPR);
  }
  return hipGetLastError();
}

}  // namespace

size_t prune_workspace_bytes(int num_seqs, int num_kv_heads, int64_t total_tokens, bool shared) {
  return align256(sizeof(float) * (size_t)(num_kv_heads + (shared ? 1 : 0)) * (size_t)total_tokens) +
         align256(sizeof(uint32_t) * 2 * (size_t)num_seqs * num_kv_heads) +
         align256(sizeof(int32_t) * 2 * (size_t)num_kv_heads * (size_t)chunk_slots_for(total_tokens, num_seqs));
}

hipError_t launch_prefill_prune(const PruneArgs& a, hipStream_t stream) {
  if (a.is_bf16) {
    if (a.head_dim == 64) return launch<bf16_t, 64>(a, stream);
    if (a.head_dim == 128) return launch<bf16_t, 128>(a, stream);
  } else {
    if (a.head_dim == 64) return launch<float, 64>(a, stream);
    if (a.head_dim == 128) return launch<float, 128>(a, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace pe
