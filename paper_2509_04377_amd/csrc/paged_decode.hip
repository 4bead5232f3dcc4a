// Paged decode attention (Eq. 1 for one new query per sequence; Alg. 3 "PagedAttention(Q,K,V)").
//
// A workgroup owns one split of one (sequence, KV head) row: every splits-th group of four consecutive tiles
// of the row's tokens.  Each of its four waves walks tiles with a two-deep register pipeline.  Inside a tile every
// lane holds 16 bytes of four K rows and four V rows (consecutive lanes = consecutive addresses, so
// each wave-load is 1 KiB of one page, found through the block table with scalar loads).
//
//   QK:  each lane multiplies its K slice with the matching slice of all G query heads that share this
//        KV head; the partial dots are reduced over the lanes of a token row with a reduce-scatter over
//        heads, so that afterwards each lane owns the logit of ONE (token, head) pair;
//   softmax: online, state (m, l) kept per lane for its head and its own stream of tokens
//        (base-2 exponentials; the scale carries log2 e);
//   PV:  the lane's probability is broadcast inside its group of lanes and multiplies the V slice
//        into per-head fp32 accumulators.
//
// At the end the (wave, token-stream) partial states are merged through LDS; with one split the
// workgroup writes the normalised output, otherwise it writes (acc, m, l) partials that
// paged_decode_reduce_kernel merges.
//
// The FUSED variant also performs the harness append of the same decode iteration: the new token's K/V
// rows are taken from registers as one extra token of the row (they are not read back from the pool),
// the last split's workgroup links a new page if the tail page is full and stores the rows into the
// pool, and the new lengths go to a second array (the caller swaps the two), so no workgroup can see a
// length that another one has already bumped.
//
// The SHARED variant reads the head-shared cache layout: one table row per sequence and pages of
// [B][Hk][D], so the token rows of this workgroup's head are Hk rows apart (a wave-load is then TPL runs
// of one row each instead of one contiguous KiB).  Everything after the loads is the same.
#include "pe_device.h"
#include "pe_launch.h"

namespace pe {
namespace {

constexpr float kNegInf = -__builtin_inff();

constexpr int next_pow2(int x) { return x <= 1 ? 1 : 2 * next_pow2((x + 1) / 2); }

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// The 16 bytes of one query head that face a lane's 16-byte K slice.
template <typename T>
struct QSlice;
template <>
struct QSlice<float> {
  float v[4];
  __device__ __forceinline__ void load(const float* p) {
    const uint4 r = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(r.x);
    v[1] = __uint_as_float(r.y);
    v[2] = __uint_as_float(r.z);
    v[3] = __uint_as_float(r.w);
  }
  __device__ __forceinline__ void zero() { v[0] = v[1] = v[2] = v[3] = 0.f; }
  __device__ __forceinline__ float dot(const uint4& k) const {
    float a = __uint_as_float(k.x) * v[0];
    a = fmaf(__uint_as_float(k.y), v[1], a);
    a = fmaf(__uint_as_float(k.z), v[2], a);
    a = fmaf(__uint_as_float(k.w), v[3], a);
    return a;
  }
};
template <>
struct QSlice<bf16_t> {
  uint32_t v[4];  // 8 bf16, packed as in memory
  __device__ __forceinline__ void load(const bf16_t* p) {
    const uint4 r = *reinterpret_cast<const uint4*>(p);
    v[0] = r.x;
    v[1] = r.y;
    v[2] = r.z;
    v[3] = r.w;
  }
  __device__ __forceinline__ void zero() { v[0] = v[1] = v[2] = v[3] = 0u; }
  static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c,
                                           false);
  }
  __device__ __forceinline__ float dot(const uint4& k) const {
    float a = dot2(k.x, v[0], 0.f);
    a = dot2(k.y, v[1], a);
    a = dot2(k.z, v[2], a);
    a = dot2(k.w, v[3], a);
    return a;
  }
};

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Slot i of lane l carries head (i ^ c(l)), c(l) = bit_reverse(l & (GP-1)).  A stage with partner
// l ^ M keeps the lower half of the slots and adds the partner's upper half, which carries the same
// heads.  After log2(GP) stages slot 0 is the dot product of head c(l) summed over GP lanes.
template <int N, int M>
__device__ __forceinline__ float head_scatter(float (&v)[N]) {
  if constexpr (N == 1) {
    return v[0];
  } else {
    float w[N / 2];
#pragma unroll
    for (int i = 0; i < N / 2; ++i) w[i] = v[i] + lane_xor_f32<M>(v[i + N / 2]);
    return head_scatter<N / 2, M * 2>(w);
  }
}

// Sum over the remaining lane bits FROM .. LPR/2 of a token row (every lane gets the total).
template <int FROM, int LPR>
__device__ __forceinline__ float row_all_reduce(float v) {
  if constexpr (FROM >= LPR) {
    return v;
  } else if constexpr (FROM == 4 && LPR >= 16) {
    v += dpp_f32<0x124>(v);  // row_ror:4
    v += dpp_f32<0x128>(v);  // row_ror:8 -> total over the four quads of the 16-lane row
    return row_all_reduce<16, LPR>(v);
  } else if constexpr (FROM == 8 && LPR >= 16) {
    v += dpp_f32<0x128>(v);  // row_ror:8 is lane ^ 8 inside a 16-lane row
    return row_all_reduce<16, LPR>(v);
  } else {
    v += lane_xor_f32<FROM>(v);
    return row_all_reduce<FROM * 2, LPR>(v);
  }
}

// acc[h][:] *= alpha of head h, which lives on lane position bit_reverse(h) of each GP-lane group.
template <int G, int GP, int EPL, int H = 0>
__device__ __forceinline__ void rescale_acc(float (&acc)[G][EPL], float alpha) {
  if constexpr (H < G) {
    const float a = group_bcast_f32<GP, bit_reverse<ilog2(GP)>(H)>(alpha);
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[H][e] *= a;
    rescale_acc<G, GP, EPL, H + 1>(acc, alpha);
  }
}

// acc[h][:] += prob of head h (broadcast as above) * v[:].
template <int G, int GP, int EPL, int H = 0>
__device__ __forceinline__ void accumulate_pv(float (&acc)[G][EPL], float prob, const float (&v)[EPL]) {
  if constexpr (H < G) {
    const float ph = group_bcast_f32<GP, bit_reverse<ilog2(GP)>(H)>(prob);
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[H][e] = fmaf(ph, v[e], acc[H][e]);
    accumulate_pv<G, GP, EPL, H + 1>(acc, prob, v);
  }
}

struct DecodeParams {
  const void* q;
  const void* k_pool;
  const void* v_pool;
  const int32_t* block_table;
  const int32_t* seq_lens;
  void* out;
  float* partials;
  float scale_log2e;
  int num_kv_heads, num_q_heads, max_blocks, log2_block, splits, xcd_map, g_real;
  // fused append (FUSED kernels only)
  const void* new_k;
  const void* new_v;
  int32_t* freed_phys;
  const int32_t* spare;
  int32_t* spare_used;
  int32_t* seq_lens_out;  // [S], must not alias seq_lens
  int n_spare;
};

template <typename T, int D, int G, int LOADS>
struct Tile {
  using Geo = RowGeom<T, D>;
  static constexpr int EPL = Geo::kPerVec;
  static constexpr int LPR = Geo::kLanesPerRow;
  static constexpr int TPL = Geo::kTokensPerLoad;
  static constexpr int NLT = LOADS;  // wave-loads of K (and of V) per tile
  static constexpr int TT = NLT * TPL;  // tokens per tile
  static constexpr int GP = next_pow2(G);
  static_assert(GP <= LPR && GP <= 8, "query group too large");

  // A tile touches at most NPT pages (two when a 32-token tile meets 16-token pages).
  static constexpr int NPT = TT > 16 ? TT / 16 : 1;

  // Scalar loads of the physical page ids of tile `tile`.  The index is clamped to the table row, and an
  // unused entry (-1, beyond the row's last page) is replaced by page 0: the tokens of such a page are
  // masked later, so any address inside the pool will do.  Nothing here depends on the row length, so
  // the first lookup can be issued before the length has arrived.
  static __device__ __forceinline__ void lookup(int (&phys)[NPT], int tile, const int32_t* bt, int max_blocks,
                                                int log2_block) {
    const int p0 = (tile * TT) >> log2_block;
#pragma unroll
    for (int e = 0; e < NPT; ++e) {
      int pi = p0 + e;
      pi = pi < max_blocks ? pi : max_blocks - 1;
      const int ph = __builtin_amdgcn_readfirstlane(bt[pi]);
      phys[e] = ph < 0 ? 0 : ph;
    }
  }

  // Issue the 2*NLT wave-loads of tile `tile`, whose page ids were looked up one step earlier (the table
  // access is off the critical path of the loads).  `lane_off` is the lane id, or 0 in every lane for a
  // placeholder issue whose data is never used (all lanes then fetch the same 16 bytes): issues stay
  // unconditional, which keeps the order of outstanding loads known at compile time, so waiting for the
  // oldest tile leaves the younger ones in flight.
  static __device__ __forceinline__ void issue(uint4 (&kb)[NLT], uint4 (&vb)[NLT], int tile, const int (&phys)[NPT],
                                               const T* k_pool, const T* v_pool, int log2_block, int lane_off,
                                               int row_vecs = LPR) {
    const int tok0 = tile * TT;
#pragma unroll
    for (int i = 0; i < NLT; ++i) {
      const int t = tok0 + i * TPL;
      int ph = phys[0];
#pragma unroll
      for (int e = 1; e < NPT; ++e)
        if (((i * TPL) >> log2_block) == e) ph = phys[e];
      const int slot0 = t & ((1 << log2_block) - 1);
      const int64_t vec = (((int64_t)ph << log2_block) + slot0) * row_vecs + lane_off;
      kb[i] = load_vec_stream(k_pool, vec);
      vb[i] = load_vec_stream(v_pool, vec);
    }
  }

  // Consume NL wave-loads whose first token is tok0: logits, online softmax update, PV accumulation.
  template <int NL>
  static __device__ __forceinline__ void compute(uint4 (&kb)[NL], uint4 (&vb)[NL], int tok0, int len, int grp,
                                                 float scale_log2e, const QSlice<T> (&qs)[GP], float& m_run,
                                                 float& l_run, float (&acc)[G][EPL]) {
    float x[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      float sd[GP];
#pragma unroll
      for (int j = 0; j < GP; ++j) sd[j] = qs[j].dot(kb[i]);
      float r = head_scatter<GP, 1>(sd);
      r = row_all_reduce<GP, LPR>(r);
      x[i] = r * scale_log2e;
    }
    if (tok0 + NL * TPL > len) {  // the tile reaches past the row: mask logits, keep junk V out of the sum
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const bool ok = tok0 + i * TPL + grp < len;
        x[i] = ok ? x[i] : kNegInf;
        if (!ok) vb[i] = make_uint4(0u, 0u, 0u, 0u);
      }
    }
    float m_new = m_run;
#pragma unroll
    for (int i = 0; i < NL; ++i) m_new = fmaxf(m_new, x[i]);
    const float m_safe = m_new == kNegInf ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
    float pr[NL];
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      pr[i] = __builtin_amdgcn_exp2f(x[i] - m_safe);
      psum += pr[i];
    }
    l_run = fmaf(l_run, alpha, psum);
    const bool changed = m_new != m_run;
    m_run = m_new;
    if (__builtin_amdgcn_ballot_w64(changed) != 0ull) rescale_acc<G, GP, EPL>(acc, alpha);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      float ve[EPL];
#pragma unroll
      for (int e = 0; e < EPL; ++e) ve[e] = vec_elem<T>(vb[i], e);
      accumulate_pv<G, GP, EPL>(acc, pr[i], ve);
    }
  }
};

template <typename T, int D, int G, int WAVES, int DEPTH, int LOADS, bool FUSED, bool SHARED = false>
__global__ __launch_bounds__(WAVES * kWave) void paged_decode_kernel(const DecodeParams p) {
  static_assert(!(FUSED && SHARED), "the fused append is per-head only");
  using TL = Tile<T, D, G, LOADS>;
  constexpr int EPL = TL::EPL, LPR = TL::LPR, TPL = TL::TPL, NLT = TL::NLT, TT = TL::TT, GP = TL::GP;
  constexpr int GBITS = ilog2(GP);
  constexpr int NCONTRIB = WAVES * TPL;

  constexpr int HC = G < 4 ? G : 4;  // heads merged per LDS pass
  __shared__ float sm_m[NCONTRIB][GP];
  __shared__ float sm_l[NCONTRIB][GP];
  __shared__ float sm_ML[G][2];
  __shared__ __attribute__((aligned(16))) float sm_acc[NCONTRIB][HC][D];

  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int u = lane % LPR;    // which 16-byte slice of the token row
  const int grp = lane / LPR;  // which token row of a wave-load
  const int c_lane = bit_reverse<GBITS>(lane & (GP - 1));

  int row, split;
  {
    const int b = (int)blockIdx.x;
    if (p.xcd_map) {  // workgroup b runs on XCD b % 8: keep all splits of a row on one XCD
      const int xcd = b & 7, k = b >> 3;
      row = (k / p.splits) * 8 + xcd;
      split = k % p.splits;
    } else {
      row = b / p.splits;
      split = b % p.splits;
    }
  }
  const int s = row / p.num_kv_heads;
  const int hk = row % p.num_kv_heads;
  // SHARED: one table row per sequence; a page holds [B][Hk][D], so consecutive tokens of this head are
  // Hk rows apart and a lane's offset inside a wave-load carries the head
  const int32_t* bt = p.block_table + (int64_t)(SHARED ? s : row) * p.max_blocks;
  const int row_vecs = SHARED ? LPR * p.num_kv_heads : LPR;
  const int lane_vec = SHARED ? (grp * p.num_kv_heads + hk) * LPR + u : lane;
  const T* k_pool = static_cast<const T*>(p.k_pool);
  const T* v_pool = static_cast<const T*>(p.v_pool);

  // ---- prologue: everything that does not depend on the row length is requested first --------------
  // query slices: slot i holds head (i ^ c_lane) of this KV head's group (heads past the group: zeros)
  QSlice<T> qs[GP];
#pragma unroll
  for (int i = 0; i < GP; ++i) {
    const int head = i ^ c_lane;
    const int head_ld = head < p.g_real ? head : 0;
    qs[i].load(static_cast<const T*>(p.q) + ((int64_t)s * p.num_q_heads + hk * p.g_real + head_ld) * D + u * EPL);
  }
  uint4 nk[1], nv[1];  // FUSED: the new token's K/V rows, held by the first lane group of every wave
  if constexpr (FUSED) {
    const int64_t vec = (int64_t)row * LPR + u;
    nk[0] = load_vec(p.new_k, vec);
    nv[0] = load_vec(p.new_v, vec);
  }
  // The row's tiles are dealt out round-robin: tile t belongs to split (t / WAVES) % splits, wave t % WAVES.  A
  // wave's first tile is therefore the same whatever the row length, and the lookup of its page travels
  // together with the length itself instead of waiting for it (one dependent round trip to memory less).
  const int stride = p.splits * WAVES;
  const int first = split * WAVES + wave;
  int phys[TL::NPT];
  TL::lookup(phys, first, bt, p.max_blocks, p.log2_block);
  const int len_pool = p.seq_lens[s];               // tokens that are read from the pool
  const int len = FUSED ? len_pool + 1 : len_pool;  // tokens attended to
#pragma unroll
  for (int i = 0; i < GP; ++i)
    if ((i ^ c_lane) >= p.g_real) qs[i].zero();
  // FUSED: requests for what the append needs, issued now and used after the main loop
  const bool appender = FUSED && split == p.splits - 1 && wave == WAVES - 1;  // wave-uniform
  int ap_freed = -1, ap_used = 0;
  if constexpr (FUSED) {
    if (appender) {
      ap_freed = p.freed_phys[row];
      ap_used = p.spare_used[row];
    }
  }
  const int ntiles = (len_pool + TT - 1) / TT;

  float m_run = kNegInf;  // running max of head c_lane over this lane's stream of tokens
  float l_run = 0.f;
  float acc[G][EPL];
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;

  // This wave's tiles are first + i*stride, i = 0 .. n_mine-1.  DEPTH register buffers: while tile i is
  // consumed, tiles i+1 .. i+DEPTH-1 are in flight.
  const int n_mine = first < ntiles ? (ntiles - first + stride - 1) / stride : 0;
  if (n_mine > 0) {
    uint4 kb[DEPTH][NLT], vb[DEPTH][NLT];
    const auto tile_at = [&](int i) { return first + (i < n_mine ? i : n_mine - 1) * stride; };
#pragma unroll
    for (int d = 0; d < DEPTH - 1; ++d) {
      TL::issue(kb[d], vb[d], tile_at(d), phys, k_pool, v_pool, p.log2_block, d < n_mine ? lane_vec : 0, row_vecs);
      TL::lookup(phys, tile_at(d + 1), bt, p.max_blocks, p.log2_block);
    }
    for (int i = 0; i < n_mine; i += DEPTH) {
#pragma unroll
      for (int ph = 0; ph < DEPTH; ++ph) {
        const int ahead = i + ph + DEPTH - 1;
        TL::issue(kb[(ph + DEPTH - 1) % DEPTH], vb[(ph + DEPTH - 1) % DEPTH], tile_at(ahead), phys, k_pool, v_pool,
                  p.log2_block, ahead < n_mine ? lane_vec : 0, row_vecs);
        TL::lookup(phys, tile_at(ahead + 1), bt, p.max_blocks, p.log2_block);
        if (i + ph < n_mine) {
          TL::template compute<NLT>(kb[ph], vb[ph], (first + (i + ph) * stride) * TT, len_pool, grp, p.scale_log2e, qs,
                                    m_run, l_run, acc);
        }
      }
    }
  }

  if constexpr (FUSED) {
    // the new token is token number len_pool of the row: wave 0 of the last split attends to it from
    // registers ...
    if (split == p.splits - 1 && wave == 0)
      TL::template compute<1>(nk, nv, len_pool, len_pool + (grp == 0 ? 1 : 0), 0, p.scale_log2e, qs, m_run, l_run, acc);
    // ... and the first lane group of its last wave stores it into the pool, linking a new page first when
    // the tail page is full (the page freed by the eviction just before, else the next spare)
    if (appender) {
      const int B = 1 << p.log2_block;
      const int slot = len_pool & (B - 1);
      const int jb = len_pool >> p.log2_block;
      if (len_pool >= 0 && jb < p.max_blocks) {  // a length outside the table row is a caller error: touch nothing
        int page;
        if (slot == 0) {
          page = ap_freed;
          if (page < 0) {
            page = ap_used < p.n_spare ? p.spare[(int64_t)row * p.n_spare + ap_used] : -1;
            if (lane == 0) p.spare_used[row] = ap_used + 1;
          } else if (lane == 0) {
            p.freed_phys[row] = -1;
          }
          if (lane == 0) const_cast<int32_t*>(bt)[jb] = page;
        } else {
          page = bt[jb];
        }
        if (page >= 0 && grp == 0) {
          const int64_t vec = (((int64_t)page << p.log2_block) + slot) * LPR + u;
          reinterpret_cast<uint4*>(const_cast<void*>(p.k_pool))[vec] = nk[0];
          reinterpret_cast<uint4*>(const_cast<void*>(p.v_pool))[vec] = nv[0];
        }
      }
      if (hk == 0 && lane == 0) p.seq_lens_out[s] = len_pool + 1;
    }
  }

  // ---- merge the WAVES x TPL token streams of this workgroup through LDS ------------------------------
  // (1) every stream publishes its (m, l) per head; (2) one thread per head folds them into the row's
  // (M, L); (3) every lane rescales its accumulators to M and publishes them, up to four heads per pass;
  // (4) all threads sum the streams and write the output (or the split partial).
  const int contrib = wave * TPL + grp;
  if (u < GP) {
    sm_m[contrib][c_lane] = m_run;
    sm_l[contrib][c_lane] = l_run;
  }
  __syncthreads();
  if ((int)threadIdx.x < G) {
    const int h = (int)threadIdx.x;
    float mm = kNegInf;
    for (int c = 0; c < NCONTRIB; ++c) mm = fmaxf(mm, sm_m[c][h]);
    const float ms = mm == kNegInf ? 0.f : mm;
    float ll = 0.f;
    for (int c = 0; c < NCONTRIB; ++c) ll = fmaf(sm_l[c][h], __builtin_amdgcn_exp2f(sm_m[c][h] - ms), ll);
    sm_ML[h][0] = mm;
    sm_ML[h][1] = ll;
  }
  __syncthreads();
#pragma unroll
  for (int h0 = 0; h0 < G; h0 += HC) {
    if (h0 > 0) __syncthreads();  // the previous pass has been read
#pragma unroll
    for (int hh = 0; hh < HC; ++hh) {
      const int h = h0 + hh;
      if (h < G) {
        const float mm = sm_ML[h][0];
        const float ms = mm == kNegInf ? 0.f : mm;
        const float f = __builtin_amdgcn_exp2f(sm_m[contrib][h] - ms);
        float4* dst = reinterpret_cast<float4*>(&sm_acc[contrib][hh][u * EPL]);
#pragma unroll
        for (int e = 0; e < EPL; e += 4)
          dst[e / 4] = make_float4(acc[h][e] * f, acc[h][e + 1] * f, acc[h][e + 2] * f, acc[h][e + 3] * f);
      }
    }
    __syncthreads();
    for (int idx = (int)threadIdx.x; idx < HC * D; idx += WAVES * kWave) {
      const int hh = idx / D, d = idx % D;
      const int h = h0 + hh;
      if (h >= p.g_real) continue;
      const float mm = sm_ML[h][0], ll = sm_ML[h][1];
      float o = 0.f;
#pragma unroll 8
      for (int c = 0; c < NCONTRIB; ++c) o += sm_acc[c][hh][d];
      if (p.splits == 1) {
        const float r = ll > 0.f ? o / ll : 0.f;
        const int64_t off = ((int64_t)s * p.num_q_heads + hk * p.g_real + h) * D + d;
        if constexpr (sizeof(T) == 4) {
          static_cast<float*>(p.out)[off] = r;
        } else {
          static_cast<uint16_t*>(p.out)[off] = f32_to_bf16(r);
        }
      } else {
        float* part = p.partials + (((int64_t)row * p.splits + split) * p.g_real + h) * (D + 2);
        part[d] = o;
        if (d == 0) {
          part[D] = mm;
          part[D + 1] = ll;
        }
      }
    }
  }
}

// Merge the split partials of one (sequence, query head): one workgroup of D threads.
template <typename T, int D>
__global__ __launch_bounds__(D) void paged_decode_reduce_kernel(const float* __restrict__ partials,
                                                                void* __restrict__ out, int num_kv_heads, int g_real,
                                                                int splits) {
  const int sh = (int)blockIdx.x;  // s * Hq + hq
  const int num_q_heads = num_kv_heads * g_real;
  const int s = sh / num_q_heads, hq = sh % num_q_heads;
  const int row = s * num_kv_heads + hq / g_real;
  const int h = hq % g_real;
  const int d = (int)threadIdx.x;
  const float* base = partials + (((int64_t)row * splits) * g_real + h) * (D + 2);
  const int64_t stride = (int64_t)g_real * (D + 2);
  // one pass, online: all loads are independent of the running state, so they overlap
  float mm = kNegInf, o = 0.f, l = 0.f;
#pragma unroll 4
  for (int sp = 0; sp < splits; ++sp) {
    const float m_sp = base[sp * stride + D];
    const float l_sp = base[sp * stride + D + 1];
    const float a_sp = base[sp * stride + d];
    const float m_new = fmaxf(mm, m_sp);
    const float ms = m_new == kNegInf ? 0.f : m_new;
    const float w_old = __builtin_amdgcn_exp2f(mm - ms), w_new = __builtin_amdgcn_exp2f(m_sp - ms);
    l = fmaf(l, w_old, l_sp * w_new);
    o = fmaf(o, w_old, a_sp * w_new);
    mm = m_new;
  }
  const float r = l > 0.f ? o / l : 0.f;
  const int64_t off = (int64_t)sh * D + d;
  if constexpr (sizeof(T) == 4) {
    static_cast<float*>(out)[off] = r;
  } else {
    static_cast<uint16_t*>(out)[off] = f32_to_bf16(r);
  }
}

template <typename T, int D, int G, int WAVES, int DEPTH, int LOADS>
hipError_t launch_one(const DecodeArgs& a, hipStream_t stream) {
  DecodeParams p;
  p.q = a.q;
  p.k_pool = a.k_pool;
  p.v_pool = a.v_pool;
  p.block_table = a.block_table;
  p.seq_lens = a.seq_lens;
  p.out = a.out;
  p.partials = a.partials;
  p.scale_log2e = a.scale * 1.4426950408889634f;
  p.num_kv_heads = a.num_kv_heads;
  p.num_q_heads = a.num_q_heads;
  p.max_blocks = a.max_blocks;
  p.log2_block = ilog2(a.block_size);
  p.splits = a.splits;
  p.g_real = a.num_q_heads / a.num_kv_heads;
  p.new_k = a.new_k;
  p.new_v = a.new_v;
  p.freed_phys = a.freed_phys;
  p.spare = a.spare;
  p.spare_used = a.spare_used;
  p.seq_lens_out = a.seq_lens_out;
  p.n_spare = a.n_spare;
  const int64_t rows = (int64_t)a.num_seqs * a.num_kv_heads;
  p.xcd_map = (a.xcd_map && rows % 8 == 0) ? 1 : 0;
  const int64_t grid = rows * a.splits;
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  if (a.shared) {
    if (a.new_k != nullptr) return hipErrorInvalidValue;
    if constexpr (WAVES == 4 && DEPTH == 2 && LOADS == 2) {
      hipLaunchKernelGGL((paged_decode_kernel<T, D, G, WAVES, DEPTH, LOADS, false, true>), dim3((unsigned)grid),
                         dim3(WAVES * kWave), 0, stream, p);
    } else {
      return hipErrorInvalidValue;
    }
  } else if (a.new_k != nullptr) {
    hipLaunchKernelGGL((paged_decode_kernel<T, D, G, WAVES, DEPTH, LOADS, true>), dim3((unsigned)grid), dim3(WAVES * kWave), 0,
                       stream, p);
  } else {
    hipLaunchKernelGGL((paged_decode_kernel<T, D, G, WAVES, DEPTH, LOADS, false>), dim3((unsigned)grid), dim3(WAVES * kWave),
                       0, stream, p);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.splits == 1) return e;
  hipLaunchKernelGGL((paged_decode_reduce_kernel<T, D>), dim3((unsigned)(a.num_seqs * a.num_q_heads)), dim3(D), 0,
                     stream, a.partials, a.out, a.num_kv_heads, p.g_real, a.splits);
  return hipGetLastError();
}

// Workgroup shape: four waves, two register buffers, two wave-loads of K and of V per tile (4 KiB per tile,
// 8 KiB per wave in flight while it waits).  On an MI355X the stream runs fastest at about 8 MiB in flight
// over the chip: measured on the headline shape 45.0 us per launch against 46.8 (4 loads per tile),
// 45.9 (three buffers), 47.3 (eight waves) and 62 (one load per tile).  The other shapes are selectable
// for tuning on the headline instantiation only.
template <typename T, int D, int G>
hipError_t launch_variant(const DecodeArgs& a, hipStream_t stream) {
  if constexpr (sizeof(T) == 2 && D == 128 && G == 4) {
    switch (a.waves * 100 + a.depth * 10 + a.loads) {
      case 422: return launch_one<T, D, G, 4, 2, 2>(a, stream);
      case 424: return launch_one<T, D, G, 4, 2, 4>(a, stream);
      case 432: return launch_one<T, D, G, 4, 3, 2>(a, stream);
      case 822: return launch_one<T, D, G, 8, 2, 2>(a, stream);
      default: return hipErrorInvalidValue;
    }
  } else {
    return launch_one<T, D, G, 4, 2, 2>(a, stream);
  }
}

template <typename T, int D>
hipError_t launch_group(const DecodeArgs& a, hipStream_t stream) {
  const int g = a.num_q_heads / a.num_kv_heads;
  switch (g) {
    case 1: return launch_variant<T, D, 1>(a, stream);
    case 2: return launch_variant<T, D, 2>(a, stream);
    case 3: return launch_variant<T, D, 3>(a, stream);
    case 4: return launch_variant<T, D, 4>(a, stream);
    case 5: case 6: case 7: case 8: return launch_variant<T, D, 8>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

size_t decode_partials_bytes(int num_seqs, int num_q_heads, int head_dim, int splits) {
  if (splits <= 1) return 0;
  return (size_t)num_seqs * num_q_heads * splits * (head_dim + 2) * sizeof(float);
}

hipError_t launch_paged_decode(const DecodeArgs& a, hipStream_t stream) {
  if (a.is_bf16) {
    if (a.head_dim == 64) return launch_group<bf16_t, 64>(a, stream);
    if (a.head_dim == 128) return launch_group<bf16_t, 128>(a, stream);
  } else {
    if (a.head_dim == 64) return launch_group<float, 64>(a, stream);
    if (a.head_dim == 128) return launch_group<float, 128>(a, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace pe
