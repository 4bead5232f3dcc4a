/*
 * pe_oracle.c -- plain CPU oracle for the PagedEviction hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
 * what the path computes.  It is called by the tests, by the smoke check and by
 * the CPU-baseline leg of the benchmark, and by nothing else.  It shares no code,
 * header, table or helper with the HIP library and neither includes the other.
 *
 * All floating point is fp64 on inputs that are handed over as fp32 arrays (a
 * bf16 value converts to fp32 exactly, so the caller loses nothing).  Loops run
 * in the index order of the paper's definitions: no blocking, no fusion, no
 * reordering.  The only parallelism is an OpenMP "parallel for" over rows that
 * are independent by definition (one row = one (sequence, KV head)).
 *
 * What each function follows:
 *   token ratio            Alg. 1 (token mode):  S_i = ||V_i||_2 / ||K_i||_2
 *   block score            Alg. 1 (block mode):  S_j = (1/B) sum_{i in block j} S_i ; Sec. 4.3
 *   prefill prune          Alg. 2 (score, E = L - C, evict E tokens, split into pages of B)
 *   evict                  Alg. 3 (when L % B == 0: evict the page with the lowest score,
 *                                  update the block table)
 *   paged decode           Eq. 1 / Alg. 3 "PagedAttention(Q,K,V)": softmax(q K^T * scale) V
 *                          over the tokens the block table still holds
 *   append                 harness step between evict and attention (new token's K/V
 *                          goes to the tail page; a new page when the tail is full)
 *
 * Readings taken where the paper is silent (each is also listed in the design notes):
 *   - decisions are per (sequence, KV head); every row owns its table row and pages;
 *   - block score = mean of per-token ratios (Alg. 1 and Sec. 4.3; not a whole-page
 *     Frobenius ratio);
 *   - eviction is gated on the budget: a row evicts only if its tail page is full and
 *     it holds >= C tokens (otherwise budget >= context could not reproduce full attention);
 *   - ties go to the lowest index: lowest logical page in decode; in prefill, among equal
 *     scores the lower token index is evicted first;
 *   - every full page is a candidate (no protected sink or recent page);
 *   - the table is compacted by a stable left shift, vacated tail entry = -1;
 *   - E = max(0, L - C);  C must be a multiple of B;
 *   - ||K|| = 0 gives +inf, 0/0 gives 0;
 *   - a score is computed in fp64 and rounded once to fp32; decisions compare those fp32 values.
 *
 * Parity pins: see tests/test_oracle_*.py (closed forms, library reductions, brute force,
 * the full-cache special case, a shadow token-id model).  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG -1
#define ORACLE_ERR_CAPACITY -2

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Alg. 1, token mode: r = ||v||_2 / ||k||_2, sums of squares taken in index order. */
double oracle_token_ratio(const float* k_row, const float* v_row, int D) {
  double sk = 0.0, sv = 0.0;
  for (int d = 0; d < D; ++d) sk += (double)k_row[d] * (double)k_row[d];
  for (int d = 0; d < D; ++d) sv += (double)v_row[d] * (double)v_row[d];
  if (sv == 0.0) return 0.0;
  if (sk == 0.0) return INFINITY;
  return sqrt(sv) / sqrt(sk);
}

/* Alg. 1, token mode over a packed prompt: k_in, v_in are [total_tokens][Hk][D];
 * ratio_out is [Hk][total_tokens] (fp64), one contiguous run per head. */
void oracle_token_ratios(const float* k_in, const float* v_in, int64_t total_tokens, int Hk, int D,
                         double* ratio_out) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < total_tokens; ++t)
    for (int h = 0; h < Hk; ++h) {
      const int64_t off = (t * Hk + h) * (int64_t)D;
      ratio_out[(int64_t)h * total_tokens + t] = oracle_token_ratio(k_in + off, v_in + off, D);
    }
}

/* Alg. 1, block mode, through the block table (Alg. 3: "Compute Score of Page i").
 * Pools are [P][B][D]; block_table is [S][Hk][max_blocks] (-1 = unused); seq_lens is [S].
 * scores_out [S][Hk][max_blocks]: full pages j < len/B get the mean ratio, summed in slot
 * order in fp64 and rounded once to fp32; every other entry is +inf. */
void oracle_score_blocks(const float* k_pool, const float* v_pool, const int32_t* block_table,
                         const int32_t* seq_lens, int S, int Hk, int D, int B, int max_blocks,
                         float* scores_out) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int row = 0; row < S * Hk; ++row) {
    const int s = row / Hk;
    const int nfull = seq_lens[s] / B;
    const int32_t* bt = block_table + (int64_t)row * max_blocks;
    float* out = scores_out + (int64_t)row * max_blocks;
    for (int j = 0; j < max_blocks; ++j) {
      if (j >= nfull) { out[j] = INFINITY; continue; }
      const int64_t page = (int64_t)bt[j] * B * D;
      double sum = 0.0;
      for (int i = 0; i < B; ++i)
        sum += oracle_token_ratio(k_pool + page + (int64_t)i * D, v_pool + page + (int64_t)i * D, D);
      out[j] = (float)(sum / (double)B);
    }
  }
}

typedef struct { float score; int32_t idx; } scored_token;

static int cmp_scored(const void* a, const void* b) {
  const scored_token* x = (const scored_token*)a;
  const scored_token* y = (const scored_token*)b;
  if (x->score < y->score) return -1;
  if (x->score > y->score) return 1;
  return (x->idx > y->idx) - (x->idx < y->idx);
}

static int cmp_i32(const void* a, const void* b) {
  const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* Alg. 2 (score every prompt token, evict E = L - C of them, then split what is left into
 * pages of B).  k_in, v_in [total][Hk][D]; cu_seqlens [S+1]; block_table [S][Hk][max_blocks]
 * is an input that names the physical page for each logical page the row will use.
 * Tokens are ordered by (fp32 score ascending, index ascending); the first E are evicted; the
 * kept ones keep their original order; kept token number i lands in page bt[i / B], slot i % B.
 * seq_lens_out[s] = min(L, C).  kept_idx_out [S][Hk][C] (may be NULL) receives the original
 * in-sequence indices of the kept tokens, -1 padded.  token_score_out [Hk][total] (may be
 * NULL) receives the fp32 token scores. */
int oracle_prefill_prune(const float* k_in, const float* v_in, const int32_t* cu_seqlens, int S, int Hk,
                         int D, int B, int C, int max_blocks, float* k_pool, float* v_pool,
                         const int32_t* block_table, int32_t* seq_lens_out, int32_t* kept_idx_out,
                         float* token_score_out) {
  if (C <= 0 || C % B != 0) return ORACLE_ERR_ARG;
  const int64_t total = cu_seqlens[S];
  int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (int row = 0; row < S * Hk; ++row) {
    const int s = row / Hk, h = row % Hk;
    const int64_t t0 = cu_seqlens[s];
    const int L = (int)(cu_seqlens[s + 1] - t0);
    const int keep = L < C ? L : C;
    const int E = L - keep; /* max(0, L - C) */
    if ((keep + B - 1) / B > max_blocks) {
#pragma omp critical
      status = ORACLE_ERR_CAPACITY;
      continue;
    }
    scored_token* tok = (scored_token*)malloc(sizeof(scored_token) * (size_t)(L > 0 ? L : 1));
    int32_t* kept = (int32_t*)malloc(sizeof(int32_t) * (size_t)(keep > 0 ? keep : 1));
    for (int i = 0; i < L; ++i) {
      const int64_t off = ((t0 + i) * Hk + h) * (int64_t)D;
      tok[i].score = (float)oracle_token_ratio(k_in + off, v_in + off, D);
      tok[i].idx = i;
      if (token_score_out) token_score_out[(int64_t)h * total + t0 + i] = tok[i].score;
    }
    qsort(tok, (size_t)L, sizeof(scored_token), cmp_scored);
    for (int i = 0; i < keep; ++i) kept[i] = tok[E + i].idx;
    qsort(kept, (size_t)keep, sizeof(int32_t), cmp_i32);
    const int32_t* bt = block_table + (int64_t)row * max_blocks;
    for (int i = 0; i < keep; ++i) {
      const int64_t src = ((t0 + kept[i]) * Hk + h) * (int64_t)D;
      const int64_t dst = ((int64_t)bt[i / B] * B + (i % B)) * (int64_t)D;
      memcpy(k_pool + dst, k_in + src, sizeof(float) * (size_t)D);
      memcpy(v_pool + dst, v_in + src, sizeof(float) * (size_t)D);
    }
    if (kept_idx_out) {
      int32_t* ko = kept_idx_out + (int64_t)row * C;
      for (int i = 0; i < C; ++i) ko[i] = i < keep ? kept[i] : -1;
    }
    if (h == 0) seq_lens_out[s] = keep;
    free(tok);
    free(kept);
  }
  return status;
}

/* Alg. 3, the eviction itself, from given fp32 page scores [S][Hk][max_blocks].
 * A sequence triggers when len % B == 0, len >= C and len > 0.  Each of its rows drops the
 * first page that attains the minimum score over j < len/B; later entries shift left by one,
 * the vacated tail entry becomes -1.  evicted_logical / freed_phys [S][Hk] get the logical
 * index / physical id, or -1 when the row did not evict.  seq_lens[s] -= B once. */
int oracle_evict_blocks(const float* scores, int32_t* block_table, int32_t* seq_lens, int S, int Hk, int B,
                        int max_blocks, int C, int32_t* evicted_logical_out, int32_t* freed_phys_out) {
  if (C <= 0 || C % B != 0) return ORACLE_ERR_ARG;
  for (int s = 0; s < S; ++s) {
    const int len = seq_lens[s];
    const int trigger = (len > 0) && (len % B == 0) && (len >= C);
    for (int h = 0; h < Hk; ++h) {
      const int row = s * Hk + h;
      if (!trigger) {
        evicted_logical_out[row] = -1;
        freed_phys_out[row] = -1;
        continue;
      }
      const int n = len / B;
      const float* sc = scores + (int64_t)row * max_blocks;
      int32_t* bt = block_table + (int64_t)row * max_blocks;
      int best = 0;
      for (int j = 1; j < n; ++j)
        if (sc[j] < sc[best]) best = j; /* strict "<": ties stay with the lowest index */
      evicted_logical_out[row] = best;
      freed_phys_out[row] = bt[best];
      for (int j = best; j + 1 < n; ++j) bt[j] = bt[j + 1];
      bt[n - 1] = -1;
    }
    if (trigger) seq_lens[s] = len - B;
  }
  return ORACLE_OK;
}

/* Variants of the eviction on the same table machinery (not the paper's main method; Sec. 5.2 and
 * App. A describe StreamingLLM, which keeps a few first tokens as attention sinks plus a window of the
 * most recent ones; Sec. 2.4 leaves open whether heads decide separately):
 *   policy 0  lowest score (as above);  policy 1  oldest page (sliding window, scores unused);
 *   protect_first / protect_last  pages at the start / end of a row that are never candidates;
 *   share_heads != 0  one decision per sequence: the page score is the mean over the sequence's KV
 *                     heads of the fp32 page scores, summed in head order in fp64 and rounded once
 *                     to fp32, and every head of the sequence drops the same logical page.
 * Candidates are the logical pages lo .. hi-1 with lo = min(protect_first, n-1) and
 * hi = max(n - protect_last, lo + 1): protection yields before the budget does, so there is always
 * one candidate.  Ties go to the lowest index.  Everything else is as in oracle_evict_blocks. */
int oracle_evict_blocks_ex(const float* scores, int32_t* block_table, int32_t* seq_lens, int S, int Hk, int B,
                           int max_blocks, int C, int policy, int protect_first, int protect_last,
                           int share_heads, int32_t* evicted_logical_out, int32_t* freed_phys_out) {
  if (C <= 0 || C % B != 0) return ORACLE_ERR_ARG;
  if (policy < 0 || policy > 1 || protect_first < 0 || protect_last < 0) return ORACLE_ERR_ARG;
  if (policy == 0 && scores == NULL) return ORACLE_ERR_ARG;
  for (int s = 0; s < S; ++s) {
    const int len = seq_lens[s];
    const int trigger = (len > 0) && (len % B == 0) && (len >= C);
    const int n = len / B;
    int lo = 0, hi = 0;
    if (trigger) {
      lo = protect_first < n - 1 ? protect_first : n - 1;
      hi = n - protect_last > lo + 1 ? n - protect_last : lo + 1;
    }
    for (int h = 0; h < Hk; ++h) {
      const int row = s * Hk + h;
      if (!trigger) {
        evicted_logical_out[row] = -1;
        freed_phys_out[row] = -1;
        continue;
      }
      int best = lo;
      if (policy == 0) {
        float best_score = 0.0f;
        for (int j = lo; j < hi; ++j) {
          float sc;
          if (share_heads) {
            double sum = 0.0;
            for (int g = 0; g < Hk; ++g) sum += (double)scores[((int64_t)s * Hk + g) * max_blocks + j];
            sc = (float)(sum / (double)Hk);
          } else {
            sc = scores[(int64_t)row * max_blocks + j];
          }
          if (j == lo || sc < best_score) { /* strict "<": ties stay with the lowest index */
            best = j;
            best_score = sc;
          }
        }
      }
      int32_t* bt = block_table + (int64_t)row * max_blocks;
      evicted_logical_out[row] = best;
      freed_phys_out[row] = bt[best];
      for (int j = best; j + 1 < n; ++j) bt[j] = bt[j + 1];
      bt[n - 1] = -1;
    }
    if (trigger) seq_lens[s] = len - B;
  }
  return ORACLE_OK;
}

/* Harness step between eviction and attention: the new token's K/V row of every (s, hk)
 * goes to slot len % B of the tail page.  When len % B == 0 a new page is linked in at
 * logical index len / B: the page this row freed in the eviction just before
 * (freed_phys[row] >= 0, consumed and reset to -1), else the next unused entry of the row's
 * spare list spare[row][spare_used[row]++].  seq_lens[s] += 1 once per sequence. */
int oracle_append_kv(const float* new_k, const float* new_v /* [S][Hk][D] */, float* k_pool, float* v_pool,
                     int32_t* block_table, int32_t* seq_lens, int32_t* freed_phys, const int32_t* spare,
                     int32_t* spare_used, int n_spare, int S, int Hk, int D, int B, int max_blocks) {
  for (int s = 0; s < S; ++s) {
    const int len = seq_lens[s];
    if (len / B >= max_blocks) return ORACLE_ERR_CAPACITY;
    for (int h = 0; h < Hk; ++h) {
      const int row = s * Hk + h;
      int32_t* bt = block_table + (int64_t)row * max_blocks;
      if (len % B == 0) {
        int32_t page;
        if (freed_phys[row] >= 0) {
          page = freed_phys[row];
          freed_phys[row] = -1;
        } else {
          if (spare_used[row] >= n_spare) return ORACLE_ERR_CAPACITY;
          page = spare[(int64_t)row * n_spare + spare_used[row]];
          spare_used[row] += 1;
        }
        bt[len / B] = page;
      }
      const int64_t dst = ((int64_t)bt[len / B] * B + (len % B)) * (int64_t)D;
      memcpy(k_pool + dst, new_k + (int64_t)row * D, sizeof(float) * (size_t)D);
      memcpy(v_pool + dst, new_v + (int64_t)row * D, sizeof(float) * (size_t)D);
    }
    seq_lens[s] = len + 1;
  }
  return ORACLE_OK;
}

/* Eq. 1 for one new query per sequence, read through the block table.
 * q [S][Hq][D]; query head hq uses KV head hq / (Hq/Hk).  Token t of row (s, g) sits in page
 * bt[t / B], slot t % B.  logit_t = scale * <q, k_t>;  m = max logit;  p_t = exp(logit_t - m);
 * out = sum_t p_t v_t / sum_t p_t.  A sequence with no cached token yields zeros.
 * out [S][Hq][D] fp64.  weights_sum_out [S][Hq] (may be NULL) receives
 * sum_t (p_t / sum p), which must be 1 up to rounding. */
void oracle_paged_decode(const float* q, const float* k_pool, const float* v_pool, const int32_t* block_table,
                         const int32_t* seq_lens, int S, int Hk, int Hq, int D, int B, int max_blocks,
                         double scale, double* out, double* weights_sum_out) {
  const int G = Hq / Hk;
#pragma omp parallel for schedule(dynamic, 1)
  for (int sh = 0; sh < S * Hq; ++sh) {
    const int s = sh / Hq, hq = sh % Hq, g = hq / G;
    const int len = seq_lens[s];
    const float* qv = q + (int64_t)sh * D;
    const int32_t* bt = block_table + ((int64_t)s * Hk + g) * max_blocks;
    double* o = out + (int64_t)sh * D;
    for (int d = 0; d < D; ++d) o[d] = 0.0;
    if (weights_sum_out) weights_sum_out[sh] = 0.0;
    if (len <= 0) continue;
    double* logit = (double*)malloc(sizeof(double) * (size_t)len);
    double m = -INFINITY;
    for (int t = 0; t < len; ++t) {
      const float* kr = k_pool + ((int64_t)bt[t / B] * B + (t % B)) * (int64_t)D;
      double dot = 0.0;
      for (int d = 0; d < D; ++d) dot += (double)qv[d] * (double)kr[d];
      logit[t] = scale * dot;
      if (logit[t] > m) m = logit[t];
    }
    double denom = 0.0;
    for (int t = 0; t < len; ++t) {
      logit[t] = exp(logit[t] - m); /* now p_t */
      denom += logit[t];
    }
    double wsum = 0.0;
    for (int t = 0; t < len; ++t) {
      const float* vr = v_pool + ((int64_t)bt[t / B] * B + (t % B)) * (int64_t)D;
      wsum += logit[t] / denom;
      for (int d = 0; d < D; ++d) o[d] += logit[t] * (double)vr[d];
    }
    for (int d = 0; d < D; ++d) o[d] /= denom;
    if (weights_sum_out) weights_sum_out[sh] = wsum;
    free(logit);
  }
}
