/*
 * pe_oracle_shared.c -- plain CPU oracle for the head-shared reading of PagedEviction.
 *
 * TEST INFRASTRUCTURE ONLY (see pe_oracle.c; the same rules hold here).
 *
 * Sec. 2.4 describes pages that hold the keys and values of a fixed number of tokens and Sec. 3 / 4
 * never say whether heads decide separately.  The second reading, the one a stock paged cache with
 * one block table per sequence imposes, is written out here:
 *   - ONE table row per sequence; page p holds, for each of its B token slots, the K (sibling pool:
 *     V) rows of ALL Hk heads:  element (p, slot i, head h, d) sits at ((p*B + i)*Hk + h)*D + d;
 *   - ONE decision per sequence.  A token's / page's importance is the mean over the KV heads of the
 *     per-head fp32 scores of Alg. 1 (summed in head order in fp64, divided by Hk, rounded once to
 *     fp32): tokens (prefill, Alg. 2) and pages (decode, Alg. 3) are dropped for all heads at once.
 * Everything else (budget gate, ties to the lowest index, stable compaction, E = max(0, L - C),
 * zero-norm conventions, one rounding per score) is as in pe_oracle.c.
 *
 * Parity pins: tests/test_oracle_shared.py (Hk = 1 reduces to pe_oracle.c; head slices of a shared
 * pool fed to the per-head functions; brute force; closed forms).  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG -1
#define ORACLE_ERR_CAPACITY -2

double oracle_token_ratio(const float* k_row, const float* v_row, int D); /* pe_oracle.c, Alg. 1 token mode */

/* offset of the D-vector of (page p, slot i, head h) */
static int64_t sh_off(int64_t p, int i, int h, int B, int Hk, int D) { return ((p * B + i) * Hk + h) * (int64_t)D; }

/* mean over heads of fp32 values: head order, fp64, one rounding */
static float head_mean(const float* per_head, int Hk) {
  double sum = 0.0;
  for (int h = 0; h < Hk; ++h) sum += (double)per_head[h];
  return (float)(sum / (double)Hk);
}

/* Alg. 1 block mode per head, then the mean over heads.  block_table [S][max_blocks], seq_lens [S].
 * head_scores_out [S][Hk][max_blocks] (fp32 per-head page scores, +inf for entries that are not full
 * pages); page_scores_out [S][max_blocks] (their head mean; +inf likewise). */
void oracle_sh_score_blocks(const float* k_pool, const float* v_pool, const int32_t* block_table,
                            const int32_t* seq_lens, int S, int Hk, int D, int B, int max_blocks,
                            float* head_scores_out, float* page_scores_out) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int s = 0; s < S; ++s) {
    float* tmp = (float*)malloc(sizeof(float) * (size_t)Hk);
    const int nfull = seq_lens[s] / B;
    for (int j = 0; j < max_blocks; ++j) {
      for (int h = 0; h < Hk; ++h) {
        float sc = INFINITY;
        if (j < nfull) {
          const int64_t p = block_table[(int64_t)s * max_blocks + j];
          double sum = 0.0;
          for (int i = 0; i < B; ++i)
            sum += oracle_token_ratio(k_pool + sh_off(p, i, h, B, Hk, D), v_pool + sh_off(p, i, h, B, Hk, D), D);
          sc = (float)(sum / (double)B);
        }
        tmp[h] = sc;
        head_scores_out[((int64_t)s * Hk + h) * max_blocks + j] = sc;
      }
      page_scores_out[(int64_t)s * max_blocks + j] = j < nfull ? head_mean(tmp, Hk) : INFINITY;
    }
    free(tmp);
  }
}

typedef struct { float score; int32_t idx; } sh_scored;

static int sh_cmp(const void* a, const void* b) {
  const sh_scored* x = (const sh_scored*)a;
  const sh_scored* y = (const sh_scored*)b;
  if (x->score < y->score) return -1;
  if (x->score > y->score) return 1;
  return (x->idx > y->idx) - (x->idx < y->idx);
}

static int sh_cmp_i32(const void* a, const void* b) {
  const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* Alg. 2 with one decision per sequence.  k_in, v_in [total][Hk][D]; cu_seqlens [S+1]; block_table
 * [S][max_blocks] names the page of each logical page the sequence will use.  Token score = head mean
 * of the per-head fp32 ratios.  Tokens are ordered by (score ascending, index ascending); the first
 * E = max(0, L - C) go, for every head; the kept ones keep their order; kept token number i lands in
 * page bt[i / B], slot i % B, all heads.  kept_idx_out [S][C] (may be NULL), -1 padded;
 * token_score_out [total] (may be NULL). */
int oracle_sh_prefill_prune(const float* k_in, const float* v_in, const int32_t* cu_seqlens, int S, int Hk, int D,
                            int B, int C, int max_blocks, float* k_pool, float* v_pool,
                            const int32_t* block_table, int32_t* seq_lens_out, int32_t* kept_idx_out,
                            float* token_score_out) {
  if (C <= 0 || C % B != 0) return ORACLE_ERR_ARG;
  int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (int s = 0; s < S; ++s) {
    const int64_t t0 = cu_seqlens[s];
    const int L = (int)(cu_seqlens[s + 1] - t0);
    const int keep = L < C ? L : C;
    const int E = L - keep;
    if ((keep + B - 1) / B > max_blocks) {
#pragma omp critical
      status = ORACLE_ERR_CAPACITY;
      continue;
    }
    float* tmp = (float*)malloc(sizeof(float) * (size_t)Hk);
    sh_scored* tok = (sh_scored*)malloc(sizeof(sh_scored) * (size_t)(L > 0 ? L : 1));
    int32_t* kept = (int32_t*)malloc(sizeof(int32_t) * (size_t)(keep > 0 ? keep : 1));
    for (int i = 0; i < L; ++i) {
      for (int h = 0; h < Hk; ++h) {
        const int64_t off = ((t0 + i) * Hk + h) * (int64_t)D;
        tmp[h] = (float)oracle_token_ratio(k_in + off, v_in + off, D);
      }
      tok[i].score = head_mean(tmp, Hk);
      tok[i].idx = i;
      if (token_score_out) token_score_out[t0 + i] = tok[i].score;
    }
    qsort(tok, (size_t)L, sizeof(sh_scored), sh_cmp);
    for (int i = 0; i < keep; ++i) kept[i] = tok[E + i].idx;
    qsort(kept, (size_t)keep, sizeof(int32_t), sh_cmp_i32);
    const int32_t* bt = block_table + (int64_t)s * max_blocks;
    for (int i = 0; i < keep; ++i)
      for (int h = 0; h < Hk; ++h) {
        const int64_t src = ((t0 + kept[i]) * Hk + h) * (int64_t)D;
        const int64_t dst = sh_off(bt[i / B], i % B, h, B, Hk, D);
        memcpy(k_pool + dst, k_in + src, sizeof(float) * (size_t)D);
        memcpy(v_pool + dst, v_in + src, sizeof(float) * (size_t)D);
      }
    if (kept_idx_out)
      for (int i = 0; i < C; ++i) kept_idx_out[(int64_t)s * C + i] = i < keep ? kept[i] : -1;
    seq_lens_out[s] = keep;
    free(tok);
    free(kept);
    free(tmp);
  }
  return status;
}

/* Alg. 3 eviction with one decision per sequence, from per-head fp32 page scores [S][Hk][max_blocks]
 * (NULL allowed for policy 1).  policy 0: the page with the lowest head-mean score; policy 1: the oldest
 * candidate.  Candidates lo .. hi-1 with lo = min(protect_first, n-1), hi = max(n - protect_last, lo+1).
 * block_table [S][max_blocks]; evicted_logical_out / freed_phys_out [S]. */
int oracle_sh_evict_blocks(const float* head_scores, int32_t* block_table, int32_t* seq_lens, int S, int Hk, int B,
                           int max_blocks, int C, int policy, int protect_first, int protect_last,
                           int32_t* evicted_logical_out, int32_t* freed_phys_out) {
  if (C <= 0 || C % B != 0) return ORACLE_ERR_ARG;
  if (policy < 0 || policy > 1 || protect_first < 0 || protect_last < 0) return ORACLE_ERR_ARG;
  if (policy == 0 && head_scores == NULL) return ORACLE_ERR_ARG;
  float* tmp = (float*)malloc(sizeof(float) * (size_t)Hk);
  for (int s = 0; s < S; ++s) {
    const int len = seq_lens[s];
    evicted_logical_out[s] = -1;
    freed_phys_out[s] = -1;
    if (!((len > 0) && (len % B == 0) && (len >= C))) continue;
    const int n = len / B;
    const int lo = protect_first < n - 1 ? protect_first : n - 1;
    const int hi = n - protect_last > lo + 1 ? n - protect_last : lo + 1;
    int best = lo;
    if (policy == 0) {
      float best_score = 0.0f;
      for (int j = lo; j < hi; ++j) {
        for (int h = 0; h < Hk; ++h) tmp[h] = head_scores[((int64_t)s * Hk + h) * max_blocks + j];
        const float sc = head_mean(tmp, Hk);
        if (j == lo || sc < best_score) { /* strict "<": ties stay with the lowest index */
          best = j;
          best_score = sc;
        }
      }
    }
    int32_t* bt = block_table + (int64_t)s * max_blocks;
    evicted_logical_out[s] = best;
    freed_phys_out[s] = bt[best];
    for (int j = best; j + 1 < n; ++j) bt[j] = bt[j + 1];
    bt[n - 1] = -1;
    seq_lens[s] = len - B;
  }
  free(tmp);
  return ORACLE_OK;
}

/* Harness append: the new token's K/V rows of all heads go to slot len % B of the sequence's tail page;
 * when len % B == 0 a page is linked in first (the page freed just before, else the next spare one).
 * freed_phys [S], spare [S][n_spare], spare_used [S]. */
int oracle_sh_append_kv(const float* new_k, const float* new_v /* [S][Hk][D] */, float* k_pool, float* v_pool,
                        int32_t* block_table, int32_t* seq_lens, int32_t* freed_phys, const int32_t* spare,
                        int32_t* spare_used, int n_spare, int S, int Hk, int D, int B, int max_blocks) {
  for (int s = 0; s < S; ++s) {
    const int len = seq_lens[s];
    if (len / B >= max_blocks) return ORACLE_ERR_CAPACITY;
    int32_t* bt = block_table + (int64_t)s * max_blocks;
    if (len % B == 0) {
      int32_t page;
      if (freed_phys[s] >= 0) {
        page = freed_phys[s];
        freed_phys[s] = -1;
      } else {
        if (spare_used[s] >= n_spare) return ORACLE_ERR_CAPACITY;
        page = spare[(int64_t)s * n_spare + spare_used[s]];
        spare_used[s] += 1;
      }
      bt[len / B] = page;
    }
    for (int h = 0; h < Hk; ++h) {
      const int64_t dst = sh_off(bt[len / B], len % B, h, B, Hk, D);
      memcpy(k_pool + dst, new_k + ((int64_t)s * Hk + h) * D, sizeof(float) * (size_t)D);
      memcpy(v_pool + dst, new_v + ((int64_t)s * Hk + h) * D, sizeof(float) * (size_t)D);
    }
    seq_lens[s] = len + 1;
  }
  return ORACLE_OK;
}

/* Eq. 1 through the per-sequence table: query head hq reads head hq / (Hq/Hk) of every cached token.
 * out [S][Hq][D] fp64; weights_sum_out [S][Hq] may be NULL. */
void oracle_sh_paged_decode(const float* q, const float* k_pool, const float* v_pool, const int32_t* block_table,
                            const int32_t* seq_lens, int S, int Hk, int Hq, int D, int B, int max_blocks,
                            double scale, double* out, double* weights_sum_out) {
  const int G = Hq / Hk;
#pragma omp parallel for schedule(dynamic, 1)
  for (int sh = 0; sh < S * Hq; ++sh) {
    const int s = sh / Hq, hq = sh % Hq, g = hq / G;
    const int len = seq_lens[s];
    const float* qv = q + (int64_t)sh * D;
    const int32_t* bt = block_table + (int64_t)s * max_blocks;
    double* o = out + (int64_t)sh * D;
    for (int d = 0; d < D; ++d) o[d] = 0.0;
    if (weights_sum_out) weights_sum_out[sh] = 0.0;
    if (len <= 0) continue;
    double* p = (double*)malloc(sizeof(double) * (size_t)len);
    double m = -INFINITY;
    for (int t = 0; t < len; ++t) {
      const float* kr = k_pool + sh_off(bt[t / B], t % B, g, B, Hk, D);
      double dot = 0.0;
      for (int d = 0; d < D; ++d) dot += (double)qv[d] * (double)kr[d];
      p[t] = scale * dot;
      if (p[t] > m) m = p[t];
    }
    double denom = 0.0;
    for (int t = 0; t < len; ++t) {
      p[t] = exp(p[t] - m);
      denom += p[t];
    }
    double wsum = 0.0;
    for (int t = 0; t < len; ++t) {
      const float* vr = v_pool + sh_off(bt[t / B], t % B, g, B, Hk, D);
      wsum += p[t] / denom;
      for (int d = 0; d < D; ++d) o[d] += p[t] * (double)vr[d];
    }
    for (int d = 0; d < D; ++d) o[d] /= denom;
    if (weights_sum_out) weights_sum_out[sh] = wsum;
    free(p);
  }
}
