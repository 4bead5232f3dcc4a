/*
 * pe.h -- C ABI of libpe: the data-parallel hot path of PagedEviction on one AMD MI355X (gfx950).
 *
 * The path has three parts over a paged KV cache (Sec. 2.4: fixed-size blocks of B tokens, a block
 * table that maps logical to physical blocks):
 *   1. attention-free importance scores from the cached K/V (Alg. 1), one per block;
 *   2. structured eviction: token-level pruning of the prompt to the budget C before it is split
 *      into pages (Alg. 2), then, during decode, dropping the lowest-scoring block of a row whenever
 *      its newest block has filled, and compacting the block table (Alg. 3);
 *   3. the single-query paged attention that reads what is left (Eq. 1; Alg. 3 "PagedAttention").
 *
 * Granularity: every decision is taken per ROW = one (sequence, KV head).  A row owns one row of the
 * block table and its own pages; a page holds B x D elements of K (and a sibling page of V, same
 * physical index in v_pool) of ONE KV head.  Layers are independent: for (1), (2) a caller may fold
 * layers into the sequence dimension.  (This is desc->layout == PE_LAYOUT_PER_HEAD, the default; pe_layout
 * below describes the head-shared alternative and each call states what changes under it.)
 *
 * Conventions that hold for every call below:
 *   - Every pointer except `desc` is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees or synchronises; `stream` is a hipStream_t passed as void* (NULL = the null
 *     stream).  A call enqueues its kernels on `stream` and returns a host-side status at once.
 *   - Tensors are dense, row-major, in the shapes given; K/V/q/out element type is desc->dtype
 *     (PE_F32: IEEE binary32, PE_BF16: bfloat16); tables and lengths are int32.
 *   - Pools: [num_phys_blocks][block_size][head_dim]; page p starts at element p*B*D (head-shared layout:
 *     [num_phys_blocks][block_size][num_kv_heads][head_dim]).
 *   - block_table: [num_seqs][num_kv_heads][max_blocks]; entry j of a row is the physical page of its
 *     logical page j; entries at and beyond ceil(len/B) are -1.  seq_lens: [num_seqs] cached tokens
 *     (the same for all KV heads of a sequence).
 *   - Host-detectable misuse (NULL pointer, unsupported shape, budget not a positive multiple of B,
 *     workspace too small or misaligned) returns a negative status and launches nothing.  A failed
 *     launch returns PE_ERR_HIP.  What the host cannot see without a sync is a CALLER PRECONDITION:
 *     every used table entry lies in [0, num_phys_blocks), rows do not share pages,
 *     seq_lens[s] <= max_blocks*B, and all K/V values are finite.
 *   - Workspaces must be 256-byte aligned.  Calls that share a workspace must be ordered on one stream.
 *     (pe_paged_decode_static keeps its split partials in a static device array of the library instead.)
 */
#ifndef PE_H_
#define PE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PE_OK = 0,
  PE_ERR_INVALID_ARG = -1, /* NULL pointer, inconsistent or non-positive sizes, bad budget */
  PE_ERR_UNSUPPORTED = -2, /* a shape the kernels are not built for (see pe_cache_desc) */
  PE_ERR_WORKSPACE = -3,   /* workspace NULL, misaligned or smaller than pe_workspace_bytes() */
  PE_ERR_HIP = -4          /* the HIP runtime refused a launch */
} pe_status;

typedef enum { PE_F32 = 0, PE_BF16 = 1 } pe_dtype;

typedef enum {
  PE_OP_SCORE_BLOCKS = 0,
  PE_OP_PREFILL_PRUNE = 1,
  PE_OP_EVICT_BLOCKS = 2,
  PE_OP_PAGED_DECODE = 3,
  PE_OP_APPEND_PAGED_DECODE = 4
} pe_op;

/* Cache layout (Sec. 2.4 leaves the granularity open).
 * PE_LAYOUT_PER_HEAD (default): a row is one (sequence, KV head); every row owns a block-table row and its
 *   pages; a page holds [B][D] elements of one head; decisions are per row.
 * PE_LAYOUT_SHARED: the layout of a stock paged cache.  ONE table row per sequence, a page holds
 *   [B][Hk][D] (token slot, head, element), ONE decision per sequence: a token's / page's score is the mean
 *   over the KV heads of the per-head fp32 scores (summed in head order in fp64, rounded once), and the token
 *   / page is dropped for all heads.  Array shapes then lose their Hk dimension where the documentation
 *   below says so ("shared: ...").  pe_score_evict is per-head only (PE_ERR_UNSUPPORTED otherwise). */
typedef enum { PE_LAYOUT_PER_HEAD = 0, PE_LAYOUT_SHARED = 1 } pe_layout;

typedef struct pe_cache_desc {
  int32_t dtype;           /* pe_dtype of q, pools, k_in/v_in, out */
  int32_t num_seqs;        /* S >= 1 */
  int32_t num_kv_heads;    /* Hk >= 1 */
  int32_t num_q_heads;     /* Hq, a multiple of Hk with Hq/Hk <= 8; q head h reads KV head h/(Hq/Hk) */
  int32_t head_dim;        /* D: 64 or 128 */
  int32_t block_size;      /* B: 16, 32, 64 or 128 tokens per page */
  int32_t max_blocks;      /* row stride of block_table and of the score array */
  int64_t num_phys_blocks; /* P: pages in each pool */
  int32_t layout;          /* pe_layout; 0 when the struct is zero- or positionally initialised up to P */
  /* Launch shape of the attention calls (4).  All zero = the library's choice; a caller that tunes sets them
   * per descriptor, so two callers in one process never interfere, and pe_workspace_bytes(), pe_decode_splits()
   * and the launch read the same fields and agree by construction. */
  int32_t decode_splits;   /* 0: chosen from the shape and the device's compute-unit count; 1..256: that many
                              splits of every row (1 = no partials, no workspace) */
  int32_t decode_shape;    /* 0: default; else waves*100 + buffers*10 + loads of the attention workgroup.  Built:
                              422 (default), 424, 432, 822, and only for bf16, D = 128, Hq/Hk = 4, per-head layout;
                              anything else returns PE_ERR_UNSUPPORTED from the attention calls */
  int32_t decode_flat_order; /* 0: workgroup order that keeps the splits of a row on one XCD; 1: plain row-major */
} pe_cache_desc;

/* Bytes of device workspace `op` needs for `desc`.  `total_tokens` is the packed prompt length
 * (sum of L) for PE_OP_PREFILL_PRUNE and ignored otherwise.  Returns 0 for ops that need none and
 * for an invalid desc.  For the attention ops the size follows pe_decode_splits(desc). */
size_t pe_workspace_bytes(int op, const pe_cache_desc* desc, int64_t total_tokens);

/* Static string for a pe_status value. */
const char* pe_status_string(int status);

/* ABI version: major*10000 + minor*100 + patch. */
int pe_version(void);

/* Number of splits of a row the attention calls (4) use for `desc` on the current device: desc->decode_splits
 * when that is set, else enough splits to give every compute unit of the device one workgroup, never shorter
 * than 256 tokens each.  0 for an invalid desc.  (The compute-unit count is read from the HIP runtime once per
 * device; without a device it is taken as 256, an MI355X.) */
int pe_decode_splits(const pe_cache_desc* desc);

/*
 * (1) Block scores -- Alg. 1 (block mode), used by Alg. 3 "Compute Score of Page i"; Sec. 4.3.
 *     For every row and every FULL page j < seq_lens[s]/B:
 *        scores_out[s][hk][j] = (1/B) * sum over the page's B tokens of ||V_i||_2 / ||K_i||_2,
 *     accumulated in fp64 and rounded once to fp32.  Every other entry (partial tail page, unused)
 *     is +INF.  A token with ||V|| = 0 contributes 0; otherwise ||K|| = 0 contributes +INF.
 *     scores_out: [S][Hk][max_blocks] fp32, fully overwritten.  Reads pools/table/lens only.
 *     workspace: none needed (may be NULL / 0).
 *     shared: block_table is [S][max_blocks]; scores_out keeps its shape and holds the per-head page scores
 *     (the head mean is taken where the decision is, in (3)).
 */
int pe_score_blocks(const pe_cache_desc* desc, const void* k_pool, const void* v_pool,
                    const int32_t* block_table, const int32_t* seq_lens, float* scores_out, void* workspace,
                    size_t workspace_bytes, void* stream);

/*
 * (2) Prefill prune -- Alg. 2, the steps after the prompt's own attention: score every prompt token
 *     (S_i = ||V_i||_2/||K_i||_2, fp64, rounded once to fp32), evict the E = max(0, L - C) tokens that
 *     come first in the order (score ascending, index ascending), and write the survivors, in their
 *     original order, into pages: kept token number i of row (s, hk) goes to page
 *     block_table[s][hk][i / B], slot i % B.  seq_lens_out[s] = min(L_s, C).
 *     k_in, v_in: packed prompt [total_tokens][Hk][D] (the layout before paging), read only.
 *     cu_seqlens: [S+1] int32 prefix sums of the prompt lengths, cu_seqlens[S] == total_tokens.
 *     max_seqlen: an upper bound on every L_s (host value, sizes the launch).
 *     budget_tokens: C, a positive multiple of B.
 *     block_table is an INPUT: the caller has put ceil(min(L_s, C)/B) distinct physical pages in each
 *     row (ceil(min(max_seqlen, C)/B) > max_blocks is refused with PE_ERR_INVALID_ARG).  Slots of the tail
 *     page past the kept count are left untouched.
 *     kept_idx_out: NULL, or [S][Hk][budget_tokens] int32 that receives the in-sequence indices of the
 *     kept tokens in ascending order, -1 padded.
 *     workspace: pe_workspace_bytes(PE_OP_PREFILL_PRUNE, desc, total_tokens).
 *     shared: a token's score is the head mean of its per-head fp32 scores, one selection per sequence, the
 *     survivors' rows of all heads go to page block_table[s][i / B], slot i % B; block_table [S][max_blocks],
 *     kept_idx_out [S][budget_tokens].
 */
int pe_prefill_prune(const pe_cache_desc* desc, const void* k_in, const void* v_in, const int32_t* cu_seqlens,
                     int64_t total_tokens, int32_t max_seqlen, int32_t budget_tokens, void* k_pool,
                     void* v_pool, const int32_t* block_table, int32_t* seq_lens_out, int32_t* kept_idx_out,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * (3) Evict -- Alg. 3, "Evict One page with the lowest score" and "Update the KV Cache Block Table".
 *     A sequence s triggers when seq_lens[s] > 0, seq_lens[s] % B == 0 and seq_lens[s] >= budget_tokens
 *     (its newest page has just filled and it is at budget).  Each of its rows removes logical page
 *     j* = the first index that attains min_j scores[s][hk][j] over j < seq_lens[s]/B (ties: lowest
 *     index), shifts the later entries left by one (order kept) and writes -1 into the vacated tail
 *     entry.  evicted_logical_out / freed_phys_out [S][Hk] receive j* / the physical page that was
 *     removed, or -1 for rows that did not evict.  seq_lens[s] -= B, once per triggering sequence.
 *     Exactly one page per row per call.  scores: [S][Hk][max_blocks] fp32 (e.g. from (1)); compared
 *     as fp32 values.  A NaN score never compares lower than another; if every candidate of a row is NaN
 *     (finite K/V never produce one) the row's first candidate page goes, so the call stays inside the row.
 *     block_table and seq_lens are updated in place.  A budget beyond the row capacity max_blocks*B never
 *     triggers.
 *     shared: the sequence's one table row [S][max_blocks] drops the page with the lowest head-mean score
 *     (scores stays [S][Hk][max_blocks]); evicted_logical_out / freed_phys_out are [S].  The same holds for
 *     the variants below (share_heads is then implied).
 */
int pe_evict_blocks(const pe_cache_desc* desc, const float* scores, int32_t* block_table, int32_t* seq_lens,
                    int32_t budget_tokens, int32_t* evicted_logical_out, int32_t* freed_phys_out, void* stream);

/*
 * Cached page scores (an optimisation of (1)+(3), not the paper's stated procedure, which re-scores every
 * page on every trigger; Sec. 3 "computed on-the-fly"): a full page's tokens never change, so neither
 * does its score.  A caller may keep scores[S][Hk][max_blocks] alive across steps:
 *   - pe_score_recent_blocks computes only the `recent` >= 1 most recently filled pages of every row,
 *     j in [max(0, seq_lens[s]/B - recent), seq_lens[s]/B), and leaves every other entry untouched;
 *   - pe_evict_blocks_cached is pe_evict_blocks that also deletes entry j* from the score row (later
 *     scores shift left with the table, the vacated tail entry becomes +INF).
 * Starting from a pe_score_blocks call (which also sets the +INF entries), the array then always equals
 * what pe_score_blocks would return, and the decisions are the same.
 */
int pe_score_recent_blocks(const pe_cache_desc* desc, const void* k_pool, const void* v_pool,
                           const int32_t* block_table, const int32_t* seq_lens, int32_t recent,
                           float* scores_inout, void* stream);
int pe_evict_blocks_cached(const pe_cache_desc* desc, float* scores_inout, int32_t* block_table, int32_t* seq_lens,
                           int32_t budget_tokens, int32_t* evicted_logical_out, int32_t* freed_phys_out,
                           void* stream);

/*
 * (1) restricted to the sequences that (3) will act on: Alg. 3 scores pages only inside its "L % B == 0"
 * branch, i.e. for a sequence whose newest page has just filled and which is at budget.  (Alg. 3 lists the
 * budget C among its inputs but its printed trigger is only "L % B == 0"; here and in (3) the trigger is gated on
 * seq_lens[s] >= C, so that a budget >= context reproduces full attention: Sec. 4.3, Alg. 3.)
 * Rows of sequences that do not trigger at `budget_tokens` are neither read nor written (their entries of
 * scores_inout keep whatever they held); rows of triggering sequences are written exactly as by (1).  With
 * sequences that reach a page boundary at different steps this reads a fraction of what (1) reads.
 */
int pe_score_triggered_blocks(const pe_cache_desc* desc, const void* k_pool, const void* v_pool,
                              const int32_t* block_table, const int32_t* seq_lens, int32_t budget_tokens,
                              float* scores_inout, void* stream);

/*
 * (1)+(3) in one pass over the pages -- the whole "if L % B == 0" branch of Alg. 3.  Equal in effect to
 * pe_score_blocks followed by pe_evict_blocks, except that only triggering sequences are scored: their rows' pages
 * are swept once (one workgroup per row, so a few evicting sequences use the chip as well as a whole batch), the
 * running minimum is kept (ties: lowest index), the table row is compacted, and a second, tiny launch behind the
 * sweep sets seq_lens[s] -= B (every row of a sequence has to see the length from before the eviction).  No score
 * array travels through memory unless asked for.
 * scores_out: NULL, or [S][Hk][max_blocks] fp32; rows of triggering sequences receive the scores the decision
 * was taken on (before compaction; entries j >= seq_lens[s]/B are +INF), rows of other sequences are left
 * untouched.  evicted_logical_out / freed_phys_out as in (3).
 */
int pe_score_evict(const pe_cache_desc* desc, const void* k_pool, const void* v_pool, int32_t* block_table,
                   int32_t* seq_lens, int32_t budget_tokens, float* scores_out, int32_t* evicted_logical_out,
                   int32_t* freed_phys_out, void* stream);

/*
 * Eviction variants on the same table machinery (not the paper's main method).  Sec. 5.2 / App. A describe
 * StreamingLLM (a few first tokens kept as attention sinks plus a window of the most recent ones); Sec. 2.4
 * leaves open whether heads decide separately.  opts->policy: PE_POLICY_LOWEST_SCORE (as (3)) or
 * PE_POLICY_OLDEST (the oldest unprotected page goes; `scores` may be NULL).  protect_first / protect_last:
 * pages at the start / end of a row that are never candidates.  Candidates are logical pages lo .. hi-1 with
 * lo = min(protect_first, n-1), hi = max(n - protect_last, lo + 1): protection yields before the budget
 * does.  share_heads != 0: one decision per sequence; the page score is the mean over the sequence's KV
 * heads of the fp32 page scores (summed in head order in fp64, rounded once) and every head drops the same
 * logical page.  cached_scores != 0: `scores` is in/out and entry j* is deleted from each score row as in
 * pe_evict_blocks_cached.  Trigger, tie-break (lowest index), outputs and in-place updates are as in (3).
 */
typedef enum { PE_POLICY_LOWEST_SCORE = 0, PE_POLICY_OLDEST = 1 } pe_evict_policy;
typedef struct pe_evict_opts {
  int32_t policy;
  int32_t protect_first;
  int32_t protect_last;
  int32_t share_heads;
  int32_t cached_scores;
} pe_evict_opts;
int pe_evict_blocks_ex(const pe_cache_desc* desc, const pe_evict_opts* opts, float* scores, int32_t* block_table,
                       int32_t* seq_lens, int32_t budget_tokens, int32_t* evicted_logical_out,
                       int32_t* freed_phys_out, void* stream);

/*
 * (4) Paged decode attention -- Eq. 1 for one new query per sequence; Alg. 3 "PagedAttention(Q,K,V)".
 *     out[s][h][:] = sum_t softmax_t(softmax_scale * <q[s][h], K_t>) V_t over the seq_lens[s] tokens of
 *     row (s, h / (Hq/Hk)), token t being slot t % B of page block_table[s][hk][t / B].
 *     fp32 accumulation, output rounded to desc->dtype.  seq_lens[s] == 0 gives zeros.
 *     q, out: [S][Hq][D].  workspace: pe_workspace_bytes(PE_OP_PAGED_DECODE, desc, 0) (split partials).
 *     shared: block_table [S][max_blocks]; query head h reads head h/(Hq/Hk) of the sequence's pages.
 */
int pe_paged_decode(const pe_cache_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                    const int32_t* block_table, const int32_t* seq_lens, float softmax_scale, void* out,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * (4) for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as pe_paged_decode, but
 * the split partials live in a static device array inside the library (PE_STATIC_SCRATCH_BYTES per GPU, held
 * until the process ends) instead of a caller workspace.  The call allocates and frees nothing.  A shape whose
 * partials, pe_workspace_bytes(PE_OP_PAGED_DECODE, desc, 0), exceed PE_STATIC_SCRATCH_BYTES is refused with
 * PE_ERR_WORKSPACE and nothing is launched (lower desc->decode_splits, or use pe_paged_decode).  The first call
 * on a device looks the array's address up once (hipGetSymbolAddress; make that call outside stream capture).
 * All calls on one GPU share the one array: calls that overlap in time on the same GPU (different streams) race;
 * order them on one stream.  Nothing needs clearing between calls: every record the merge reads is written by
 * the same call's attention kernel.
 */
#define PE_STATIC_SCRATCH_BYTES (8 * 1024 * 1024)
int pe_paged_decode_static(const pe_cache_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                           const int32_t* block_table, const int32_t* seq_lens, float softmax_scale, void* out,
                           void* stream);

/*
 * Harness convenience (not part of the paper's method): the step between (3) and (4) in a decode
 * iteration.  Writes the new token's K/V row of every (s, hk) into slot seq_lens[s] % B of the tail
 * page.  When seq_lens[s] % B == 0 a new page is linked in at logical index seq_lens[s]/B: the page
 * the row freed in the eviction just before (freed_phys[s][hk] >= 0; consumed, reset to -1), else
 * spare[s][hk][spare_used[s][hk]++].  Then seq_lens[s] += 1.
 * new_k, new_v: [S][Hk][D].  spare: [S][Hk][n_spare] int32.  spare_used, freed_phys: [S][Hk] int32,
 * updated in place.  Preconditions: seq_lens[s] < max_blocks*B; the spare list is not exhausted.
 * shared: one page per sequence takes the rows of all heads; spare [S][n_spare], spare_used and freed_phys [S].
 */
int pe_append_kv(const pe_cache_desc* desc, const void* new_k, const void* new_v, void* k_pool, void* v_pool,
                 int32_t* block_table, int32_t* seq_lens, int32_t* freed_phys, const int32_t* spare,
                 int32_t* spare_used, int32_t n_spare, void* stream);

/*
 * The two calls above in ONE launch: the effect of pe_append_kv followed by pe_paged_decode (Alg. 3: the
 * new token joins the cache, then "PagedAttention(Q,K,V)" over everything cached), i.e. attention over
 * the seq_lens[s] cached tokens plus the new token, the new K/V rows stored into the tail page (a new
 * page linked in first when seq_lens[s] % B == 0).  The new rows are attended to from registers instead
 * of being read back from the pool.  seq_lens is only read; the new lengths seq_lens[s] + 1 are written
 * to seq_lens_out [S], which must not alias seq_lens (callers keep two arrays and swap them), so that no
 * workgroup of the launch can observe a length that another one has already bumped.
 * workspace: pe_workspace_bytes(PE_OP_APPEND_PAGED_DECODE, desc, 0).
 * shared: same contract and shapes as pe_append_kv / pe_paged_decode in that layout, carried out as two launches
 * (one workgroup per sequence does the page bookkeeping for all heads before the attention reads it).
 */
int pe_append_paged_decode(const pe_cache_desc* desc, const void* new_k, const void* new_v, const void* q,
                           void* k_pool, void* v_pool, int32_t* block_table, const int32_t* seq_lens,
                           int32_t* seq_lens_out, int32_t* freed_phys, const int32_t* spare, int32_t* spare_used,
                           int32_t n_spare, float softmax_scale, void* out, void* workspace, size_t workspace_bytes,
                           void* stream);

/*
 * The call above for `num_layers` layers that share one pool, issued from native code in layer order on `stream`
 * (a host-side loop, nothing more: layer l+1's launch follows layer l's on the stream, as the layers of a model
 * do).  `desc` describes ONE layer (num_seqs = S).  Per-layer arrays are stacked along their first axis, layers
 * folded into the sequence dimension: new_k, new_v [layers*S][Hk][D]; q, out [layers*S][Hq][D]; block_table
 * [layers*S][Hk][max_blocks]; seq_lens, seq_lens_out [layers*S]; freed_phys, spare_used [layers*S][Hk]; spare
 * [layers*S][Hk][n_spare] (shared layout: the shapes that layout gives, stacked the same way).  The one workspace
 * (pe_workspace_bytes(PE_OP_APPEND_PAGED_DECODE, desc, 0)) serves every layer.  Returns the first non-OK status;
 * layers before it have been enqueued.
 */
int pe_append_paged_decode_layers(const pe_cache_desc* desc, int32_t num_layers, const void* new_k, const void* new_v,
                                  const void* q, void* k_pool, void* v_pool, int32_t* block_table,
                                  const int32_t* seq_lens, int32_t* seq_lens_out, int32_t* freed_phys,
                                  const int32_t* spare, int32_t* spare_used, int32_t n_spare, float softmax_scale,
                                  void* out, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PE_H_ */
