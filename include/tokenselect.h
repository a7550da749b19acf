/*
 * tokenselect.h -- C ABI of the MI355X (gfx950) TokenSelect hot path.
 *
 * One decode step of one attention layer (Fig. 4; Algorithm 1) is five calls on one HIP stream:
 *
 *   ts_selcache_check     Algorithm 1, the condition and the C_Q / first-flag update
 *   ts_paged_qk_scores    Algorithm 2 (Paged Dot Product Kernel) + per-head softmax statistics
 *   ts_soft_vote          Eq. 5, per-head softmax over tokens summed over heads
 *   ts_topk               the TopK of Eq. 5 (radix select, ties to the lower token index)
 *   ts_sparse_paged_attn  Eq. 2, attention over the selected tokens read through the page table
 *
 * (ts_paged_qk_scores_checked / ts_paged_qk_codes_checked take Algorithm 1's condition inside the score launch,
 * which makes the first call unnecessary.)
 * With forced tokens (ts_problem.num_initial / num_local) the same five calls rank only the middle of
 * each sequence and attend over initial block + selection + most recent block.
 * A chunk of C > 1 queries (chunked prefill) uses ts_chunk_row_stats + ts_chunk_soft_vote (or
 * ts_chunk_mean_query + the decode calls), ts_topk and ts_sparse_paged_attn with chunk = C.
 *
 * Conventions
 *   - Every pointer marked [device] is caller-owned device memory; [host] is host memory.
 *     The library never allocates, frees, synchronises the stream or reads device memory on the
 *     host.  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Every function returns TS_OK (0) or a negative ts_status.  Argument errors are detected on
 *     the host before anything is launched; nothing has been written in that case.
 *   - Inputs containing NaN/Inf give unspecified results, but no fault: count[b] stays within [0, min(k, N_b)] and
 *     every idx entry is a token of the sequence or -1.
 *   - Sequences whose skip[b] byte is non-zero are left untouched by the three selection calls
 *     (their previous idx / count stay valid: Algorithm 1's "I <- C_I" branch).
 *   - Calls that share a workspace must not overlap in time (one stream, or ordered streams).  Calls on different
 *     workspaces and different output buffers may overlap on different streams (they may share the pools, the page
 *     table and the query): the library keeps no state of its own between calls besides the ts_debug_* knobs.
 *
 * Paged KV layout (the paper's K in R^{N_kv x H_kv x D} with index list I, Algorithm 2, grouped in
 * pages): pool[num_pages][page_size][H_kv][D]; logical token t of sequence b lives in physical slot
 * page_indices[page_indptr[b] + t / page_size] * page_size + t % page_size.
 * GQA: query head h reads KV head h / (H / H_kv).
 */
#ifndef TOKENSELECT_H_
#define TOKENSELECT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ts_status {
  TS_OK = 0,
  TS_ERR_INVALID_ARG = -1, /* NULL pointer, non-positive size, H % H_kv != 0, k <= 0, ...         */
  TS_ERR_UNSUPPORTED = -2, /* shape / dtype / page size outside what the kernels are built for    */
  TS_ERR_WORKSPACE = -3,   /* workspace missing or smaller than ts_workspace_bytes()              */
  TS_ERR_HIP = -4          /* a HIP launch reported an error                                      */
} ts_status;

typedef enum ts_dtype { TS_F32 = 0, TS_BF16 = 1 } ts_dtype;

/* Shape and paged-pool description shared by all calls.  Passed by const pointer [host]. */
typedef struct ts_problem {
  int32_t batch;        /* B  in [1, 65535]                                                      */
  int32_t chunk;        /* C  queries per sequence; 1 = decode                                   */
  int32_t num_q_heads;  /* H  (<= 128)                                                           */
  int32_t num_kv_heads; /* H_kv, a power of two, H % H_kv == 0, H / H_kv <= 8                    */
  int32_t head_dim;     /* D  in {64, 128}                                                       */
  int32_t page_size;    /* P  a power of two with P * min(H_kv, 8) % 8 == 0 (16 in the configs)   */
  int32_t max_seq_len;  /* host-known upper bound on every seq_lens[b]; also the token extent of   */
                        /* scores[B][max_seq_len][H] and votes[B][max_seq_len]                    */
  int32_t dtype;        /* ts_dtype of q, k_pool, v_pool, cached_q and out                        */
  const void* k_pool;   /* [device] [num_pages][P][H_kv][D]                                      */
  const void* v_pool;   /* [device] same layout (may be NULL for calls that do not read V)        */
  const int32_t* page_indptr;  /* [device] [B+1] CSR offsets into page_indices                    */
  const int32_t* page_indices; /* [device] physical page ids in logical order                     */
  const int32_t* seq_lens;     /* [device] [B] cached tokens N_b (0 <= N_b <= max_seq_len)        */
  /* Forced tokens (Sec. 6.1, implementation details: 128 initial and n_local most recent tokens are
   * attended in addition to the k selected ones).  With lo_b = min(num_initial, N_b) and
   * hi_b = max(lo_b, N_b - num_local), the selection function is applied to the ranked range
   * [lo_b, hi_b) only: the softmax statistics of ts_paged_qk_scores / ts_soft_vote cover that range,
   * votes outside it are 0, ts_topk returns min(k, hi_b - lo_b) tokens of it, and ts_sparse_paged_attn
   * attends over tokens [0, lo_b), the selected ones, and [hi_b, N_b) of the *current* N_b (a cached
   * selection made at a smaller N_b stays valid).  Both 0 = no forced tokens.
   * Chunk form (chunk = C > 1): the blocks are taken from the N_b - C cached tokens before the chunk -- the first
   * num_initial of them and the num_local just before the chunk -- and are attended by every query of the chunk;
   * ts_chunk_row_stats / ts_chunk_soft_vote / ts_topk rank the cached tokens between them. */
  int32_t num_initial;
  int32_t num_local;
} ts_problem;

/* Library version (major*10000 + minor*100 + patch).  Host only. */
int32_t ts_version(void);

/* Static string for a ts_status value.  Host only. */
const char* ts_strerror(int32_t status);

/* Bytes of device workspace that the calls below need for this problem when selecting at most
 * `k` tokens.  One workspace serves all calls of a step.  [host] out.
 * Decode (chunk == 1): ts_sparse_paged_attn attends over at most 32768 tokens, so
 * k + num_initial + num_local > 32768 is TS_ERR_UNSUPPORTED here already (and in ts_sparse_paged_attn). */
int32_t ts_workspace_bytes(const ts_problem* p, int32_t k, size_t* bytes);

/* Clears a fresh workspace (launches a fill kernel on `stream`; safe under graph capture).  Must
 * run once before the first use of a workspace; the kernels leave it ready for the next call.
 * The radix-select histograms inside it must be zero when a selection starts and are zeroed again by the last
 * kernel of every ts_topk / ts_topk_exact / ts_head_vote call.  If one of those calls (or ts_soft_vote_bounds) returns
 * an error after it has launched part of its kernels, or a stream is torn down between its launches, the
 * workspace is in an undefined state: call ts_workspace_init again before reusing it.  The call zeroes every
 * byte, so the next selection must start with its score pass (which it does anyway). */
int32_t ts_workspace_init(void* ws, size_t ws_bytes, void* stream);

/* Algorithm 2 (Paged Dot Product Kernel).  For every sequence b, head h, cached token t < N_b:
 *   scores[b][t][h] = < q[b][0][h][:], K[slot(b,t)][h / G][:] >          (raw, unscaled; the matrix
 *   S of Algorithm 2 stored token-major so that it streams out in contiguous bursts)
 * and, feeding Eq. 5, per-workgroup partial softmax statistics (running max and sum of
 * exp(score_scale * (score - max)) per head) are left in the workspace for ts_soft_vote.
 * q [device] [B][C][H][D]; scores [device] float [B][max_seq_len][H] (rows t >= N_b untouched);
 * score_scale >= 0 (Eq. 5 as printed uses 1).  One kernel launch.
 * Decode only: chunk must be 1 (TS_ERR_UNSUPPORTED otherwise). */
int32_t ts_paged_qk_scores(const ts_problem* p, const void* q, float* scores, float score_scale,
                           const uint8_t* skip /* [device] [B] or NULL */, void* ws, size_t ws_bytes, void* stream);

/* Eq. 5 (head soft vote).  First merges the partial statistics that the preceding
 * ts_paged_qk_scores call (same problem, same workspace, same score_scale) left behind into
 *   row_stats[b][h][0] = max_t scores[b][t][h]
 *   row_stats[b][h][1] = sum_t exp(score_scale * (scores[b][t][h] - max))
 * then computes
 *   votes[b][t] = sum_h exp(score_scale*(scores[b][t][h] - max_h)) / sumexp_h        for t < N_b
 * (difference, scaling and argument reduction in double precision, the fractional power of two by the
 * float hardware exponential, the sum over heads in double, rounded once to float: about 1e-7 relative).
 * With forced tokens the statistics and the votes cover the ranked range only; votes outside it are 0.
 * row_stats [device] float [B][H][2] out; votes [device] float [B][max_seq_len] (entries t >= N_b
 * untouched). */
int32_t ts_soft_vote(const ts_problem* p, const float* scores, float score_scale, float* row_stats, float* votes,
                     const uint8_t* skip, void* ws, size_t ws_bytes, void* stream);

/* Eq. 5 and the start of the TopK in one launch: ts_soft_vote that also counts, while the votes are in registers,
 * the histogram of their top 11 key bits -- the first pass of ts_topk's radix select (one launch less per decode
 * step).  Same arguments, same row_stats and votes as ts_soft_vote, bit for bit.
 * Contract: the histogram lives in ws until a ts_topk call with TS_TOPK_VOTE_HIST, the same votes, skip mask and ws
 * consumes and clears it; that call must be the next selection call on ws (ts_soft_vote_bounds / ts_topk_exact share
 * the section).  After a call that was not followed that way, ts_workspace_init restores the workspace. */
int32_t ts_soft_vote_ranked(const ts_problem* p, const float* scores, float score_scale, float* row_stats,
                            float* votes, const uint8_t* skip, void* ws, size_t ws_bytes, void* stream);

/* TopK of Eq. 3-5 over votes[b][0..N_b): the min(k, N_b) largest values, equal values taken in
 * order of increasing token index, written as ascending logical token ids.
 * idx [device] int32 [B][k] (slots past the count are set to -1); count [device] int32 [B].
 * -0.0 compares equal to +0.0.
 * flags: 0, or TS_TOPK_FLAT_VOTES.  By default (decode) the radix select runs as three launches whose last one
 * finishes each sequence on one workgroup: fast when few votes lie within a quarter octave of the k-th vote, as
 * with the peaked votes of Eq. 5, and slow (still exact) when most do.  TS_TOPK_FLAT_VOTES selects the five-launch
 * form whose time does not depend on the distribution; chunk problems (chunk > 1) always use it.
 * TS_TOPK_VOTE_HIST: the votes were written by ts_soft_vote_ranked, which left the radix select's first histogram in
 * ws (see there): the pass that builds it is skipped (decode only; not for ts_topk_noalloc). */
#define TS_TOPK_FLAT_VOTES 1
#define TS_TOPK_VOTE_HIST 2
int32_t ts_topk(const ts_problem* p, const float* votes, int32_t k, int32_t* idx, int32_t* count,
                const uint8_t* skip, int32_t flags, void* ws, size_t ws_bytes, void* stream);

/* ts_topk for callers that cannot allocate or bring a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same result as ts_topk, but the radix select's
 * histograms, state words, chunk counts and candidate list live in a device array that is part of the library
 * image (about 4.4 MiB per GPU, held until the process ends) instead of a caller workspace.  The call allocates
 * nothing and frees nothing.
 * Limits: batch <= 16 and batch * ceil(max_seq_len / 2048) <= 256 (524288 tokens over the batch), else
 * TS_ERR_UNSUPPORTED before anything is launched.  Every call on a GPU shares that GPU's array: calls that
 * overlap in time on one GPU (different streams, different threads) race; the histograms are cleared at the
 * start of every call, so a call that was abandoned half way does not disturb the next one. */
int32_t ts_topk_noalloc(const ts_problem* p, const float* votes, int32_t k, int32_t* idx, int32_t* count,
                        const uint8_t* skip, int32_t flags, void* stream);

/* ---- Compact form of the selection (decode, chunk == 1): Algorithm 2, Eq. 5 and the TopK with the same result
 * as ts_paged_qk_scores + ts_soft_vote + ts_topk (up to tokens whose votes differ from the k-th vote by less than
 * the float scores' own rounding, about 1e-5 relative), without the score matrix S ever reaching memory.  On this
 * machine a write stream mixed into the K read stream costs several times its bytes, and S is 4*H bytes per
 * token; the compact form writes H bytes per token and makes up for the lost precision by re-evaluating the few
 * tokens that can still be among the k largest.
 *
 * ts_paged_qk_codes    Algorithm 2.  The scores (float accumulation of exact products; on the matrix cores for bf16
 *                      where the shape allows, else with the arithmetic of ts_paged_qk_scores) leave as
 *                      codes[b][t][h] = clamp(255 + ceil(4 * c2 * (s - M)), 0, 255), where c2 = score_scale * log2(e)
 *                      and M is the maximum of head h over the ranked tokens of the token's block (32 consecutive
 *                      tokens, aligned): the distance below the block maximum in quarter octaves of softmax weight,
 *                      rounded towards the maximum; 0 also stands for everything 63.75 octaves or more below it.
 *                      The block maxima and per-workgroup softmax statistics go to the workspace.
 * ts_soft_vote_bounds  Eq. 5.  Merges the block statistics into row_stats (as ts_soft_vote defines it) and gives
 *                      every ranked token an interval that contains its vote as ts_soft_vote would compute it:
 *                      vote_lo[b][t] <= votes[b][t] <= vote_hi[b][t], vote_hi / vote_lo about 2^(1/4); both 0
 *                      outside the ranked range.  Must follow ts_paged_qk_codes with the same problem, workspace
 *                      and score_scale.
 * ts_topk_exact        The TopK of Eq. 5.  Every token whose upper bound reaches the k-th largest lower bound
 *                      (a superset of the k largest votes; usually 1.1-1.5 k tokens) has its scores recomputed
 *                      from K (exact products, double accumulation: closer to Eq. 5 than the float scores of the score
 *                      pass) and its vote evaluated with the arithmetic of ts_soft_vote;
 *                      the k largest of those votes are returned exactly as ts_topk returns them (ties to the
 *                      lower token index, ascending token ids, unused slots -1); sel_votes [device] float [B][k],
 *                      if not NULL, receives the vote of idx[b][j] at [b][j] (0 in unused slots).  Must follow
 *                      ts_soft_vote_bounds with the same problem, workspace, q and score_scale.  Two launches.
 * codes [device] uint8 [B][max_seq_len][H]; vote_hi, vote_lo [device] float [B][max_seq_len] (vote_lo may be NULL:
 * ts_topk_exact needs the upper bounds only, the lower ones live on in the workspace as a histogram); the other arguments
 * as for the three calls they stand in for.  Sequences with skip[b] != 0 are left untouched.  The cost of
 * ts_topk_exact grows with the number of candidates: flat votes (a small score_scale) give more of them, never a
 * wrong result. */
int32_t ts_paged_qk_codes(const ts_problem* p, const void* q, uint8_t* codes, float score_scale,
                          const uint8_t* skip, void* ws, size_t ws_bytes, void* stream);
int32_t ts_soft_vote_bounds(const ts_problem* p, const uint8_t* codes, float score_scale, float* row_stats,
                            float* vote_hi, float* vote_lo, const uint8_t* skip, void* ws, size_t ws_bytes, void* stream);
int32_t ts_topk_exact(const ts_problem* p, const void* q, const float* vote_hi, const float* row_stats,
                      float score_scale, int32_t k, int32_t* idx, int32_t* count, float* sel_votes, const uint8_t* skip,
                      void* ws, size_t ws_bytes, void* stream);

/* The two selection functions the paper ablates against Eq. 5 (Sec. 5.1), as other ways to fill `votes`
 * from the scores of ts_paged_qk_scores; ts_topk then ranks them as usual (decode only, chunk == 1).
 *
 * ts_sum_vote   Eq. 3 (I_topk), read as the top-k of the dot products summed over the heads:
 *                 votes[b][t] = sum_h scores[b][t][h]      (double accumulation in head order, rounded once)
 * ts_head_vote  Eq. 4 (I_head-vote): every head takes the k_head largest of its own dot products (equal values
 *               in order of increasing token index) and
 *                 votes[b][t] = number of heads that took token t     (an integer 0..H stored as float)
 * Votes outside the ranked range (forced tokens) are 0; sequences with skip[b] != 0 are left untouched.
 * ts_head_vote needs its own scratch of ts_head_vote_scratch_bytes() bytes [device], 256-byte aligned,
 * contents irrelevant on entry (a transposed copy of the scores plus B * H radix-select states). */
int32_t ts_sum_vote(const ts_problem* p, const float* scores, float* votes, const uint8_t* skip, void* stream);
int32_t ts_head_vote_scratch_bytes(const ts_problem* p, size_t* bytes);
int32_t ts_head_vote(const ts_problem* p, const float* scores, int32_t k_head, float* votes, const uint8_t* skip,
                     void* scratch, size_t scratch_bytes, void* stream);

/* Algorithm 1 (Selection Cache), condition and state update, per sequence b:
 *   reuse[b] = (first[b] == 0) and cos(q[b], cached_q[b]) >= theta      (one cosine over H*D values,
 *   double precision; a zero-norm operand gives cos = 0)
 *   on a miss: cached_q[b] <- q[b], first[b] <- 0.
 * Passing reuse as `skip` to the three calls above and keeping idx/count as the cached C_I gives
 * the whole algorithm.  q, cached_q [device] [B][H][D] in p->dtype (chunk must be 1);
 * first [device] uint8 [B] in/out; reuse [device] uint8 [B] out. */
int32_t ts_selcache_check(const ts_problem* p, const void* q, void* cached_q, uint8_t* first, float theta,
                          uint8_t* reuse, void* stream);

/* Algorithm 1's test inside the score launch (one launch less per decode step): ts_paged_qk_scores_checked and
 * ts_paged_qk_codes_checked are ts_paged_qk_scores / ts_paged_qk_codes with the condition of ts_selcache_check
 * evaluated in the prologue of every workgroup — the same sums in the same order, hence the same decision as
 * ts_selcache_check, bit for bit — instead of a `skip` mask.  Sequences whose test passes are skipped; workgroup 0
 * of every sequence writes the state after the step.  Because other workgroups of the launch still read the state
 * before the step, the two live in different buffers: the caller keeps two (cached_q, first) pairs and swaps them
 * after every step.
 *   reuse[b]         = (first[b] == 0) and cos(q[b], cached_q[b]) >= theta        (out; pass it as `skip` to the
 *                      calls that follow in the step)
 *   cached_q_next[b] = reuse[b] ? cached_q[b] : q[b];   first_next[b] = reuse[b] ? first[b] : 0
 * cached_q, cached_q_next [device] [B][H][D] in p->dtype, 16-byte aligned, not overlapping; first, first_next,
 * reuse [device] uint8 [B], first_next not overlapping first.  Errors as for the plain calls; a null or
 * overlapping member of sc is TS_ERR_INVALID_ARG. */
typedef struct {
  const void*    cached_q;
  void*          cached_q_next;
  const uint8_t* first;
  uint8_t*       first_next;
  uint8_t*       reuse;
  float          theta;
} ts_selcache;
int32_t ts_paged_qk_scores_checked(const ts_problem* p, const void* q, const ts_selcache* sc, float* scores,
                                   float score_scale, void* ws, size_t ws_bytes, void* stream);
int32_t ts_paged_qk_codes_checked(const ts_problem* p, const void* q, const ts_selcache* sc, uint8_t* codes,
                                  float score_scale, void* ws, size_t ws_bytes, void* stream);

/* Eq. 2 (selective sparse attention), decode form (chunk == 1): for every b, h
 *   out[b][0][h][:] = sum_j softmax_j( <q[b][0][h], K[slot(b, idx[b][j])][h/G]> * sm_scale ) * V[slot(b, idx[b][j])][h/G]
 * over j < count[b]; float accumulation, result rounded to p->dtype.  idx [device] int32 [B][k]
 * (logical token ids, k = idx_stride); count [device] int32 [B]; out [device] [B][C][H][D];
 * lse [device] float [B][C][H] or NULL (log-sum-exp of the scaled logits).  count[b] == 0 gives
 * out = 0 and lse = -inf.  idx and count are read defensively (they may be a cached selection of an earlier step):
 * token ids are clamped into [0, N_b), count[b] into [0, k], and a sequence with N_b == 0 attends nothing whatever its
 * count says.  The page table itself is trusted: every page id of a sequence must lie inside the pools.
 * Chunk form (chunk = C > 1, bf16): query c of the chunk (logical token N_b - C + c) attends over the
 * count[b] selected tokens and the chunk's own tokens 0..c in one joint softmax (Eq. 2's
 * [K_select, K_current] with a causal mask inside the chunk); the weights that multiply V are rounded
 * to bf16 (matrix-core operand).  A sequence with N_b < C holds no chunk (an idle slot of the batch): its rows of
 * out are zero, its lse -inf, and nothing is read through its page table (the selection calls give it count 0). */
int32_t ts_sparse_paged_attn(const ts_problem* p, const void* q, const int32_t* idx, int32_t idx_stride,
                             const int32_t* count, float sm_scale, void* out, float* lse, void* ws,
                             size_t ws_bytes, void* stream);

/* ---- Chunked prefill (chunk = C > 1, bf16): the C queries of a chunk are the last C tokens of their
 * sequence (seq_lens counts them); selection looks at the N_b - C cached tokens before them.
 * Sec. 5.2 selects once per chunk; here every query of the chunk votes (Eq. 5 per query) and the
 * votes are summed over heads and over the chunk's queries:
 *   votes[b][t] = sum_{c < C} sum_h softmax_t(score_scale * <q[b][c][h], K[t][h/G]>)[t],  t < N_b - C.
 * The score matrix is computed on the matrix cores (MFMA) and never stored: two sweeps over K.
 *
 * ts_chunk_row_stats  sweep 1: row_stats[b][c][h] = L = log2 sum_t 2^(score_scale * log2(e) * s), the base-2
 *                     log-sum-exp of the row, stored as a (high, low) float pair with high + low = L.
 * ts_chunk_soft_vote  sweep 2: votes as above from the same q, row_stats and score_scale.
 * ts_topk with the same problem (chunk > 1) then ranks only the N_b - C cached tokens.
 * q [device] [B][C][H][D]; row_stats [device] float [B][C][H][2]; votes [device] float [B][max_seq_len]
 * (entries t >= N_b - C untouched).  fp32 inputs: TS_ERR_UNSUPPORTED. */
int32_t ts_chunk_row_stats(const ts_problem* p, const void* q, float score_scale, float* row_stats, void* ws,
                           size_t ws_bytes, void* stream);
int32_t ts_chunk_soft_vote(const ts_problem* p, const void* q, const float* row_stats, float score_scale, float* votes,
                           void* ws, size_t ws_bytes, void* stream);

/* Sec. 5.2 as printed (chunk-wise selection with one query per chunk): q_mean[b][0][h][:] = mean over the
 * chunk's C queries of q[b][c][h][:], formed exactly, rounded to float and then to bf16 (nearest-even).
 * The result is a decode query: feed it to ts_paged_qk_scores / ts_soft_vote / ts_topk with a chunk == 1
 * problem over the same pool whose seq_lens hold the cached lengths N_b - C, then attend with the chunk
 * problem.  q [device] [B][C][H][D] bf16; q_mean [device] [B][1][H][D] bf16.  fp32: TS_ERR_UNSUPPORTED. */
int32_t ts_chunk_mean_query(const ts_problem* p, const void* q, void* q_mean, void* stream);

/* ======================================================================================================
 * Everything below is for benchmarks and tests, not for serving code: process-wide tuning knobs and timing
 * helpers.  They are not thread-safe and must not be changed while a call on another thread is between
 * its argument checks and its launches.  No result depends on them: what a later call of a step needs to know
 * about an earlier launch (how many statistics partials it left) travels through the workspace, so a knob that
 * changes between two calls of one step does not change the step's result.
 * ====================================================================================================== */

/* Tuning knob for benchmarks and tests (process-wide, not thread-safe, not part of the method):
 * variant 0 = score pass with fma arithmetic, 1 = packed bf16 dot2 arithmetic (bf16 inputs only),
 * 2 = the matrix-core kernel for the shapes it covers (bf16, 3 to 8 query heads per KV head; elsewhere as 1): the
 * default;
 * wg = workgroups per sequence in the score pass, 0 = automatic;
 * run_tiles = 32-token tiles a wave stages in LDS before it writes their scores as one run: 1, 2, 4,
 * or 0 = automatic (longer runs for longer sequences).  Results do not depend on wg or run_tiles.
 * Host only. */
int32_t ts_debug_set_score_variant(int32_t variant, int32_t wg, int32_t run_tiles);

/* Tuning knob (process-wide, tests and benchmarks): mfma = 1 (default) lets ts_paged_qk_codes run on the matrix
 * cores where the shape allows (bf16; 3-4 query heads per KV head with at least 8 KV heads, or 5-8 with exactly 4),
 * 0 forces the vector form; run_tiles = 32-token tiles whose bytes a wave collects before writing them (1..8),
 * 0 = automatic.  The bytes and the selection do not depend on either.  Host only. */
int32_t ts_debug_set_codes_path(int32_t mfma, int32_t run_tiles);

/* Tuning knob (process-wide, tests and benchmarks): five_pass = 1 makes ts_topk / ts_head_vote use the
 * five-pass radix select (three global histogram passes, count, emit) that otherwise only serves sequences
 * beyond 16 Mi tokens; 0 (default) = histogram pass, compaction of the candidates, one finishing workgroup
 * per sequence.  Both give the same result.  Host only. */
int32_t ts_debug_set_topk_path(int32_t five_pass);

/* Benchmark helpers (host only; process-wide, not thread-safe).  ts_debug_set_score_timing_events(start, stop)
 * makes every following ts_paged_qk_scores launch record `start` when its kernel begins and `stop` when it ends
 * (events bound to the dispatch itself, so their difference is the kernel's duration without what stream-ordered
 * event records add around a launch); (NULL, NULL) switches it off.  The events are hipEvent_t handles made by
 * ts_debug_event_create; read them with ts_debug_event_elapsed_ms after the stream has been synchronised. */
int32_t ts_debug_event_create(void** event);
int32_t ts_debug_event_destroy(void* event);
int32_t ts_debug_event_elapsed_ms(void* start, void* stop, float* ms);
int32_t ts_debug_set_score_timing_events(void* start, void* stop);

#ifdef __cplusplus
}
#endif
#endif /* TOKENSELECT_H_ */
