// Kernel argument blocks and launch entry points shared by the host API and the kernel files.
#pragma once
#include "ts_common.h"

namespace ts {

struct ScoreArgs {
  const uint8_t* q;
  const uint8_t* k_pool;
  const int32_t* page_indptr;
  const int32_t* page_indices;
  const int32_t* seq_lens;
  const uint8_t* skip;
  float* scores;
  float* partials;        // [B][kScoreMaxWg][H][2] per-workgroup (max, sum-exp)
  int H, H_kv, P, p_shift, max_seq_len;
  int HB, hb_shift, NU;   // KV heads per wave tile (min(H_kv, 8)), its log2, H_kv / HB
  int uniform_page;       // every step of a wave reads one page (P >= tokens per step)
  int vec_store;          // score rows can be written as 16-byte pieces
  int RR;                 // consecutive tiles a wave stages in LDS and writes out as one run (1, 2 or 4)
  int n_init, n_local;    // forced tokens: the statistics cover [min(n_init, N), max(that, N - n_local)) only
  float scale, c2;        // score_scale and score_scale * log2(e)
  uint32_t* hdr;          // [B][8] what later calls must know about this launch (partials / block size, score_scale)
  // compact form (codes != nullptr): one byte per score plus exact per-block statistics instead of S
  uint8_t* codes;         // [B][max_seq_len][H]
  float* blk_max;         // [B][nblk][H] maximum of each head over the block's ranked tokens
  int nblk;               // blocks per sequence the array is strided by: ceil(max_seq_len / 32)
  int ncp_shift;          // log2 of the power of two >= HB * G
  int nt_codes;           // matrix-core compact form, whole token rows per wave (NU == 1): bytes and block maxima leave as non-temporal stores
  // Algorithm 1's test inside this launch (sc_cached_q != nullptr; `skip` is then unused): every workgroup takes
  // the decision itself from Q and C_Q, workgroup 0 of a sequence writes the state after the step
  const uint8_t* sc_cached_q;   // [B][H][D] C_Q before the step, read only
  uint8_t* sc_cached_q_next;    // [B][H][D] C_Q after the step, another buffer
  const uint8_t* sc_first;      // [B]
  uint8_t* sc_first_next;       // [B]
  uint8_t* sc_reuse;            // [B] out
  float sc_theta;
};

// compact form of the selection: statistics merge, vote bounds, exact re-evaluation of the candidates
struct BoundArgs {
  const uint8_t* codes;
  const float* blk_max;
  const uint32_t* hdr;
  const float* row_stats; // [B][H][2] merged (max, sum-exp)
  float* vote_hi;         // [B][max_seq_len] upper bound of every vote
  float* vote_lo;         // [B][max_seq_len] lower bound
  uint32_t* hist;         // [B][kBoundHistCopies][kTopkBins]: top 11 key bits of the lower bounds, one replica per workgroup residue
  const int32_t* seq_lens;
  const uint8_t* skip;
  int H, max_seq_len, nblk;
  int n_init, n_local;
  int vec;                // H % 4 == 0 and aligned buffers: codes and block maxima are read four heads at a time
  float scale;
};

struct VoteArgs {
  const float* scores;
  const float* partials;  // per-workgroup statistics left by the score pass
  const uint32_t* hdr;    // [B][8]: word 0 = workgroups per sequence the score pass ran with (its partials)
  float* row_stats_out;   // merged (max, sum-exp) per head, written by the merge kernel
  const float* row_stats; // same buffer, read by the vote kernel
  float* votes;
  const int32_t* seq_lens;
  const uint8_t* skip;
  int H, max_seq_len;
  int n_init, n_local;    // forced tokens: votes outside [min(n_init, N), max(that, N - n_local)) are 0
  float scale;
  uint32_t* rank_hist;    // ranked vote only: [B][kBoundHistCopies][kTopkBins], top 11 key bits of the votes it writes
};

struct TopkArgs {
  int head;             // leading tokens of every sequence that do not take part (forced initial tokens)
  int tail;             // trailing tokens that do not take part (the chunk's own tokens / forced recent tokens)
  const float* votes;
  const int32_t* seq_lens;
  const uint8_t* skip;
  int32_t* idx;
  int32_t* count;
  uint32_t* hist;       // [B][3][kTopkBins]
  uint32_t* state;      // [B][8]
  uint32_t* blk;        // [B][nblk]
  uint2* list;          // [B][nblk][kTopkChunk] (key, token) entries of the short path; nullptr = five-pass form
  int k, max_seq_len, nblk;
  int heads;            // virtual sequences per real one (Eq. 4: one per head over transposed scores); 1 = plain
  float* vote_acc;      // Eq. 4: the emit pass adds 1 to vote_acc[real sequence][t] for every winner instead of writing idx
  float* sel_votes;     // compact selection: [B][k] votes of the selected tokens in idx order, or nullptr
  uint32_t* bound_hist; // compact selection: [B][kBoundHistCopies][kTopkBins] histogram of the vote lower bounds (else nullptr)
  uint32_t* rep_hist;   // the first histogram was left by the vote kernel, replicated like bound_hist (else nullptr: pass 0 builds it)
};

// exact votes of the candidates (tokens whose upper bound reaches the bin of the k-th largest lower bound)
struct RefineArgs {
  TopkArgs t;             // votes = the upper bounds; hist / state / blk / list as in the short top-k path
  const uint8_t* q;
  const uint8_t* k_pool;
  const int32_t* page_indptr;
  const int32_t* page_indices;
  const float* row_stats;
  int H, H_kv, P, p_shift;
  int HB, hb_shift, NU;
  float scale;
  int parts;              // workgroups per 2048-token chunk: each re-evaluates its share of the chunk's candidates
};

struct SelcacheArgs {
  const uint8_t* q;
  uint8_t* cached_q;
  uint8_t* first;
  uint8_t* reuse;
  int n;          // H * D elements per sequence
  int dtype;
  float theta;
};

struct AttnArgs {
  const uint8_t* q;
  const uint8_t* k_pool;
  const uint8_t* v_pool;
  const int32_t* page_indptr;
  const int32_t* page_indices;
  const int32_t* seq_lens;
  const int32_t* idx;
  const int32_t* count;
  uint8_t* out;
  float* lse;
  float* part_out;     // [B][H][nsplit][D]
  float* part_ml;      // [B][H][nsplit][2]
  int H, H_kv, P, p_shift, idx_stride, nsplit, max_seq_len;
  int n_init, n_local;  // forced tokens attended before / after the selected ones
  int nch;              // chunks of kAttnChunk tokens per workgroup (1 .. kAttnMaxRun); nsplit counts workgroups
  float sm_scale;
};

// chunked-prefill selection (both sweeps)
struct PrefillArgs {
  const uint8_t* q;          // [B][C][H][D] bf16
  const uint8_t* k_pool;
  const int32_t* page_indptr;
  const int32_t* page_indices;
  const int32_t* seq_lens;
  float* stat_part;          // [B][TS][C][H][2] sweep-1 partial (max, sum-exp) per token split
  float* row_stats_out;      // [B][C][H][2] merged
  const float* row_stats;    // [B][C][H][2] read by sweep 2
  float* vote_part;          // [B][RB * H_kv][max_seq_len] sweep-2 partial votes per (row block, KV head)
  float* votes;              // [B][max_seq_len]
  int B, C, H, H_kv, G, D, P, p_shift, max_seq_len;
  int RB;                    // 256-row blocks per KV head: ceil(C * G / 256)
  int n_init, n_local;       // forced tokens: only cached tokens [min(n_init, Nc), max(that, Nc - n_local)) are ranked
  int TS;                    // token splits
  float scale, c2;
};

hipError_t launch_prefill_stats(const PrefillArgs& a, hipStream_t s);
hipError_t launch_prefill_votes(const PrefillArgs& a, hipStream_t s);

// chunk-form sparse attention
struct ChunkAttnArgs {
  const uint8_t* q;          // [B][C][H][D] bf16
  const uint8_t* k_pool;
  const uint8_t* v_pool;
  const int32_t* page_indptr;
  const int32_t* page_indices;
  const int32_t* seq_lens;
  const int32_t* idx;
  const int32_t* count;
  int32_t* slots;            // [B][idx_stride + C] physical slots of the key list
  uint8_t* out;              // [B][C][H][D] bf16
  float* lse;                // [B][C][H] or null
  int C, H, H_kv, G, D, P, p_shift, idx_stride, max_seq_len;
  int nsplit;                // key-list splits per row block (1 = the kernel writes the result itself)
  int n_init, n_local;       // forced cached tokens attended before / after the selected ones
  int slot_stride;           // row stride of slots: idx_stride + n_init + n_local + C
  float* part_o;             // [B][C][H][nsplit][D] un-normalised partial outputs (nsplit > 1)
  float* part_ml;            // [B][C][H][nsplit][2] (reference exponent, row sum) of each partial
  float sm_scale;
};
hipError_t launch_sparse_attn_chunk(const ChunkAttnArgs& a, int B, hipStream_t s);

// variant: 0 = fma arithmetic, 1 = packed bf16 dot2 (bf16 only)
hipError_t launch_score_decode(int dtype, int D, int G, int variant, const ScoreArgs& a, dim3 grid, size_t lds, hipStream_t s);
hipError_t launch_soft_vote(const VoteArgs& a, int B, hipStream_t s);
// Eq. 5 (statistics merge + vote) plus the first radix histogram of the votes (a.rank_hist)
hipError_t launch_soft_vote_ranked(const VoteArgs& a, int B, hipStream_t s);
hipError_t launch_stats_merge(const VoteArgs& a, int B, hipStream_t s);
hipError_t launch_vote_bounds(const BoundArgs& a, int B, hipStream_t s);
hipError_t launch_topk_refine(int dtype, int D, int G, const RefineArgs& a, int B, hipStream_t s);
hipError_t launch_topk(const TopkArgs& a, int B, hipStream_t s);
hipError_t launch_topk_final_full(const TopkArgs& a, int B, hipStream_t s);
constexpr int kTopkFinalMaxBlk = 8192;   // chunks per sequence the finishing workgroup can index (16 Mi tokens)
hipError_t launch_selcache(const SelcacheArgs& a, int B, hipStream_t s);
hipError_t launch_sparse_attn_decode(int dtype, int D, int G, const AttnArgs& a, int B, hipStream_t s);
hipError_t launch_chunk_mean_query(const void* q, void* out, int B, int C, int n, hipStream_t s);
hipError_t launch_sum_vote(const VoteArgs& a, int B, hipStream_t s);
hipError_t launch_transpose_scores(const VoteArgs& a, float* st, int B, hipStream_t s);
hipError_t launch_zero_votes(const VoteArgs& a, int B, hipStream_t s);
hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s);
void set_score_timing_events(hipEvent_t start, hipEvent_t stop);
void set_codes_timing_events(hipEvent_t start, hipEvent_t stop);
bool score_codes_mfma_supported(int dtype, int D, int G, int H_kv);
size_t score_codes_mfma_lds_bytes(int D, int G, int RR, bool dense = false);
hipError_t launch_score_codes_mfma(int D, int G, const ScoreArgs& a, dim3 grid, size_t lds, hipStream_t s);

}  // namespace ts
