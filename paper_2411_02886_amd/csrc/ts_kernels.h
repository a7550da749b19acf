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
};

struct VoteArgs {
  const float* scores;
  const float* partials;  // per-workgroup statistics left by the score pass
  int nparts;             // workgroups per sequence the score pass ran with
  float* row_stats_out;   // merged (max, sum-exp) per head, written by the merge kernel
  const float* row_stats; // same buffer, read by the vote kernel
  float* votes;
  const int32_t* seq_lens;
  const uint8_t* skip;
  int H, max_seq_len;
  int n_init, n_local;    // forced tokens: votes outside [min(n_init, N), max(that, N - n_local)) are 0
  float scale;
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
hipError_t launch_topk(const TopkArgs& a, int B, hipStream_t s);
hipError_t launch_selcache(const SelcacheArgs& a, int B, hipStream_t s);
hipError_t launch_sparse_attn_decode(int dtype, int D, int G, const AttnArgs& a, int B, hipStream_t s);
hipError_t launch_chunk_mean_query(const void* q, void* out, int B, int C, int n, hipStream_t s);
hipError_t launch_sum_vote(const VoteArgs& a, int B, hipStream_t s);
hipError_t launch_transpose_scores(const VoteArgs& a, float* st, int B, hipStream_t s);
hipError_t launch_zero_votes(const VoteArgs& a, int B, hipStream_t s);
hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s);
void set_score_timing_events(hipEvent_t start, hipEvent_t stop);

}  // namespace ts
