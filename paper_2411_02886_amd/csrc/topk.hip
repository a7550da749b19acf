// TopK of Eq. 3-5 as an exact radix select over 32-bit order-preserving keys.
//
// Three histogram passes (11 + 11 + 10 bits) find the key of the k-th largest value: every
// workgroup histograms its 2048-key chunk in LDS and adds the non-empty bins to a global histogram;
// the next kernel's workgroups each walk that (8 KiB, cache-resident) histogram from the top and fix
// the digit for themselves, so no kernel waits on another workgroup and nothing but the kernel
// boundary orders the passes.  A counting pass then records per chunk the number of keys above /
// equal to the threshold key, and the emit pass writes the winners in token order: all keys above
// the threshold plus the first (k - #above) keys equal to it.  That is the "lower token index wins ties" rule and yields
// ascending indices without a sort.
#include "ts_kernels.h"

namespace ts {


// exclusive prefix sum over the 256 threads of a workgroup; *total receives the sum
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* total, uint32_t* lds /* >= 5 words */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  __syncthreads();
  if (lane == 63) lds[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint32_t x = lds[w];
    if (w < wave) base += x;
    tot += x;
  }
  *total = tot;
  return base + incl - v;
}

// Walks a global histogram from its top bin down and finds the bin holding the k_rem-th largest key.
// All 256 threads call it and all get the result: digit and the rank remaining inside that bin.
// An empty selection (k_rem == 0) returns digit = NB (no key can match it).
template <int NB>
__device__ __forceinline__ void find_digit(const uint32_t* gh, uint32_t k_rem, uint32_t* digit, uint32_t* k_next,
                                           uint32_t* lds /* >= 8 words */) {
  constexpr int PER = NB / 256;
  uint32_t c[PER];
  uint32_t sum = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) {   // thread 0 owns the top PER bins, in descending order
    c[e] = gh[NB - 1 - (threadIdx.x * PER + e)];
    sum += c[e];
  }
  uint32_t total;
  uint32_t above = block_exclusive_scan(sum, &total, lds);
  __syncthreads();
  if (threadIdx.x == 0) { lds[5] = NB; lds[6] = 0u; }
  __syncthreads();
  if (k_rem != 0) {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (above < k_rem && k_rem <= above + c[e]) { lds[5] = NB - 1 - (threadIdx.x * PER + e); lds[6] = k_rem - above; }
      above += c[e];
    }
  }
  __syncthreads();
  *digit = lds[5];
  *k_next = lds[6];
  __syncthreads();
}

// find_digit over a histogram kept as kBoundHistCopies replicas (the vote kernel's flush spreads its atomics
// over them): the copies are summed on the way in.
template <int NB>
__device__ __forceinline__ void find_digit_rep(const uint32_t* gh, uint32_t k_rem, uint32_t* digit, uint32_t* k_next,
                                               uint32_t* lds /* >= 8 words */) {
  constexpr int PER = NB / 256;
  static_assert(PER % 4 == 0, "vector loads of the thread's bins");
  uint32_t c[PER];
  // the thread's PER bins are consecutive in memory (descending bin order = ascending address from `lowest`)
  const int lowest = NB - PER - (int)threadIdx.x * PER;
#pragma unroll
  for (int e = 0; e < PER; ++e) c[e] = 0u;
#pragma unroll
  for (int r = 0; r < kBoundHistCopies; ++r)
#pragma unroll
    for (int q4 = 0; q4 < PER / 4; ++q4) {
      const uint4 w = *reinterpret_cast<const uint4*>(gh + r * NB + lowest + q4 * 4);
      c[PER - 1 - q4 * 4] += w.x; c[PER - 2 - q4 * 4] += w.y; c[PER - 3 - q4 * 4] += w.z; c[PER - 4 - q4 * 4] += w.w;
    }
  uint32_t sum = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) sum += c[e];
  uint32_t total;
  uint32_t above = block_exclusive_scan(sum, &total, lds);
  __syncthreads();
  if (threadIdx.x == 0) { lds[5] = NB; lds[6] = 0u; }
  __syncthreads();
  if (k_rem != 0) {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (above < k_rem && k_rem <= above + c[e]) { lds[5] = NB - 1 - (threadIdx.x * PER + e); lds[6] = k_rem - above; }
      above += c[e];
    }
  }
  __syncthreads();
  *digit = lds[5];
  *k_next = lds[6];
  __syncthreads();
}

// the replicated first histogram folded into histogram 0 and cleared: the five-pass form reads one copy
__global__ __launch_bounds__(256) void topk_fold_rep_hist_kernel(TopkArgs a) {
  const int b = blockIdx.y;
  if (a.skip != nullptr && a.skip[b / a.heads] != 0) return;
  const int i = blockIdx.x * 256 + threadIdx.x;         // gridDim.x * 256 == kTopkBins
  uint32_t* rep = a.rep_hist + (size_t)b * kBoundHistCopies * kTopkBins;
  uint32_t sum = 0;
#pragma unroll
  for (int r = 0; r < kBoundHistCopies; ++r) { sum += rep[r * kTopkBins + i]; rep[r * kTopkBins + i] = 0u; }
  a.hist[((size_t)b * 3 + 0) * kTopkBins + i] = sum;
}

// state words per sequence
enum { ST_PREFIX0 = 0, ST_KREM0 = 1, ST_KEFF = 2, ST_PREFIX1 = 3, ST_KREM1 = 4, ST_THR = 5, ST_NEED_EQ = 6, ST_NONE = 7 };

// tokens [LO, N) of a sequence take part: forced initial tokens, the chunk's own tokens and forced recent
// tokens do not
// (b is the virtual sequence: a.heads of them share one real sequence's length)
__device__ __forceinline__ int ranked_lo(const TopkArgs& a, int b) {
  return min(a.head, min(max(a.seq_lens[b / a.heads], 0), a.max_seq_len));
}
__device__ __forceinline__ int ranked_hi(const TopkArgs& a, int b, int lo) {
  return max(lo, min(max(a.seq_lens[b / a.heads], 0), a.max_seq_len) - a.tail);
}

__device__ __forceinline__ void load_keys(const float* v, int base, int LO, int N, uint32_t* key, bool* valid) {
#pragma unroll
  for (int i = 0; i < kTopkChunk / 256; ++i) {
    const int t = base + i * 256 + threadIdx.x;
    valid[i] = t >= LO && t < N;
    key[i] = valid[i] ? float_key(v[t]) : 0u;
  }
}

__device__ __forceinline__ void flush_hist(const uint32_t* h, uint32_t* gh, int nb) {
  for (int i = threadIdx.x; i < nb; i += 256)
    if (h[i] != 0) atomicAdd(&gh[i], h[i]);
}

// pass 0: histogram of the top 11 key bits.  A workgroup walks every gridDim.x-th chunk and flushes its LDS
// histogram once: the flush is atomics on a few hundred hot bins, so fewer, fatter workgroups contend less.
__global__ __launch_bounds__(256) void topk_hist0_kernel(TopkArgs a) {
  __shared__ uint32_t h[kTopkBins];
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b / a.heads] : 0;   // issued together with the length
  const int LO = ranked_lo(a, b), N = ranked_hi(a, b, LO);
  if (skip_flag != 0) return;
  if ((int)blockIdx.x * kTopkChunk >= N) return;
  for (int i = threadIdx.x; i < kTopkBins; i += 256) h[i] = 0;
  __syncthreads();
  for (int base = blockIdx.x * kTopkChunk; base < N; base += gridDim.x * kTopkChunk) {
    uint32_t key[kTopkChunk / 256]; bool valid[kTopkChunk / 256];
    load_keys(a.votes + (size_t)b * a.max_seq_len, base, LO, N, key, valid);
#pragma unroll
    for (int i = 0; i < kTopkChunk / 256; ++i)
      if (valid[i]) atomicAdd(&h[key[i] >> 21], 1u);
  }
  __syncthreads();
  flush_hist(h, a.hist + ((size_t)b * 3 + 0) * kTopkBins, kTopkBins);
}

// pass 1: fix digit 0 from histogram 0, histogram the next 11 bits of the keys that carry it
__global__ __launch_bounds__(256) void topk_hist1_kernel(TopkArgs a) {
  __shared__ uint32_t h[kTopkBins];
  __shared__ uint32_t lds[8];
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b / a.heads] : 0;   // issued together with the length
  const int LO = ranked_lo(a, b), N = ranked_hi(a, b, LO);
  if (skip_flag != 0) return;
  const int base = blockIdx.x * kTopkChunk;
  if (base >= N && blockIdx.x != 0) return;
  uint32_t key[kTopkChunk / 256]; bool valid[kTopkChunk / 256];
  load_keys(a.votes + (size_t)b * a.max_seq_len, base, LO, N, key, valid);
  for (int i = threadIdx.x; i < kTopkBins; i += 256) h[i] = 0;
  const uint32_t k_eff = (uint32_t)min(a.k, N - LO);
  uint32_t d0, krem0;
  find_digit<kTopkBins>(a.hist + ((size_t)b * 3 + 0) * kTopkBins, k_eff, &d0, &krem0, lds);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    a.state[b * 8 + ST_PREFIX0] = d0 << 21; a.state[b * 8 + ST_KREM0] = krem0; a.state[b * 8 + ST_KEFF] = k_eff;
  }
#pragma unroll
  for (int i = 0; i < kTopkChunk / 256; ++i)
    if (valid[i] && (key[i] >> 21) == d0) atomicAdd(&h[(key[i] >> 10) & 2047u], 1u);
  __syncthreads();
  flush_hist(h, a.hist + ((size_t)b * 3 + 1) * kTopkBins, kTopkBins);
}

// pass 2: fix digit 1, histogram the last 10 bits; histogram 0 is no longer needed and is cleared
__global__ __launch_bounds__(256) void topk_hist2_kernel(TopkArgs a) {
  __shared__ uint32_t h[1024];
  __shared__ uint32_t lds[8];
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b / a.heads] : 0;   // issued together with the length
  const int LO = ranked_lo(a, b), N = ranked_hi(a, b, LO);
  if (skip_flag != 0) return;
  const int base = blockIdx.x * kTopkChunk;
  if (base >= N && blockIdx.x != 0) return;
  uint32_t key[kTopkChunk / 256]; bool valid[kTopkChunk / 256];
  load_keys(a.votes + (size_t)b * a.max_seq_len, base, LO, N, key, valid);
  for (int i = threadIdx.x; i < 1024; i += 256) h[i] = 0;
  const uint32_t prefix0 = a.state[b * 8 + ST_PREFIX0], krem0 = a.state[b * 8 + ST_KREM0];
  uint32_t d1, krem1;
  find_digit<kTopkBins>(a.hist + ((size_t)b * 3 + 1) * kTopkBins, krem0, &d1, &krem1, lds);
  // an empty selection keeps an impossible prefix so that nothing matches below
  const bool none = krem0 == 0;
  const uint32_t prefix1 = prefix0 | ((d1 & 2047u) << 10);
  if (blockIdx.x == 0) {
    if (threadIdx.x == 0) { a.state[b * 8 + ST_PREFIX1] = prefix1; a.state[b * 8 + ST_KREM1] = none ? 0u : krem1; }
    uint32_t* g0 = a.hist + ((size_t)b * 3 + 0) * kTopkBins;
    for (int i = threadIdx.x; i < kTopkBins; i += 256) g0[i] = 0u;
  }
#pragma unroll
  for (int i = 0; i < kTopkChunk / 256; ++i)
    if (valid[i] && !none && (key[i] >> 10) == (prefix1 >> 10)) atomicAdd(&h[key[i] & 1023u], 1u);
  __syncthreads();
  flush_hist(h, a.hist + ((size_t)b * 3 + 2) * kTopkBins, 1024);
}

// fix the last digit (the threshold key is now exact) and count, per chunk, the keys above / equal to it
__global__ __launch_bounds__(256) void topk_count_kernel(TopkArgs a) {
  __shared__ uint32_t lds[8];
  __shared__ uint32_t red[4];
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b / a.heads] : 0;   // issued together with the length
  const int LO = ranked_lo(a, b), N = ranked_hi(a, b, LO);
  if (skip_flag != 0) return;
  const int base = blockIdx.x * kTopkChunk;
  uint32_t key[kTopkChunk / 256]; bool valid[kTopkChunk / 256];
  load_keys(a.votes + (size_t)b * a.max_seq_len, base, LO, N, key, valid);
  const uint32_t prefix1 = a.state[b * 8 + ST_PREFIX1], krem1 = a.state[b * 8 + ST_KREM1];
  uint32_t d2, need_eq;
  find_digit<1024>(a.hist + ((size_t)b * 3 + 2) * kTopkBins, krem1, &d2, &need_eq, lds);
  const bool none = krem1 == 0;
  const uint32_t thr = none ? 0xffffffffu : (prefix1 | (d2 & 1023u));
  if (none) need_eq = 0;
  if (blockIdx.x == 0) {
    if (threadIdx.x == 0) {
      a.state[b * 8 + ST_THR] = thr; a.state[b * 8 + ST_NEED_EQ] = need_eq; a.state[b * 8 + ST_NONE] = none;
    }
    uint32_t* g1 = a.hist + ((size_t)b * 3 + 1) * kTopkBins;
    for (int i = threadIdx.x; i < kTopkBins; i += 256) g1[i] = 0u;
  }
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int i = 0; i < kTopkChunk / 256; ++i) {
    gt += valid[i] && !none && key[i] > thr;
    eq += valid[i] && !none && key[i] == thr;
  }
  uint32_t packed = gt | (eq << 16);   // a chunk holds 2048 keys: both counts fit in 16 bits
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) packed += __shfl_xor(packed, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = packed;
  __syncthreads();
  if (threadIdx.x == 0) a.blk[(size_t)b * a.nblk + blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

// winners of a chunk, in token order; every workgroup sums the counts of the chunks before it
__global__ __launch_bounds__(256) void topk_emit_kernel(TopkArgs a) {
  __shared__ uint32_t scan_lds[8];
  __shared__ uint32_t red[2][4];
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b / a.heads] : 0;   // issued together with the length
  const int LO = ranked_lo(a, b), N = ranked_hi(a, b, LO);
  if (skip_flag != 0) return;
  const uint32_t thr = a.state[b * 8 + ST_THR];
  const uint32_t need_eq = a.state[b * 8 + ST_NEED_EQ];
  const bool none = a.state[b * 8 + ST_NONE] != 0;
  const int k_eff = (int)a.state[b * 8 + ST_KEFF];
  const bool as_votes = a.vote_acc != nullptr;      // Eq. 4: winners are counted per token, not listed
  int32_t* out = as_votes ? nullptr : a.idx + (size_t)b * a.k;
  float* acc = as_votes ? a.vote_acc + (size_t)(b / a.heads) * a.max_seq_len : nullptr;
  if (blockIdx.x == 0) {
    if (!as_votes) {
      for (int i = k_eff + threadIdx.x; i < a.k; i += 256) out[i] = -1;
      if (threadIdx.x == 0) a.count[b] = k_eff;
    }
    uint32_t* g2 = a.hist + ((size_t)b * 3 + 2) * kTopkBins;
    for (int i = threadIdx.x; i < 1024; i += 256) g2[i] = 0u;
  }
  const int base = blockIdx.x * kTopkChunk;
  if (base >= N || none) return;
  const float* v = a.votes + (size_t)b * a.max_seq_len;
  constexpr int PER = kTopkChunk / 256;
  const int t0 = base + threadIdx.x * PER;   // PER consecutive tokens per thread: order is preserved
  uint32_t key[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) key[e] = ((t0 + e) >= LO && (t0 + e) < N) ? float_key(v[t0 + e]) : 0u;
  // counts of all earlier chunks (gt in the low half is too narrow for a sum: add the halves apart)
  uint32_t pg = 0, pe = 0;
  const uint32_t* blk = a.blk + (size_t)b * a.nblk;
  for (int i = threadIdx.x; i < (int)blockIdx.x; i += 256) { const uint32_t x = blk[i]; pg += x & 0xffffu; pe += x >> 16; }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { pg += __shfl_xor(pg, off); pe += __shfl_xor(pe, off); }
  if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = pg; red[1][threadIdx.x >> 6] = pe; }
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const bool valid = (t0 + e) >= LO && (t0 + e) < N;
    gt += valid && key[e] > thr;
    eq += valid && key[e] == thr;
  }
  uint32_t total;
  const uint32_t ex = block_exclusive_scan(gt | (eq << 16), &total, scan_lds);   // has the barriers red[] needs
  uint32_t gt_before = red[0][0] + red[0][1] + red[0][2] + red[0][3] + (ex & 0xffffu);
  uint32_t eq_before = red[1][0] + red[1][1] + red[1][2] + red[1][3] + (ex >> 16);
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int t = t0 + e;
    if (t >= LO && t < N) {
      if (key[e] > thr) {
        if (as_votes) atomicAdd(&acc[t], 1.0f);      // small integers: exact and order-independent in float
        else out[gt_before + min(eq_before, need_eq)] = t;
        ++gt_before;
      } else if (key[e] == thr) {
        if (eq_before < need_eq) {
          if (as_votes) atomicAdd(&acc[t], 1.0f);
          else out[gt_before + eq_before] = t;
        }
        ++eq_before;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Short path (3 launches): after pass 0 every chunk compacts, in token order, the keys that fall in or above
// the bin of the k-th key (the winners for sure plus the few candidates that share its bin; typically k plus a
// few hundred entries in all), and one workgroup per sequence finishes the job on that list: two more radix
// digits over the candidates in LDS histograms, then the ordered emit.  Same result as the five-pass form.

constexpr int kFinalThreads = 1024;        // many threads, few entries each: the per-entry chain of a thread is the latency
                                           // that counts (256 threads x 32 entries measured 1.7x slower)
constexpr int kFinalMaxBlk = 8192;         // chunks per sequence the short path handles (16 Mi tokens)

// pass 1 of the short path: fix digit 0, compact the entries with (key >> 21) >= digit 0
__global__ __launch_bounds__(256) void topk_compact_kernel(TopkArgs a) {
  __shared__ uint32_t lds[8];
  __shared__ uint32_t scan_lds[8];
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b / a.heads] : 0;   // issued together with the length
  const int LO = ranked_lo(a, b), N = ranked_hi(a, b, LO);
  if (skip_flag != 0) return;
  const uint32_t k_eff = (uint32_t)min(a.k, N - LO);
  constexpr int PER = kTopkChunk / 256;
  const int base = blockIdx.x * kTopkChunk;
  const int t0 = base + threadIdx.x * PER;   // PER consecutive tokens per thread: order is preserved
  const float* v = a.votes + (size_t)b * a.max_seq_len;
  // the votes are loaded before the histogram is walked: the two round trips overlap
  uint32_t key[PER];
  bool valid[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    valid[e] = (t0 + e) >= LO && (t0 + e) < N;
    key[e] = valid[e] ? float_key(v[t0 + e]) : 0u;
  }
  uint32_t d0, krem0;
  if (a.rep_hist != nullptr) find_digit_rep<kTopkBins>(a.rep_hist + (size_t)b * kBoundHistCopies * kTopkBins, k_eff, &d0, &krem0, lds);
  else find_digit<kTopkBins>(a.hist + ((size_t)b * 3 + 0) * kTopkBins, k_eff, &d0, &krem0, lds);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    a.state[b * 8 + ST_PREFIX0] = d0 << 21; a.state[b * 8 + ST_KREM0] = krem0; a.state[b * 8 + ST_KEFF] = k_eff;
  }
  uint32_t n = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) n += valid[e] && (key[e] >> 21) >= d0;      // d0 == kTopkBins (empty selection) matches nothing
  uint32_t total;
  uint32_t pos = block_exclusive_scan(n, &total, scan_lds);
  uint2* list = a.list + ((size_t)b * a.nblk + blockIdx.x) * kTopkChunk;
#pragma unroll
  for (int e = 0; e < PER; ++e)
    if (valid[e] && (key[e] >> 21) >= d0) list[pos++] = make_uint2(key[e], (uint32_t)(t0 + e));
  if (threadIdx.x == 0) a.blk[(size_t)b * a.nblk + blockIdx.x] = total;
}

// exclusive prefix sum over the kFinalThreads threads of the final workgroup
__device__ __forceinline__ uint32_t final_exclusive_scan(uint32_t v, uint32_t* total, uint32_t* lds /* >= 16 words */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  __syncthreads();
  if (lane == 63) lds[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kFinalThreads / 64; ++w) {
    const uint32_t x = lds[w];
    if (w < wave) base += x;
    tot += x;
  }
  *total = tot;
  return base + incl - v;
}

// digit of the k_rem-th largest key in an LDS histogram of NB bins (all threads get the result)
template <int NB>
__device__ __forceinline__ void final_find_digit(const uint32_t* h, uint32_t k_rem, uint32_t* digit, uint32_t* k_next,
                                                 uint32_t* scan_lds, uint32_t* res /* 2 words */) {
  constexpr int PER = NB / kFinalThreads;
  uint32_t c[PER];
  uint32_t sum = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) { c[e] = h[NB - 1 - (threadIdx.x * PER + e)]; sum += c[e]; }
  uint32_t total;
  uint32_t above = final_exclusive_scan(sum, &total, scan_lds);
  if (threadIdx.x == 0) { res[0] = NB; res[1] = 0u; }
  __syncthreads();
  if (k_rem != 0) {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (above < k_rem && k_rem <= above + c[e]) { res[0] = NB - 1 - (threadIdx.x * PER + e); res[1] = k_rem - above; }
      above += c[e];
    }
  }
  __syncthreads();
  *digit = res[0];
  *k_next = res[1];
  __syncthreads();
}

// passes 2, 3 and the emit of the short path: one workgroup per (virtual) sequence
// FULL: the list holds exact votes whose top digit has not been fixed yet (compact selection: the entries are
// the re-evaluated candidates), so digit 0 is found here too, over the entries.
template <int kFinalPer, bool FULL>        // consecutive list entries per thread and batch
__global__ __launch_bounds__(kFinalThreads) void topk_final_kernel(TopkArgs a) {
  __shared__ uint32_t off[kFinalMaxBlk + 1];   // exclusive prefix of the chunks' entry counts
  __shared__ uint32_t h[kTopkBins];
  __shared__ uint32_t scan_lds[16];
  __shared__ uint32_t res[2];
  const int b = blockIdx.x;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b / a.heads] : 0;   // issued together with the state words
  const int tid = threadIdx.x;
  uint32_t d0 = FULL ? 0u : a.state[b * 8 + ST_PREFIX0] >> 21, krem0 = FULL ? 0u : a.state[b * 8 + ST_KREM0];
  const int k_eff = (int)a.state[b * 8 + ST_KEFF];
  if (skip_flag != 0) return;
  const bool as_votes = a.vote_acc != nullptr;
  int32_t* out = as_votes ? nullptr : a.idx + (size_t)b * a.k;
  float* acc = as_votes ? a.vote_acc + (size_t)(b / a.heads) * a.max_seq_len : nullptr;
  if (!as_votes) {
    // FULL: the candidates come from float comparisons; with NaN among the votes fewer than k_eff of them may
    // arrive, and the slots that then stay empty must not keep an older selection's ids (finite votes fill them all)
    for (int i = (FULL ? 0 : k_eff) + tid; i < a.k; i += kFinalThreads) out[i] = -1;
    if (FULL && a.sel_votes != nullptr)
      for (int i = k_eff + tid; i < a.k; i += kFinalThreads) a.sel_votes[(size_t)b * a.k + i] = 0.f;
    if (tid == 0) a.count[b] = k_eff;
  }
  if (FULL) {  // the replicated histogram of the lower bounds has been consumed by the refine pass: zero it again
    uint4* g0 = reinterpret_cast<uint4*>(a.bound_hist + (size_t)b * kBoundHistCopies * kTopkBins);   // 256-byte aligned section
    for (int i = tid; i < kBoundHistCopies * kTopkBins / 4; i += kFinalThreads) g0[i] = make_uint4(0u, 0u, 0u, 0u);
  } else if (a.rep_hist != nullptr) {   // the vote kernel's replicated histogram has been consumed by the compact pass
    uint4* g0 = reinterpret_cast<uint4*>(a.rep_hist + (size_t)b * kBoundHistCopies * kTopkBins);
    for (int i = tid; i < kBoundHistCopies * kTopkBins / 4; i += kFinalThreads) g0[i] = make_uint4(0u, 0u, 0u, 0u);
  } else {     // histogram 0 has been consumed by the compact pass: leave it zeroed for the next call
    uint32_t* g0 = a.hist + ((size_t)b * 3 + 0) * kTopkBins;
    for (int i = tid; i < kTopkBins; i += kFinalThreads) g0[i] = 0u;
  }
  // ---- chunk offsets
  uint32_t carry = 0;
  for (int c0 = 0; c0 < a.nblk; c0 += kFinalThreads) {
    const int c = c0 + tid;
    const uint32_t n = c < a.nblk ? a.blk[(size_t)b * a.nblk + c] : 0u;
    uint32_t tot;
    const uint32_t ex = final_exclusive_scan(n, &tot, scan_lds);
    if (c < a.nblk) off[c] = carry + ex;
    carry += tot;
    __syncthreads();
  }
  const uint32_t total = carry;
  if (tid == 0) off[a.nblk] = total;
  __syncthreads();
  if (total == 0 || k_eff == 0) return;
  const uint2* list = a.list + (size_t)b * a.nblk * kTopkChunk;

  // entries of a batch: thread tid owns the kFinalPer consecutive positions from p0
  auto load_batch = [&](uint32_t base, uint2 (&e)[kFinalPer]) {
    const uint32_t p0 = base + (uint32_t)tid * kFinalPer;
    int c = 0;
    if (p0 < total) {                         // chunk with off[c] <= p0 < off[c + 1]
      int lo = 0, hi = a.nblk;                // invariant: off[lo] <= p0 < off[hi]
      while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (off[mid] <= p0) lo = mid; else hi = mid; }
      c = lo;
    }
    uint32_t cur = off[c], next = off[c + 1];
#pragma unroll
    for (int i = 0; i < kFinalPer; ++i) {
      const uint32_t p = p0 + i;
      e[i] = make_uint2(0u, 0xffffffffu);
      if (p < total) {
        while (p >= next) { ++c; cur = next; next = off[c + 1]; }   // ends: p < total = off[nblk]
        e[i] = list[(size_t)c * kTopkChunk + (p - cur)];
      }
    }
  };
  const bool single = total <= (uint32_t)kFinalThreads * kFinalPer;   // the usual case: the list sits in registers
  uint2 e[kFinalPer];
  if (single) load_batch(0, e);

  if (FULL) {   // ---- digit 0: bits 31..21 over all entries
    for (int i = tid; i < kTopkBins; i += kFinalThreads) h[i] = 0u;
    __syncthreads();
    for (uint32_t base = 0; base < total; base += kFinalThreads * kFinalPer) {
      if (!single) load_batch(base, e);
#pragma unroll
      for (int i = 0; i < kFinalPer; ++i)
        if (e[i].y != 0xffffffffu) atomicAdd(&h[e[i].x >> 21], 1u);
    }
    __syncthreads();
    final_find_digit<kTopkBins>(h, (uint32_t)k_eff, &d0, &krem0, scan_lds, res);
  }
  // ---- digit 1: bits 20..10 of the candidates (entries of bin d0)
  for (int i = tid; i < kTopkBins; i += kFinalThreads) h[i] = 0u;
  __syncthreads();
  for (uint32_t base = 0; base < total; base += kFinalThreads * kFinalPer) {
    if (!single) load_batch(base, e);
#pragma unroll
    for (int i = 0; i < kFinalPer; ++i)
      if (e[i].y != 0xffffffffu && (e[i].x >> 21) == d0) atomicAdd(&h[(e[i].x >> 10) & 2047u], 1u);
  }
  __syncthreads();
  uint32_t d1, krem1;
  final_find_digit<kTopkBins>(h, krem0, &d1, &krem1, scan_lds, res);
  const uint32_t prefix1 = (d0 << 21) | ((d1 & 2047u) << 10);
  // ---- digit 2: the last 10 bits -- unless every entry that shares the threshold's 22-bit prefix is a winner (the
  // usual case: a few thousand entries over 2^22 prefixes leave the threshold's bin with one or two), when the
  // prefix alone decides
  uint32_t thr, need_eq;
  const uint32_t cnt1 = d1 < (uint32_t)kTopkBins ? h[d1] : 0xffffffffu;
  if (krem1 == cnt1 && prefix1 != 0u) {
    thr = prefix1 - 1u; need_eq = 0u;          // "above thr" = "prefix at least prefix1"; nothing equals thr among the winners
  } else {
    __syncthreads();                            // every thread has read cnt1 before the histogram is cleared
    for (int i = tid; i < 1024; i += kFinalThreads) h[i] = 0u;
    __syncthreads();
    for (uint32_t base = 0; base < total; base += kFinalThreads * kFinalPer) {
      if (!single) load_batch(base, e);
#pragma unroll
      for (int i = 0; i < kFinalPer; ++i)
        if (e[i].y != 0xffffffffu && (e[i].x >> 10) == (prefix1 >> 10)) atomicAdd(&h[e[i].x & 1023u], 1u);
    }
    __syncthreads();
    uint32_t d2;
    final_find_digit<1024>(h, krem1, &d2, &need_eq, scan_lds, res);
    thr = prefix1 | (d2 & 1023u);
  }
  // ---- emit in token order: every key above the threshold, and the first need_eq keys equal to it
  uint32_t gt_done = 0, eq_done = 0;
  for (uint32_t base = 0; base < total; base += kFinalThreads * kFinalPer) {
    if (!single) load_batch(base, e);
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < kFinalPer; ++i) {
      const bool valid = e[i].y != 0xffffffffu;
      gt += valid && e[i].x > thr;
      eq += valid && e[i].x == thr;
    }
    uint32_t tot;
    const uint32_t ex = final_exclusive_scan(gt | (eq << 16), &tot, scan_lds);   // a batch holds at most 8192 entries: 14 bits each half
    uint32_t gt_before = gt_done + (ex & 0xffffu), eq_before = eq_done + (ex >> 16);
#pragma unroll
    for (int i = 0; i < kFinalPer; ++i) {
      if (e[i].y == 0xffffffffu) continue;
      const int t = (int)e[i].y;
      if (e[i].x > thr) {
        if (as_votes) atomicAdd(&acc[t], 1.0f);
        else {
          out[gt_before + min(eq_before, need_eq)] = t;
          if (FULL && a.sel_votes != nullptr) a.sel_votes[(size_t)b * a.k + gt_before + min(eq_before, need_eq)] = key_float(e[i].x);
        }
        ++gt_before;
      } else if (e[i].x == thr) {
        if (eq_before < need_eq) {
          if (as_votes) atomicAdd(&acc[t], 1.0f);
          else {
            out[gt_before + eq_before] = t;
            if (FULL && a.sel_votes != nullptr) a.sel_votes[(size_t)b * a.k + gt_before + eq_before] = key_float(e[i].x);
          }
        }
        ++eq_before;
      }
    }
    gt_done += tot & 0xffffu; eq_done += tot >> 16;
    __syncthreads();
  }
}

hipError_t launch_topk(const TopkArgs& a, int B, hipStream_t s) {
  dim3 grid(a.nblk, B);
  const bool short_path = a.list != nullptr && a.nblk <= kFinalMaxBlk;
  if (a.rep_hist == nullptr) {
    hipLaunchKernelGGL(topk_hist0_kernel, dim3(a.nblk < 128 ? a.nblk : 128, B), dim3(256), 0, s, a);
  } else if (!short_path) {
    hipLaunchKernelGGL(topk_fold_rep_hist_kernel, dim3(kTopkBins / 256, B), dim3(256), 0, s, a);
  }
  if (short_path) {
    hipLaunchKernelGGL(topk_compact_kernel, grid, dim3(256), 0, s, a);
    // the list holds about k entries plus the few that share the k-th key's bin: one batch in the usual case
    if (a.k <= 3072) hipLaunchKernelGGL((topk_final_kernel<4, false>), dim3(B), dim3(kFinalThreads), 0, s, a);
    else hipLaunchKernelGGL((topk_final_kernel<8, false>), dim3(B), dim3(kFinalThreads), 0, s, a);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(topk_hist1_kernel, grid, dim3(256), 0, s, a);
  hipLaunchKernelGGL(topk_hist2_kernel, grid, dim3(256), 0, s, a);
  hipLaunchKernelGGL(topk_count_kernel, grid, dim3(256), 0, s, a);
  hipLaunchKernelGGL(topk_emit_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

// finishing workgroup over a list of exact votes (compact selection)
hipError_t launch_topk_final_full(const TopkArgs& a, int B, hipStream_t s) {
  if (a.k <= 2048) hipLaunchKernelGGL((topk_final_kernel<4, true>), dim3(B), dim3(kFinalThreads), 0, s, a);
  else hipLaunchKernelGGL((topk_final_kernel<8, true>), dim3(B), dim3(kFinalThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace ts
