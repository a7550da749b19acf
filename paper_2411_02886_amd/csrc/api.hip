// C ABI of the library: argument validation, workspace carving and kernel launches.
#include "ts_kernels.h"

namespace ts {

__global__ void fill_zero_kernel(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

static int g_score_variant = 2;   // 0 = fma, 1 = packed bf16 dot2, 2 = matrix cores where the shape allows, else 1 (tuning knob, see ts_debug_set_score_variant)
static int g_score_wg = 0;        // 0 = automatic
static int g_score_rr = 0;        // tiles per staged run; 0 = automatic
static int g_topk_five_pass = 0;  // 1 = force the five-pass radix select (tuning knob)
static int g_codes_mfma = 1;      // 1 = the compact score pass runs on the matrix cores where the shape allows
static int g_codes_rr = 0;        // tiles per run of the matrix-core compact score pass; 0 = automatic

// workgroups per sequence of the score pass (also the number of statistics partials it leaves)
// Tiles a wave of the score pass stages before writing them out: longer runs make the score stores
// fewer, larger bursts (a write stream mixed into the K read stream is what costs bandwidth), but every
// wave of the machine should still get a run of its own and the staging must fit 64 KiB of LDS.
static int score_run_tiles(const ts_problem* p) {
  const int hb = p->num_kv_heads < 8 ? p->num_kv_heads : 8;
  const int nu = p->num_kv_heads / hb;
  const int hs = (hb * (p->num_q_heads / p->num_kv_heads) + 3) & ~3;
  const long ntiles = (long)(p->max_seq_len + kScoreTileTokens - 1) / kScoreTileTokens;
  for (int rr = 4; rr > 1; rr >>= 1) {
    const long runs = (ntiles + rr - 1) / rr * nu;   // per sequence: others of the batch may be skipped
    if (runs >= 4096 && (size_t)4 * rr * kScoreTileTokens * hs * sizeof(float) <= 65536 - 1024) return rr;   // 1 KiB goes to the block maxima of the compact form
  }
  return 1;
}

// run length in effect: the forced one (tuning knob) halved until its staging fits, else the automatic one
static int score_run_tiles_eff(const ts_problem* p) {
  if (g_score_rr <= 0) return score_run_tiles(p);
  const int hb = p->num_kv_heads < 8 ? p->num_kv_heads : 8;
  const int hs = (hb * (p->num_q_heads / p->num_kv_heads) + 3) & ~3;
  int rr = g_score_rr;
  while (rr > 1 && (size_t)4 * rr * kScoreTileTokens * hs * sizeof(float) > 65536 - 1024) rr >>= 1;
  return rr;
}

static int score_workgroups(const ts_problem* p) {
  const int hb = p->num_kv_heads < 8 ? p->num_kv_heads : 8;
  const int nu = p->num_kv_heads / hb;
  const int rr = score_run_tiles_eff(p);
  const int ntiles = (p->max_seq_len + kScoreTileTokens - 1) / kScoreTileTokens;
  const int nruns = (ntiles + rr - 1) / rr * nu;
  // per sequence, whatever the batch: with a Selection Cache most sequences of a step may be skipped, and the
  // ones that are scanned must still fill the machine
  int wg = g_score_wg > 0 ? g_score_wg : (nruns + 3) / 4;
  if (wg > kScoreMaxWg) wg = kScoreMaxWg;
  if (wg < 1) wg = 1;
  return wg;
}

static int ilog2(int x) { int s = 0; while ((1 << s) < x) ++s; return s; }
static bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// shape checks shared by all calls; returns TS_OK or an error
static int32_t check_problem(const ts_problem* p) {
  if (p == nullptr) return TS_ERR_INVALID_ARG;
  if (p->batch < 1 || p->chunk < 1 || p->num_q_heads < 1 || p->num_kv_heads < 1 || p->head_dim < 1 ||
      p->page_size < 1 || p->max_seq_len < 1)
    return TS_ERR_INVALID_ARG;
  if (p->num_q_heads % p->num_kv_heads != 0) return TS_ERR_INVALID_ARG;
  if (p->dtype != TS_F32 && p->dtype != TS_BF16) return TS_ERR_INVALID_ARG;
  if (p->page_indptr == nullptr || p->page_indices == nullptr || p->seq_lens == nullptr) return TS_ERR_INVALID_ARG;
  if (p->head_dim != 64 && p->head_dim != 128) return TS_ERR_UNSUPPORTED;
  if (p->num_q_heads > 128) return TS_ERR_UNSUPPORTED;
  if (p->batch > 65535) return TS_ERR_UNSUPPORTED;           // the sequence is a grid dimension of every kernel
  if (!is_pow2(p->num_kv_heads) || p->num_kv_heads > 32) return TS_ERR_UNSUPPORTED;
  if (p->num_q_heads / p->num_kv_heads > 8) return TS_ERR_UNSUPPORTED;
  if (!is_pow2(p->page_size)) return TS_ERR_UNSUPPORTED;
  const int hb = p->num_kv_heads < 8 ? p->num_kv_heads : 8;
  if ((p->page_size * hb) % 8 != 0 && p->page_size != 1) return TS_ERR_UNSUPPORTED;
  if ((int64_t)p->batch * p->num_q_heads * (int64_t)p->max_seq_len > ((int64_t)1 << 40)) return TS_ERR_UNSUPPORTED;
  if (p->num_initial < 0 || p->num_local < 0) return TS_ERR_INVALID_ARG;
  if (p->num_initial > (1 << 20) || p->num_local > (1 << 20)) return TS_ERR_UNSUPPORTED;
  return TS_OK;
}

// ---- scratch of the entry point that allocates nothing: one file-scope device array per GPU, kept until the
// process ends; the name below is a host-side stand-in, the device address comes from hipGetSymbolAddress
constexpr int kNoAllocMaxBatch = 16;
constexpr int kNoAllocMaxChunks = 256;                       // 2048-token chunks over the whole batch: 524288 tokens
constexpr size_t kNoAllocHist = 0;                           // uint32 [16][3][2048]
constexpr size_t kNoAllocState = kNoAllocHist + (size_t)kNoAllocMaxBatch * 3 * kTopkBins * 4;
constexpr size_t kNoAllocBlk = kNoAllocState + 1024;         // uint32 [256]
constexpr size_t kNoAllocList = kNoAllocBlk + 1024;          // uint2 [256][2048]
constexpr size_t kNoAllocBytes = kNoAllocList + (size_t)kNoAllocMaxChunks * kTopkChunk * 8;
static __device__ __align__(256) uint8_t scratch[kNoAllocBytes];
constexpr int kMaxDevices = 64;
static uint8_t* g_scratch_ptr[kMaxDevices] = {nullptr};

// device address of this GPU's copy of the array (looked up once per device, with that device current)
static int32_t noalloc_scratch(uint8_t** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TS_ERR_HIP;
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return TS_ERR_HIP;
    g_scratch_ptr[dev] = (uint8_t*)ptr;
  }
  *out = g_scratch_ptr[dev];
  return TS_OK;
}

}  // namespace ts

using namespace ts;

extern "C" {

int32_t ts_version(void) { return 300; }   // 0.3.0: the checked score calls and the ranked vote joined (0.2.0: the compact form, ts_topk_noalloc)

const char* ts_strerror(int32_t status) {
  switch (status) {
    case TS_OK: return "ok";
    case TS_ERR_INVALID_ARG: return "invalid argument";
    case TS_ERR_UNSUPPORTED: return "unsupported shape, dtype or page size";
    case TS_ERR_WORKSPACE: return "workspace missing or too small";
    case TS_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

int32_t ts_workspace_bytes(const ts_problem* p, int32_t k, size_t* bytes) {
  if (bytes == nullptr || k < 1) return TS_ERR_INVALID_ARG;
  const int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  const WsLayout w = ws_layout(p, k);
  // the decode attention merges at most kAttnMaxSplit partials: say so here, before a selection has been run for nothing
  if (p->chunk == 1 && w.attn_nsplit > kAttnMaxSplit) return TS_ERR_UNSUPPORTED;
  *bytes = w.total;
  return TS_OK;
}

int32_t ts_workspace_init(void* ws, size_t ws_bytes, void* stream) {
  if (ws == nullptr || ws_bytes == 0 || (ws_bytes & 3) != 0 || ((uintptr_t)ws & 255) != 0) return TS_ERR_INVALID_ARG;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, (hipStream_t)stream, (uint32_t*)ws, ws_bytes / 4);
  return hipGetLastError() == hipSuccess ? TS_OK : TS_ERR_HIP;
}

/* Tuning knobs used by the benchmark and the tests to compare kernel variants; not part of the
 * method.  variant: 0 = fma arithmetic, 1 = packed bf16 dot2, 2 = the matrix-core kernel where the shape
 * allows (the default; elsewhere as 1); wg: workgroups per sequence in the score pass (0 = automatic). */
int32_t ts_debug_set_score_variant(int32_t variant, int32_t wg, int32_t run_tiles) {
  if (variant < 0 || variant > 2 || wg < 0 || wg > kScoreMaxWg) return TS_ERR_INVALID_ARG;
  if (run_tiles != 0 && run_tiles != 1 && run_tiles != 2 && run_tiles != 4) return TS_ERR_INVALID_ARG;
  g_score_variant = variant; g_score_wg = wg; g_score_rr = run_tiles;
  return TS_OK;
}

int32_t ts_debug_event_create(void** event) {
  if (event == nullptr) return TS_ERR_INVALID_ARG;
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return TS_ERR_HIP;
  *event = (void*)e;
  return TS_OK;
}

int32_t ts_debug_event_destroy(void* event) {
  if (event == nullptr) return TS_ERR_INVALID_ARG;
  return hipEventDestroy((hipEvent_t)event) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_debug_event_elapsed_ms(void* start, void* stop, float* ms) {
  if (start == nullptr || stop == nullptr || ms == nullptr) return TS_ERR_INVALID_ARG;
  return hipEventElapsedTime(ms, (hipEvent_t)start, (hipEvent_t)stop) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_debug_set_score_timing_events(void* start, void* stop) {
  if ((start == nullptr) != (stop == nullptr)) return TS_ERR_INVALID_ARG;
  set_score_timing_events((hipEvent_t)start, (hipEvent_t)stop);
  set_codes_timing_events((hipEvent_t)start, (hipEvent_t)stop);
  return TS_OK;
}

int32_t ts_debug_set_codes_path(int32_t mfma, int32_t run_tiles) {
  if ((mfma != 0 && mfma != 1) || run_tiles < 0 || run_tiles > 8) return TS_ERR_INVALID_ARG;
  g_codes_mfma = mfma; g_codes_rr = run_tiles;
  return TS_OK;
}

int32_t ts_debug_set_topk_path(int32_t five_pass) {
  if (five_pass != 0 && five_pass != 1) return TS_ERR_INVALID_ARG;
  g_topk_five_pass = five_pass;
  return TS_OK;
}

// argument block and launch shape shared by the two forms of the score pass
static int32_t fill_score_args(const ts_problem* p, const void* q, float score_scale, const uint8_t* skip, void* ws,
                               size_t ws_bytes, size_t ws_need, ScoreArgs* a, const WsLayout& w) {
  if (q == nullptr || p->k_pool == nullptr) return TS_ERR_INVALID_ARG;
  if (!(score_scale >= 0.f) || !(score_scale < 1e30f)) return TS_ERR_INVALID_ARG;
  if (p->chunk != 1) return TS_ERR_UNSUPPORTED;
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || ws_bytes < ws_need) return TS_ERR_WORKSPACE;
  const int G = p->num_q_heads / p->num_kv_heads;
  a->q = (const uint8_t*)q; a->k_pool = (const uint8_t*)p->k_pool;
  a->page_indptr = p->page_indptr; a->page_indices = p->page_indices; a->seq_lens = p->seq_lens; a->skip = skip;
  a->partials = (float*)((uint8_t*)ws + w.score_partials);
  a->hdr = (uint32_t*)((uint8_t*)ws + w.hdr);
  a->H = p->num_q_heads; a->H_kv = p->num_kv_heads; a->P = p->page_size; a->p_shift = ilog2(p->page_size);
  a->max_seq_len = p->max_seq_len;
  a->HB = p->num_kv_heads < 8 ? p->num_kv_heads : 8; a->hb_shift = ilog2(a->HB); a->NU = p->num_kv_heads / a->HB;
  a->uniform_page = p->page_size >= (8 / a->HB);
  a->ncp_shift = ilog2(a->HB * G);
  a->scale = score_scale; a->c2 = score_scale * 1.44269504088896340736f;
  a->n_init = p->num_initial; a->n_local = p->num_local;
  a->RR = score_run_tiles_eff(p);
  return TS_OK;
}

static size_t score_lds_bytes(const ScoreArgs& a, int G) {
  size_t per_wave = (size_t)a.RR * kScoreTileTokens * ((a.HB * G + 3) & ~3);
  if (per_wave < 512) per_wave = 512;   // the closing statistics exchange needs 64 x 8 floats per wave
  return 4 * (per_wave + 64) * sizeof(float);   // + 64 block maxima per wave (compact form)
}

// Launch shape of the matrix-core score kernel (both forms): fills the wave-tile fields and a.RR, returns the
// workgroups per sequence.  A wave owns one run of consecutive tiles where the sequence is short enough, so that
// its output leaves in one burst at the end of its life; about 2048 waves per sequence (measured on MI355X:
// 131072 tokens 49 us with one tile per wave, 45.7 us with two).
static void mfma_launch_shape(const ts_problem* p, int G, bool dense, ScoreArgs* a, long* wg_out) {
  a->HB = G <= 4 ? 8 : 4; a->hb_shift = ilog2(a->HB); a->NU = p->num_kv_heads / a->HB;
  a->uniform_page = p->page_size >= (8 / a->HB);
  const long ntt = (p->max_seq_len + kScoreTileTokens - 1) / kScoreTileTokens;
  const int NU = a->NU;
  auto wgs_of = [&](int r) -> long {
    long n = ((ntt + r - 1) / r * NU + 3) / 4;
    return n > kScoreMaxWg ? (long)kScoreMaxWg : n;
  };
  int rr = g_codes_rr;
  if (rr <= 0) {
    // Longest run that still gives every CU two workgroups, among those the one whose workgroups fill the
    // rounds best: the CU holds floor(160 KiB / LDS) workgroups, three at most (registers), and a last round
    // that is half empty costs as much as a full one (786432 tokens of H 28/4: 8-tile runs 151 us, 6-tile runs
    // two full rounds).
    rr = 1;
    double best = -1.0;
    for (int r = 8; r >= 1; r -= (r > 2 ? 2 : 1)) {     // 8, 6, 4, 2, 1: odd run lengths measured slower throughout
      const long n = wgs_of(r);
      if (r > 1 && n < 512) continue;
      long per_cu = (long)(163840 / score_codes_mfma_lds_bytes(p->head_dim, G, r, dense));
      if (per_cu > 3) per_cu = 3;
      if (per_cu < 1) continue;
      const long slots = 256 * per_cu, rounds = (n + slots - 1) / slots;
      const double fill = (double)n / (double)(rounds * slots);
      if (fill > best + 0.05) { best = fill; rr = r; }
    }
  }
  if (rr > 8) rr = 8;
  while (rr > 1 && score_codes_mfma_lds_bytes(p->head_dim, G, rr, dense) > 163840) --rr;
  a->RR = rr;
  long wgl = wgs_of(rr);
  if (g_score_wg > 0) wgl = g_score_wg;
  *wg_out = wgl;
}

// Algorithm 1's state for the score launches that run the test themselves
static int32_t fill_selcache(const ts_problem* p, const void* q, const ts_selcache* sc, ScoreArgs* a) {
  if (sc == nullptr || sc->cached_q == nullptr || sc->cached_q_next == nullptr || sc->first == nullptr ||
      sc->first_next == nullptr || sc->reuse == nullptr) return TS_ERR_INVALID_ARG;
  if (!(sc->theta == sc->theta)) return TS_ERR_INVALID_ARG;
  const size_t es = p->dtype == TS_BF16 ? 2 : 4;
  const size_t qbytes = (size_t)p->batch * p->num_q_heads * p->head_dim * es;
  const uintptr_t c0 = (uintptr_t)sc->cached_q, c1 = (uintptr_t)sc->cached_q_next, q0 = (uintptr_t)q;
  if (((c0 | c1 | q0) & 15) != 0) return TS_ERR_INVALID_ARG;
  if (c0 < c1 + qbytes && c1 < c0 + qbytes) return TS_ERR_INVALID_ARG;              // the two C_Q buffers overlap
  if (q0 < c1 + qbytes && c1 < q0 + qbytes) return TS_ERR_INVALID_ARG;              // the query is overwritten
  const uintptr_t f0 = (uintptr_t)sc->first, f1 = (uintptr_t)sc->first_next;
  if (f0 < f1 + (size_t)p->batch && f1 < f0 + (size_t)p->batch) return TS_ERR_INVALID_ARG;
  a->sc_cached_q = (const uint8_t*)sc->cached_q; a->sc_cached_q_next = (uint8_t*)sc->cached_q_next;
  a->sc_first = sc->first; a->sc_first_next = sc->first_next; a->sc_reuse = sc->reuse; a->sc_theta = sc->theta;
  a->skip = nullptr;
  return TS_OK;
}

static int32_t paged_qk_scores_impl(const ts_problem* p, const void* q, const ts_selcache* sc, float* scores,
                                    float score_scale, const uint8_t* skip, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (scores == nullptr) return TS_ERR_INVALID_ARG;
  const WsLayout w = ws_layout(p, 1);
  ScoreArgs a{};
  st = fill_score_args(p, q, score_scale, skip, ws, ws_bytes, w.topk_blk, &a, w);   // needs the sections up to score_partials
  if (st != TS_OK) return st;
  if (sc != nullptr && (st = fill_selcache(p, q, sc, &a)) != TS_OK) return st;
  const int G = p->num_q_heads / p->num_kv_heads;
  a.scores = scores;
  if (g_score_variant == 2 && g_codes_mfma && (p->num_q_heads % 4) == 0 && (((uintptr_t)scores & 3) == 0) &&
      score_codes_mfma_supported(p->dtype, p->head_dim, G, p->num_kv_heads)) {
    long wgl = 0;
    mfma_launch_shape(p, G, true, &a, &wgl);
    const hipError_t e = launch_score_codes_mfma(p->head_dim, G, a, dim3((unsigned)wgl, p->batch),
                                                 score_codes_mfma_lds_bytes(p->head_dim, G, a.RR, true), (hipStream_t)stream);
    return e == hipSuccess ? TS_OK : TS_ERR_HIP;
  }
  a.vec_store = (p->num_q_heads % 4 == 0) && ((a.HB * G) % 4 == 0) && (((uintptr_t)scores & 15) == 0);
  const int wg = score_workgroups(p);
  const int variant = (p->dtype == TS_BF16) ? (g_score_variant != 0 ? 1 : 0) : 0;
  const hipError_t e = launch_score_decode(p->dtype, p->head_dim, G, variant, a, dim3(wg, p->batch), score_lds_bytes(a, G), (hipStream_t)stream);
  return e == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_paged_qk_scores(const ts_problem* p, const void* q, float* scores, float score_scale,
                           const uint8_t* skip, void* ws, size_t ws_bytes, void* stream) {
  return paged_qk_scores_impl(p, q, nullptr, scores, score_scale, skip, ws, ws_bytes, stream);
}

int32_t ts_paged_qk_scores_checked(const ts_problem* p, const void* q, const ts_selcache* sc, float* scores,
                                   float score_scale, void* ws, size_t ws_bytes, void* stream) {
  if (sc == nullptr) return TS_ERR_INVALID_ARG;
  return paged_qk_scores_impl(p, q, sc, scores, score_scale, nullptr, ws, ws_bytes, stream);
}

// ---- compact form of the selection: Algorithm 2 + Eq. 5 + TopK without the score matrix in memory

static int32_t paged_qk_codes_impl(const ts_problem* p, const void* q, const ts_selcache* sc, uint8_t* codes,
                                   float score_scale, const uint8_t* skip, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (codes == nullptr) return TS_ERR_INVALID_ARG;
  const WsLayout w = ws_layout(p, 1);
  ScoreArgs a{};
  st = fill_score_args(p, q, score_scale, skip, ws, ws_bytes, w.attn_out, &a, w);   // needs the block statistics too
  if (st != TS_OK) return st;
  if (sc != nullptr && (st = fill_selcache(p, q, sc, &a)) != TS_OK) return st;
  const int G = p->num_q_heads / p->num_kv_heads;
  a.codes = codes;
  a.blk_max = (float*)((uint8_t*)ws + w.blk_max); a.nblk = w.score_nblk;
  if (g_codes_mfma && (p->num_q_heads % 4) == 0 && (((uintptr_t)codes & 3) == 0) &&
      score_codes_mfma_supported(p->dtype, p->head_dim, G, p->num_kv_heads)) {
    long wgl = 0;
    mfma_launch_shape(p, G, false, &a, &wgl);
    // Bytes and block maxima that fit the chip's L2 (eight XCDs x 4 MiB) with room to spare stay there as dirty lines
    // until the kernel ends and cost the read stream nothing; more than that thrashes it, and streaming them past the
    // L2 is the cheaper way (measured, H 28/4: 524288 tokens 89.2 us cached / 90.2 streamed, 786432 tokens 142.0 / 135.7,
    // 1048576 tokens 184.5 / 176.1; H 32/8: 524288 tokens 167.4 / 168.7, 786432 tokens 267.4 / 254.4)
    a.nt_codes = (double)p->batch * p->max_seq_len * p->num_q_heads * 1.125 > 20.0 * 1048576.0;
    const hipError_t e = launch_score_codes_mfma(p->head_dim, G, a, dim3((unsigned)wgl, p->batch),
                                                 score_codes_mfma_lds_bytes(p->head_dim, G, a.RR, false), (hipStream_t)stream);
    return e == hipSuccess ? TS_OK : TS_ERR_HIP;
  }
  a.vec_store = (p->num_q_heads % 4 == 0) && ((a.HB * G) % 4 == 0) && (((uintptr_t)codes & 3) == 0);
  const int wg = score_workgroups(p);
  const int variant = (p->dtype == TS_BF16) ? (g_score_variant != 0 ? 1 : 0) : 0;
  const hipError_t e = launch_score_decode(p->dtype, p->head_dim, G, variant, a, dim3(wg, p->batch), score_lds_bytes(a, G), (hipStream_t)stream);
  return e == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_paged_qk_codes(const ts_problem* p, const void* q, uint8_t* codes, float score_scale,
                          const uint8_t* skip, void* ws, size_t ws_bytes, void* stream) {
  return paged_qk_codes_impl(p, q, nullptr, codes, score_scale, skip, ws, ws_bytes, stream);
}

int32_t ts_paged_qk_codes_checked(const ts_problem* p, const void* q, const ts_selcache* sc, uint8_t* codes,
                                  float score_scale, void* ws, size_t ws_bytes, void* stream) {
  if (sc == nullptr) return TS_ERR_INVALID_ARG;
  return paged_qk_codes_impl(p, q, sc, codes, score_scale, nullptr, ws, ws_bytes, stream);
}

int32_t ts_soft_vote_bounds(const ts_problem* p, const uint8_t* codes, float score_scale, float* row_stats,
                            float* vote_hi, float* vote_lo, const uint8_t* skip, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (codes == nullptr || row_stats == nullptr || vote_hi == nullptr) return TS_ERR_INVALID_ARG;   // vote_lo is optional
  if (!(score_scale >= 0.f) || !(score_scale < 1e30f)) return TS_ERR_INVALID_ARG;
  if (p->chunk != 1) return TS_ERR_UNSUPPORTED;
  const WsLayout w = ws_layout(p, 1);
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || ws_bytes < w.attn_out) return TS_ERR_WORKSPACE;
  BoundArgs a{};
  a.codes = codes; a.blk_max = (const float*)((uint8_t*)ws + w.blk_max);
  a.hdr = (const uint32_t*)((uint8_t*)ws + w.hdr);
  a.row_stats = row_stats; a.vote_hi = vote_hi; a.vote_lo = vote_lo;
  a.hist = (uint32_t*)((uint8_t*)ws + w.bound_hist);
  a.seq_lens = p->seq_lens; a.skip = skip;
  a.H = p->num_q_heads; a.max_seq_len = p->max_seq_len; a.nblk = w.score_nblk;
  a.n_init = p->num_initial; a.n_local = p->num_local;
  a.vec = (p->num_q_heads % 4 == 0) && (((uintptr_t)codes & 3) == 0);
  a.scale = score_scale;
  VoteArgs m{};
  m.partials = (const float*)((uint8_t*)ws + w.score_partials); m.hdr = a.hdr;
  m.row_stats_out = row_stats; m.skip = skip; m.H = p->num_q_heads; m.scale = score_scale;
  if (launch_stats_merge(m, p->batch, (hipStream_t)stream) != hipSuccess) return TS_ERR_HIP;
  return launch_vote_bounds(a, p->batch, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_topk_exact(const ts_problem* p, const void* q, const float* vote_hi, const float* row_stats,
                      float score_scale, int32_t k, int32_t* idx, int32_t* count, float* sel_votes, const uint8_t* skip,
                      void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (q == nullptr || vote_hi == nullptr || row_stats == nullptr || idx == nullptr || count == nullptr || k < 1)
    return TS_ERR_INVALID_ARG;
  if (p->k_pool == nullptr) return TS_ERR_INVALID_ARG;
  if (!(score_scale >= 0.f) || !(score_scale < 1e30f)) return TS_ERR_INVALID_ARG;
  if (p->chunk != 1) return TS_ERR_UNSUPPORTED;
  const WsLayout w = ws_layout(p, k);
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || ws_bytes < w.attn_out) return TS_ERR_WORKSPACE;
  if (w.topk_nblk > kTopkFinalMaxBlk) return TS_ERR_UNSUPPORTED;
  RefineArgs a{};
  a.t.head = p->num_initial; a.t.tail = p->num_local;
  a.t.votes = vote_hi; a.t.seq_lens = p->seq_lens; a.t.skip = skip; a.t.idx = idx; a.t.count = count;
  a.t.hist = (uint32_t*)((uint8_t*)ws + w.topk_hist);
  a.t.bound_hist = (uint32_t*)((uint8_t*)ws + w.bound_hist);
  a.t.sel_votes = sel_votes;
  a.t.state = (uint32_t*)((uint8_t*)ws + w.topk_state);
  a.t.blk = (uint32_t*)((uint8_t*)ws + w.topk_blk);
  a.t.list = (uint2*)((uint8_t*)ws + w.topk_list);
  a.t.k = k; a.t.max_seq_len = p->max_seq_len; a.t.nblk = w.topk_nblk; a.t.heads = 1;
  a.q = (const uint8_t*)q; a.k_pool = (const uint8_t*)p->k_pool;
  a.page_indptr = p->page_indptr; a.page_indices = p->page_indices; a.row_stats = row_stats;
  a.H = p->num_q_heads; a.H_kv = p->num_kv_heads; a.P = p->page_size; a.p_shift = ilog2(p->page_size);
  a.HB = p->num_kv_heads < 8 ? p->num_kv_heads : 8; a.hb_shift = ilog2(a.HB); a.NU = p->num_kv_heads / a.HB;
  a.scale = score_scale;
  // few chunks (131072 tokens: 64): several workgroups per chunk, so that the exact re-evaluation of the candidates
  // is spread over the machine (131072 tokens: 14.1 -> 9.9 us); many chunks fill it anyway
  a.parts = 256 / (w.topk_nblk * p->batch);
  if (a.parts > 4) a.parts = 4;
  if (a.parts < 1) a.parts = 1;
  const int G = p->num_q_heads / p->num_kv_heads;
  if (launch_topk_refine(p->dtype, p->head_dim, G, a, p->batch, (hipStream_t)stream) != hipSuccess) return TS_ERR_HIP;
  return launch_topk_final_full(a.t, p->batch, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_soft_vote(const ts_problem* p, const float* scores, float score_scale, float* row_stats, float* votes,
                     const uint8_t* skip, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (scores == nullptr || row_stats == nullptr || votes == nullptr) return TS_ERR_INVALID_ARG;
  if (!(score_scale >= 0.f) || !(score_scale < 1e30f)) return TS_ERR_INVALID_ARG;
  if (p->chunk != 1) return TS_ERR_UNSUPPORTED;
  const WsLayout w = ws_layout(p, 1);
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || ws_bytes < w.topk_blk) return TS_ERR_WORKSPACE;
  VoteArgs a{};
  a.partials = (const float*)((uint8_t*)ws + w.score_partials); a.hdr = (const uint32_t*)((uint8_t*)ws + w.hdr);
  a.scores = scores; a.row_stats = row_stats; a.row_stats_out = row_stats; a.votes = votes; a.seq_lens = p->seq_lens; a.skip = skip;
  a.H = p->num_q_heads; a.max_seq_len = p->max_seq_len; a.scale = score_scale;
  a.n_init = p->num_initial; a.n_local = p->num_local;
  return launch_soft_vote(a, p->batch, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_soft_vote_ranked(const ts_problem* p, const float* scores, float score_scale, float* row_stats, float* votes,
                            const uint8_t* skip, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (scores == nullptr || row_stats == nullptr || votes == nullptr) return TS_ERR_INVALID_ARG;
  if (!(score_scale >= 0.f) || !(score_scale < 1e30f)) return TS_ERR_INVALID_ARG;
  if (p->chunk != 1) return TS_ERR_UNSUPPORTED;
  const WsLayout w = ws_layout(p, 1);
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || ws_bytes < w.topk_blk) return TS_ERR_WORKSPACE;
  VoteArgs a{};
  a.partials = (const float*)((uint8_t*)ws + w.score_partials); a.hdr = (const uint32_t*)((uint8_t*)ws + w.hdr);
  a.scores = scores; a.row_stats = row_stats; a.row_stats_out = row_stats; a.votes = votes; a.seq_lens = p->seq_lens; a.skip = skip;
  a.H = p->num_q_heads; a.max_seq_len = p->max_seq_len; a.scale = score_scale;
  a.n_init = p->num_initial; a.n_local = p->num_local;
  a.rank_hist = (uint32_t*)((uint8_t*)ws + w.bound_hist);
  return launch_soft_vote_ranked(a, p->batch, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_topk(const ts_problem* p, const float* votes, int32_t k, int32_t* idx, int32_t* count,
                const uint8_t* skip, int32_t flags, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (votes == nullptr || idx == nullptr || count == nullptr || k < 1) return TS_ERR_INVALID_ARG;
  if ((flags & ~(TS_TOPK_FLAT_VOTES | TS_TOPK_VOTE_HIST)) != 0) return TS_ERR_INVALID_ARG;
  if ((flags & TS_TOPK_VOTE_HIST) != 0 && p->chunk != 1) return TS_ERR_UNSUPPORTED;
  const WsLayout w = ws_layout(p, k);
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || ws_bytes < w.attn_out) return TS_ERR_WORKSPACE;
  TopkArgs a{};
  a.head = p->num_initial;
  a.tail = (p->chunk > 1 ? p->chunk : 0) + p->num_local;   // the chunk's own tokens and the forced recent block
  a.votes = votes; a.seq_lens = p->seq_lens; a.skip = skip; a.idx = idx; a.count = count;
  a.hist = (uint32_t*)((uint8_t*)ws + w.topk_hist);
  a.state = (uint32_t*)((uint8_t*)ws + w.topk_state);
  a.blk = (uint32_t*)((uint8_t*)ws + w.topk_blk);
  // The short path finishes on one workgroup per sequence: right when few votes share the k-th vote's
  // quarter-octave (decode votes are peaked), slow when most do.  Votes summed over a chunk's queries are flat,
  // so chunk problems (and callers that say so) take the five-pass form, whose cost does not depend on the
  // distribution.
  a.list = (g_topk_five_pass || p->chunk > 1 || (flags & TS_TOPK_FLAT_VOTES)) ? nullptr : (uint2*)((uint8_t*)ws + w.topk_list);
  a.k = k; a.max_seq_len = p->max_seq_len; a.nblk = w.topk_nblk; a.heads = 1;
  if ((flags & TS_TOPK_VOTE_HIST) != 0) a.rep_hist = (uint32_t*)((uint8_t*)ws + w.bound_hist);
  return launch_topk(a, p->batch, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_topk_noalloc(const ts_problem* p, const float* votes, int32_t k, int32_t* idx, int32_t* count,
                        const uint8_t* skip, int32_t flags, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (votes == nullptr || idx == nullptr || count == nullptr || k < 1) return TS_ERR_INVALID_ARG;
  if ((flags & ~TS_TOPK_FLAT_VOTES) != 0) return TS_ERR_INVALID_ARG;
  const int nblk = (p->max_seq_len + kTopkChunk - 1) / kTopkChunk;
  if (p->batch > kNoAllocMaxBatch || (int64_t)p->batch * nblk > kNoAllocMaxChunks) return TS_ERR_UNSUPPORTED;
  uint8_t* base = nullptr;
  st = noalloc_scratch(&base);
  if (st != TS_OK) return st;
  TopkArgs a{};
  a.head = p->num_initial;
  a.tail = (p->chunk > 1 ? p->chunk : 0) + p->num_local;
  a.votes = votes; a.seq_lens = p->seq_lens; a.skip = skip; a.idx = idx; a.count = count;
  a.hist = (uint32_t*)(base + kNoAllocHist);
  a.state = (uint32_t*)(base + kNoAllocState);
  a.blk = (uint32_t*)(base + kNoAllocBlk);
  a.list = (g_topk_five_pass || p->chunk > 1 || (flags & TS_TOPK_FLAT_VOTES)) ? nullptr : (uint2*)(base + kNoAllocList);
  a.k = k; a.max_seq_len = p->max_seq_len; a.nblk = nblk; a.heads = 1;
  // the array keeps whatever the last call on this GPU left: the histograms must start at zero (a fill kernel,
  // not a memset node: callers may be under graph capture)
  hipLaunchKernelGGL(fill_zero_kernel, dim3(24), dim3(256), 0, (hipStream_t)stream, a.hist, (size_t)p->batch * 3 * kTopkBins);
  if (hipGetLastError() != hipSuccess) return TS_ERR_HIP;
  return launch_topk(a, p->batch, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

// ---- the ablation selection functions of Sec. 5.1 (Eq. 3, Eq. 4): other ways to fill `votes` for ts_topk

int32_t ts_sum_vote(const ts_problem* p, const float* scores, float* votes, const uint8_t* skip, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (scores == nullptr || votes == nullptr) return TS_ERR_INVALID_ARG;
  if (p->chunk != 1) return TS_ERR_UNSUPPORTED;
  VoteArgs a{};
  a.scores = scores; a.votes = votes; a.seq_lens = p->seq_lens; a.skip = skip;
  a.H = p->num_q_heads; a.max_seq_len = p->max_seq_len; a.n_init = p->num_initial; a.n_local = p->num_local;
  return launch_sum_vote(a, p->batch, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

// scratch of ts_head_vote: transposed scores, then histograms / state / chunk counts of B * H radix selects
struct HeadVoteLayout { size_t st, hist, state, blk, list, total; int nblk; };
static HeadVoteLayout head_vote_layout(const ts_problem* p) {
  HeadVoteLayout l{};
  const size_t V = (size_t)p->batch * p->num_q_heads;
  l.nblk = (p->max_seq_len + kTopkChunk - 1) / kTopkChunk;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  l.st = take(V * (size_t)p->max_seq_len * 4);
  l.hist = take(V * 3 * kTopkBins * 4);
  l.state = take(V * 8 * 4);
  l.blk = take(V * (size_t)l.nblk * 4);
  l.list = take(V * (size_t)l.nblk * kTopkChunk * 8);
  l.total = off;
  return l;
}

int32_t ts_head_vote_scratch_bytes(const ts_problem* p, size_t* bytes) {
  if (bytes == nullptr) return TS_ERR_INVALID_ARG;
  const int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  *bytes = head_vote_layout(p).total;
  return TS_OK;
}

int32_t ts_head_vote(const ts_problem* p, const float* scores, int32_t k_head, float* votes, const uint8_t* skip,
                     void* scratch, size_t scratch_bytes, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (scores == nullptr || votes == nullptr || k_head < 1) return TS_ERR_INVALID_ARG;
  if (p->chunk != 1) return TS_ERR_UNSUPPORTED;
  const HeadVoteLayout l = head_vote_layout(p);
  if (scratch == nullptr || ((uintptr_t)scratch & 255) != 0 || scratch_bytes < l.total) return TS_ERR_WORKSPACE;
  if ((size_t)p->batch * p->num_q_heads > 65535) return TS_ERR_UNSUPPORTED;   // grid.y of the radix-select passes
  hipStream_t s = (hipStream_t)stream;
  uint8_t* base = (uint8_t*)scratch;
  VoteArgs v{};
  v.scores = scores; v.seq_lens = p->seq_lens; v.skip = skip; v.H = p->num_q_heads; v.max_seq_len = p->max_seq_len;
  if (launch_transpose_scores(v, (float*)(base + l.st), p->batch, s) != hipSuccess) return TS_ERR_HIP;
  // the histograms must start at zero; the vote counters too (skipped sequences keep their votes)
  if (launch_fill_u32((uint32_t*)(base + l.hist), (l.state - l.hist) / 4, 0u, s) != hipSuccess) return TS_ERR_HIP;
  if (skip == nullptr) {
    if (launch_fill_u32((uint32_t*)votes, (size_t)p->batch * p->max_seq_len, 0u, s) != hipSuccess) return TS_ERR_HIP;
  } else {
    VoteArgs z = v; z.votes = votes;
    if (launch_zero_votes(z, p->batch, s) != hipSuccess) return TS_ERR_HIP;
  }
  TopkArgs a{};
  a.head = p->num_initial; a.tail = p->num_local;
  a.votes = (const float*)(base + l.st); a.seq_lens = p->seq_lens; a.skip = skip;
  a.hist = (uint32_t*)(base + l.hist); a.state = (uint32_t*)(base + l.state); a.blk = (uint32_t*)(base + l.blk);
  a.list = g_topk_five_pass ? nullptr : (uint2*)(base + l.list);
  a.k = k_head; a.max_seq_len = p->max_seq_len; a.nblk = l.nblk; a.heads = p->num_q_heads; a.vote_acc = votes;
  return launch_topk(a, p->batch * p->num_q_heads, s) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

static int32_t fill_prefill_args(const ts_problem* p, const void* q, float score_scale, void* ws, size_t ws_bytes,
                                 PrefillArgs* a) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (q == nullptr || p->k_pool == nullptr) return TS_ERR_INVALID_ARG;
  if (!(score_scale >= 0.f) || !(score_scale < 1e30f)) return TS_ERR_INVALID_ARG;
  if (p->chunk < 2 || p->dtype != TS_BF16) return TS_ERR_UNSUPPORTED;
  const WsLayout w = ws_layout(p, 1);
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || ws_bytes < w.total) return TS_ERR_WORKSPACE;
  a->q = (const uint8_t*)q; a->k_pool = (const uint8_t*)p->k_pool;
  a->page_indptr = p->page_indptr; a->page_indices = p->page_indices; a->seq_lens = p->seq_lens;
  a->stat_part = (float*)((uint8_t*)ws + w.pf_stat_part);
  a->vote_part = (float*)((uint8_t*)ws + w.pf_vote_part);
  a->B = p->batch; a->C = p->chunk; a->H = p->num_q_heads; a->H_kv = p->num_kv_heads;
  a->G = p->num_q_heads / p->num_kv_heads; a->D = p->head_dim; a->P = p->page_size; a->p_shift = ilog2(p->page_size);
  a->max_seq_len = p->max_seq_len; a->RB = w.pf_rb; a->TS = w.pf_ts;
  a->n_init = p->num_initial; a->n_local = p->num_local;
  a->scale = score_scale; a->c2 = score_scale * 1.44269504088896340736f;
  return TS_OK;
}

int32_t ts_chunk_row_stats(const ts_problem* p, const void* q, float score_scale, float* row_stats, void* ws,
                           size_t ws_bytes, void* stream) {
  PrefillArgs a{};
  const int32_t st = fill_prefill_args(p, q, score_scale, ws, ws_bytes, &a);
  if (st != TS_OK) return st;
  if (row_stats == nullptr) return TS_ERR_INVALID_ARG;
  a.row_stats_out = row_stats; a.row_stats = row_stats;
  return launch_prefill_stats(a, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_chunk_soft_vote(const ts_problem* p, const void* q, const float* row_stats, float score_scale, float* votes,
                           void* ws, size_t ws_bytes, void* stream) {
  PrefillArgs a{};
  const int32_t st = fill_prefill_args(p, q, score_scale, ws, ws_bytes, &a);
  if (st != TS_OK) return st;
  if (row_stats == nullptr || votes == nullptr) return TS_ERR_INVALID_ARG;
  a.row_stats = row_stats; a.votes = votes;
  return launch_prefill_votes(a, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_chunk_mean_query(const ts_problem* p, const void* q, void* q_mean, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (q == nullptr || q_mean == nullptr) return TS_ERR_INVALID_ARG;
  if (p->dtype != TS_BF16 || p->chunk > 65536) return TS_ERR_UNSUPPORTED;
  return launch_chunk_mean_query(q, q_mean, p->batch, p->chunk, p->num_q_heads * p->head_dim, (hipStream_t)stream) == hipSuccess
             ? TS_OK : TS_ERR_HIP;
}

int32_t ts_selcache_check(const ts_problem* p, const void* q, void* cached_q, uint8_t* first, float theta,
                          uint8_t* reuse, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (q == nullptr || cached_q == nullptr || first == nullptr || reuse == nullptr) return TS_ERR_INVALID_ARG;
  if (!(theta == theta)) return TS_ERR_INVALID_ARG;
  if (p->chunk != 1) return TS_ERR_UNSUPPORTED;
  SelcacheArgs a{};
  a.q = (const uint8_t*)q; a.cached_q = (uint8_t*)cached_q; a.first = first; a.reuse = reuse;
  a.n = p->num_q_heads * p->head_dim; a.dtype = p->dtype; a.theta = theta;
  return launch_selcache(a, p->batch, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int32_t ts_sparse_paged_attn(const ts_problem* p, const void* q, const int32_t* idx, int32_t idx_stride,
                             const int32_t* count, float sm_scale, void* out, float* lse, void* ws,
                             size_t ws_bytes, void* stream) {
  int32_t st = check_problem(p);
  if (st != TS_OK) return st;
  if (q == nullptr || idx == nullptr || count == nullptr || out == nullptr || idx_stride < 1) return TS_ERR_INVALID_ARG;
  if (p->k_pool == nullptr || p->v_pool == nullptr) return TS_ERR_INVALID_ARG;
  if (!(sm_scale == sm_scale)) return TS_ERR_INVALID_ARG;
  const WsLayout w = ws_layout(p, idx_stride);
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || ws_bytes < w.total) return TS_ERR_WORKSPACE;
  if (p->chunk > 1) {
    if (p->dtype != TS_BF16) return TS_ERR_UNSUPPORTED;
    ChunkAttnArgs c{};
    c.q = (const uint8_t*)q; c.k_pool = (const uint8_t*)p->k_pool; c.v_pool = (const uint8_t*)p->v_pool;
    c.page_indptr = p->page_indptr; c.page_indices = p->page_indices; c.seq_lens = p->seq_lens;
    c.idx = idx; c.count = count; c.slots = (int32_t*)((uint8_t*)ws + w.attn_slots);
    c.out = (uint8_t*)out; c.lse = lse;
    c.C = p->chunk; c.H = p->num_q_heads; c.H_kv = p->num_kv_heads; c.G = p->num_q_heads / p->num_kv_heads;
    c.D = p->head_dim; c.P = p->page_size; c.p_shift = ilog2(p->page_size); c.idx_stride = idx_stride;
    c.max_seq_len = p->max_seq_len; c.sm_scale = sm_scale;
    c.nsplit = w.attn_chunk_nsplit;
    c.n_init = p->num_initial; c.n_local = p->num_local;
    c.slot_stride = idx_stride + p->num_initial + p->num_local + p->chunk;
    c.part_o = (float*)((uint8_t*)ws + w.attn_chunk_o); c.part_ml = (float*)((uint8_t*)ws + w.attn_chunk_ml);
    return launch_sparse_attn_chunk(c, p->batch, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
  }
  if (w.attn_nsplit > kAttnMaxSplit) return TS_ERR_UNSUPPORTED;
  AttnArgs a{};
  a.q = (const uint8_t*)q; a.k_pool = (const uint8_t*)p->k_pool; a.v_pool = (const uint8_t*)p->v_pool;
  a.page_indptr = p->page_indptr; a.page_indices = p->page_indices; a.seq_lens = p->seq_lens;
  a.idx = idx; a.count = count; a.out = (uint8_t*)out; a.lse = lse;
  a.part_out = (float*)((uint8_t*)ws + w.attn_out);
  a.part_ml = (float*)((uint8_t*)ws + w.attn_ml);
  a.H = p->num_q_heads; a.H_kv = p->num_kv_heads; a.P = p->page_size; a.p_shift = ilog2(p->page_size);
  a.idx_stride = idx_stride; a.max_seq_len = p->max_seq_len; a.sm_scale = sm_scale;
  // chunks per workgroup: one while the chunks alone are few workgroups (a latency problem), four when there are many
  // thousands (a throughput problem: the next chunk's rows are in flight while a chunk is worked on).  Measured
  // with 2048 tokens per sequence, H 32/8: 32 sequences 63.8 -> 59.1 us, 64 sequences 142.3 -> 134.7 us; 8 sequences
  // (2048 chunk workgroups) 20.4 us with one chunk, 20.8 / 21.6 us with two / four.
  const long chunk_wgs = (long)w.attn_nsplit * p->num_kv_heads * p->batch;
  a.nch = chunk_wgs >= 8192 ? kAttnMaxRun : 1;
  if (a.nch > w.attn_nsplit) a.nch = w.attn_nsplit;
  if (a.nch < 1) a.nch = 1;
  if (a.nch > kAttnMaxRun) a.nch = kAttnMaxRun;
  a.nsplit = (w.attn_nsplit + a.nch - 1) / a.nch;
  a.n_init = p->num_initial; a.n_local = p->num_local;
  const int G = p->num_q_heads / p->num_kv_heads;
  return launch_sparse_attn_decode(p->dtype, p->head_dim, G, a, p->batch, (hipStream_t)stream) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

}  // extern "C"
