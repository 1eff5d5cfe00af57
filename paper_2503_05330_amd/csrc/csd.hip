// csd — consensus speculative drafting for N parallel sampling paths on gfx950.
//
// Host side of the C-ABI declared in csd.h: argument checks, workspace layout,
// launches.  The method is the one of "Speculative Decoding for Multi-Sample
// Inference": suffix match across paths (Eq. 3), layered token DAG with
// aggregated edge weights (Eq. 5), greedy layer-wise extraction (rule after
// Eq. 5, Algorithm 1), and the greedy acceptance check ("Draft acceptance").
//
// Nothing here is a dense contraction, so there is no MFMA: the work is
// integer compares, hash lookups, LDS hash-histogram atomics and wavefront
// reductions.  The step is latency-bound (a chain of a few dependent memory
// round trips per path, then the serial work of one wave), so the design
// minimises round trips, barriers and instruction count:
//   * one launch per decode step (append + draft + accept fused), also for
//     steps that append several tokens per path and for the accept-driven
//     loop (whose next input the step's own tail works out),
//   * per (problem, path) one wave64 that drafts and one that appends: no
//     workgroup barriers on the hot path,
//   * matches come from an incrementally updated n-gram hash index,
//   * the DAG of a row with up to 128 matches lives in the lanes of the wave
//     (sums by lane exchanges, ballots and DPP reductions); LDS tables take
//     the rows with more.
//
// Exactness: every weight is an integer (probabilities are quantised to
// 1/65536 at append), so atomics may accumulate in any order and the result is
// still unique.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "csd.h"
#include "csd_common.cuh"
#include "csd_dag.cuh"
#include "csd_index.cuh"
#include "csd_kernels.cuh"
#include "csd_match.cuh"

using namespace csd;

namespace {

// ---------------------------------------------------------------- host side

thread_local char g_hip_msg[256] = "no HIP error recorded";

int hip_fail(hipError_t e, const char* what) {
  snprintf(g_hip_msg, sizeof g_hip_msg, "HIP error in %s: %s", what, hipGetErrorString(e));
  return CSD_ERR_HIP;
}
#define CSD_HIP(call)                                   \
  do {                                                  \
    hipError_t e_ = (call);                             \
    if (e_ != hipSuccess) return hip_fail(e_, #call);   \
  } while (0)

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  size_t tok, pq, meta, status, gram, slices, total;
  int32_t n_slices;             // workgroups that share a row's scan (scan mode, few rows)
  int32_t meta_stride, eshift;
  uint32_t n_buckets;           // per (problem, gram length); 0 in scan mode
  size_t gram_words;
};

// Rows (problem, path) up to which a row's scan is shared by several workgroups.
constexpr int64_t kSlicedScanRows = 128;

// One-edit matching can go through the index when the query has at least two tokens (with
// one token every position is within one edit: a scan's job).  The index files positions
// under grams of max_query_len - 1 tokens then; for three-token queries those are pairs,
// the chains of frequent pairs get long, and the scan is the faster matcher.  With four-token
// queries the index is the faster one except for small problems (measured with one edit, us
// per step at full history, scan / index: 8 x 1024 positions per problem 12.0 / 11.5,
// 16 x 1024 14.2 / 12.6, 32 x 2048 21.6 / 19.4, 64 x 2048 35.3 / 29.4, 64 x 4096 52.9 / 24.5;
// only 32 x 4096, few long paths, went to the scan, 26.1 / 27.2): the scan's cost grows with
// the positions, the index's with the matches.  CSD_MATCH_AUTO therefore takes the index from
// four query tokens on when there are too many rows to slice the scan or a problem has 2^14
// positions or more.
// With query back-off a query without matches is searched again in shorter forms, which the
// index (grams of max_query_len tokens only) cannot serve: CSD_MATCH_AUTO takes the scan then.
constexpr int64_t kIndexedFuzzyPositions = 1 << 14;
int matcher_of(const csd_config* c) { return c->flags & 3; }
bool uses_index(const csd_config* c) {
  if (matcher_of(c) == CSD_MATCH_SCAN) return false;
  if (matcher_of(c) == CSD_MATCH_AUTO && (c->flags & CSD_QUERY_BACKOFF)) return false;
  if (c->max_edits == 0) return true;
  if (c->max_edits > 1) return false;                  // more than one edit: by scan only
  if (matcher_of(c) == CSD_MATCH_INDEX) return c->max_query_len >= 2;
  return c->max_query_len >= 4 && ((int64_t)c->n_problems * c->n_paths > kSlicedScanRows ||
                                   (int64_t)c->n_paths * c->max_len >= kIndexedFuzzyPositions);
}
int32_t tail_len_of(const csd_config* c) {
  return c->max_query_len + ((uses_index(c) && c->max_edits > 0) ? 1 : 0);
}

int validate(const csd_config* c) {
  if (!c) return CSD_ERR_INVALID_ARG;
  if (c->n_problems <= 0 || c->n_paths <= 0 || c->max_len <= 0) return CSD_ERR_INVALID_ARG;
  if (c->vocab <= 0 || c->vocab > CSD_MAX_VOCAB) return CSD_ERR_INVALID_ARG;
  if (c->max_query_len < 1 || c->max_query_len > CSD_MAX_QUERY_LEN) return CSD_ERR_INVALID_ARG;
  if (c->max_draft_len < 1 || c->max_draft_len > CSD_MAX_DRAFT_LEN) return CSD_ERR_INVALID_ARG;
  if (!(c->alpha >= 0.0f && c->alpha <= 1.0f)) return CSD_ERR_INVALID_ARG;
  if (c->score_mode != 0 && c->score_mode != 1) return CSD_ERR_INVALID_ARG;
  if ((int64_t)c->n_paths * c->max_len > CSD_MAX_POSITIONS) return CSD_ERR_INVALID_ARG;
  if ((int64_t)c->n_problems * c->n_paths > (1 << 24)) return CSD_ERR_INVALID_ARG;
  if (c->flags < 0 || c->flags > (3 | CSD_INCLUDE_SELF | CSD_QUERY_BACKOFF) || matcher_of(c) > CSD_MATCH_INDEX)
    return CSD_ERR_UNIMPLEMENTED;
  if (c->max_edits < 0) return CSD_ERR_INVALID_ARG;
  if (c->pool_mode < CSD_POOL_DAG || c->pool_mode > CSD_POOL_LIST) return CSD_ERR_INVALID_ARG;
  if (c->max_edits > CSD_MAX_EDITS) return CSD_ERR_UNIMPLEMENTED;
  if (c->max_edits > 1 && matcher_of(c) == CSD_MATCH_INDEX) return CSD_ERR_UNIMPLEMENTED;
  if (c->max_edits == 1 && matcher_of(c) == CSD_MATCH_INDEX && c->max_query_len < 2) return CSD_ERR_UNIMPLEMENTED;
  return CSD_OK;
}

Layout make_layout(const csd_config* c) {
  Layout l;
  size_t cells = (size_t)c->n_problems * c->n_paths * c->max_len;
  size_t rows = (size_t)c->n_problems * c->n_paths;
  size_t at = 0;
  // + 32 cells: the index lookup loads a match's whole continuation window (up to
  // CSD_MAX_DRAFT_LEN cells) wherever the path ends; lanes of the scan that have no position
  // load the first six cells of their problem's first path, and a span may read two cells
  // past its path
  l.tok = at;    at += align_up((cells + CSD_MAX_DRAFT_LEN) * sizeof(int32_t));
  l.pq = at;     at += align_up((cells + CSD_MAX_DRAFT_LEN) * sizeof(uint32_t));
  l.meta_stride = (1 + tail_len_of(c) + 3) / 4 * 4;
  l.eshift = 1;
  while ((1 << l.eshift) < c->max_len) ++l.eshift;
  l.meta = at;   at += 2 * align_up(rows * l.meta_stride * sizeof(int32_t));
  l.status = at; at += align_up(4 * sizeof(uint32_t));
  l.n_buckets = 0;
  l.gram_words = 0;
  l.gram = at;
  if (uses_index(c)) {
    // 15 slots per bucket and at least positions/8 buckets: load factor <= 8/15
    // (one-edit matching stores max_query_len + 1 postings per position)
    uint64_t positions = (uint64_t)c->n_paths * c->max_len * (c->max_edits > 0 ? c->max_query_len + 1 : 1);
    uint32_t nb = 4;
    while ((uint64_t)nb * 8 < positions) nb <<= 1;
    l.n_buckets = nb;
    l.gram_words = (size_t)c->n_problems * nb * kBucketWords;
    at += align_up(l.gram_words * sizeof(int32_t));
  }
  // scan mode with few rows: a row's scan is shared by up to 8 workgroups (at most 256 in all)
  l.n_slices = 1;
  l.slices = at;
  // (the hand-over between the slices costs about 5 us: worth it for one-edit matching and
  // for long histories)
  if (!uses_index(c) && rows <= (size_t)kSlicedScanRows && !(c->flags & CSD_QUERY_BACKOFF) &&
      (c->max_edits > 0 || (int64_t)c->n_paths * c->max_len >= 32768)) {
    while (l.n_slices < 8 && rows * (size_t)l.n_slices * 2 <= 256) l.n_slices *= 2;
    if (l.n_slices > 1)         // per row the match list and a state word
      at += align_up(rows * LdsScan::kMatch * sizeof(Match)) + align_up(rows * sizeof(u64));
  }
  l.total = at;
  return l;
}

uint32_t to_alpha_q(float alpha) {
  double x = (double)alpha * 65536.0;
  long r = lrint(x);            // default rounding mode: half to even
  return (uint32_t)(r < 0 ? 0 : (r > 65536 ? 65536 : r));
}

}  // namespace

// Scratch memory of csd_accept_loop_noalloc: one copy per GPU the library runs on, held until
// the process ends.  In host code the array's name is only a stand-in for the symbol: the
// device address comes from hipGetSymbolAddress, once per device (scratch_on_this_device).
constexpr size_t kStaticScratchBytes = CSD_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

struct csd_index {
  csd_config cfg;
  IndexView view;               // meta_old / meta_new are filled per launch
  int32_t* meta[2];             // double-buffered path ends (length + tail); `cur` is valid
  int cur;
  size_t gram_words;
  ScanSlices slices;
  bool indexed;
  uint32_t alpha_q;
  int64_t len_lo, len_hi;       // host-side bounds on every path's length
  int32_t steps_per_launch;     // csd_replay / csd_accept_loop: steps one launch runs (1: a launch per step)
};

namespace {
hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

IndexView view_in_place(const csd_index* h) {     // lengths read and written in the same buffer
  IndexView v = h->view;
  v.meta_old = h->meta[h->cur];
  v.meta_new = h->meta[h->cur];
  return v;
}

int check_draft_args(const csd_index* h, int32_t query_len, int32_t draft_len) {
  if (query_len < 1 || query_len > h->cfg.max_query_len) return CSD_ERR_INVALID_ARG;
  if (draft_len < 1 || draft_len > h->cfg.max_draft_len) return CSD_ERR_INVALID_ARG;
  return CSD_OK;
}

// From this many rows on (256 CUs x 4 rows of the regular layout are resident at once) the
// one-wave kernel runs with the small LDS layout.
constexpr int64_t kSmallLdsRows = 2048;
// Steps of up to this many tokens per path run fused in the one-wave kernel (a lane per new
// position: at most a wave's worth).
constexpr int32_t kFusedStepTokens = kWave;

void launch_draft(const csd_index* h, const IndexView& v, const StepIn& in, const DraftArgs& a,
                  hipStream_t st) {
  int64_t rows = (int64_t)v.P * v.N;
  const uint32_t grid = xcd_grid(rows);
  // scan mode, few rows: n_slices workgroups per row, the rows dealt to the 8 XCDs
  const ScanSlices sl = h->slices;
  const uint32_t scan_grid = sl.n > 1 ? (uint32_t)((rows + 7) / 8 * sl.n * 8) : grid;
  if (h->indexed && v.eps > 0) {                         // one edit through the variant index
    if (v.kmax <= 4) {                           // the usual gram lengths: predicates unrolled to 4
      if (a.L <= 8) step_wave_kernel<8, true, LdsWaveFuzzy, true, 4><<<grid, step_wave_threads(true), 0, st>>>(v, in, a);
      else if (a.L <= 16) step_wave_kernel<16, true, LdsWaveFuzzy, true, 4><<<grid, step_wave_threads(true), 0, st>>>(v, in, a);
      else step_wave_kernel<32, true, LdsWaveFuzzy, true, 4><<<grid, step_wave_threads(true), 0, st>>>(v, in, a);
    }
    else if (a.L <= 8) step_wave_kernel<8, true, LdsWaveFuzzy, true, CSD_MAX_QUERY_LEN><<<grid, step_wave_threads(true), 0, st>>>(v, in, a);
    else if (a.L <= 16) step_wave_kernel<16, true, LdsWaveFuzzy, true, CSD_MAX_QUERY_LEN><<<grid, step_wave_threads(true), 0, st>>>(v, in, a);
    else step_wave_kernel<32, true, LdsWaveFuzzy, true, CSD_MAX_QUERY_LEN><<<grid, step_wave_threads(true), 0, st>>>(v, in, a);
  } else if (!h->indexed) {
    // scan mode; the general kernels (POOLS) take the tree and list pools, own history,
    // back-off and steps of several tokens
    const bool general = a.pool_mode != CSD_POOL_DAG || v.options != 0 || in.n > 1;
    const bool fuzzy = v.eps > 0, q4 = v.kmax <= 4;
    auto* kernel = general ? (fuzzy ? (q4 ? step_scan_kernel<4, true, true> : step_scan_kernel<8, true, true>)
                                    : (q4 ? step_scan_kernel<4, true, false> : step_scan_kernel<8, true, false>))
                           : (fuzzy ? (q4 ? step_scan_kernel<4, false, true> : step_scan_kernel<8, false, true>)
                                    : (q4 ? step_scan_kernel<4, false, false> : step_scan_kernel<8, false, false>));
    kernel<<<scan_grid, kScanBlock, 0, st>>>(v, in, a, sl);
  } else if (a.pool_mode != CSD_POOL_DAG || v.options != 0 || in.n > 1) {   // tree and list pools, own history, back-off, steps of several tokens: the general kernels
    if (v.kmax <= 4) {                           // the usual gram lengths: loops unrolled to 4
      if (a.L <= 8) step_wave_kernel<8, true, LdsWave, false, 4><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
      else if (a.L <= 16) step_wave_kernel<16, true, LdsWave, false, 4><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
      else step_wave_kernel<32, true, LdsWave, false, 4><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
    }
    else if (a.L <= 8) step_wave_kernel<8, true, LdsWave, false, CSD_MAX_QUERY_LEN><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
    else if (a.L <= 16) step_wave_kernel<16, true, LdsWave, false, CSD_MAX_QUERY_LEN><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
    else step_wave_kernel<32, true, LdsWave, false, CSD_MAX_QUERY_LEN><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
  }
  else if (v.kmax <= 4) {                        // the usual gram lengths: loops unrolled to 4
    if (a.L <= 8 && rows >= kSmallLdsRows)       // more rows than fit the chip at once
      step_wave_many_kernel<4><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
    else if (a.L <= 8)
      step_wave_kernel<8, false, LdsWave, false, 4><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
    else if (a.L <= 16)
      step_wave_kernel<16, false, LdsWave, false, 4><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
    else
      step_wave_kernel<32, false, LdsWave, false, 4><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
  } else if (a.L <= 8 && rows >= kSmallLdsRows)
    step_wave_many_kernel<8><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
  else if (a.L <= 8)
    step_wave_kernel<8, false, LdsWave, false, 8><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
  else if (a.L <= 16)
    step_wave_kernel<16, false, LdsWave, false, 8><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
  else
    step_wave_kernel<32, false, LdsWave, false, 8><<<grid, step_wave_threads(false), 0, st>>>(v, in, a);
}

// The device-side loops (many steps per launch) serve exact matching through the index with
// grams of at most 4 tokens and at most 16 paths per problem (a wave per path, a workgroup
// per problem).
bool multi_step_ok(const csd_index* h) {
  return h->indexed && h->view.eps == 0 && h->view.kmax <= 4 && h->view.N <= 16;
}

template <bool LOOP>
void launch_multi(const csd_index* h, const MultiArgs& m, bool general, hipStream_t st) {
  const uint32_t grid = (uint32_t)h->view.P, block = (uint32_t)h->view.N * kWave;
  const int32_t L = m.a.L;
  if (LOOP || general) {
    if (L <= 8) step_multi_kernel<8, true, 4, LOOP><<<grid, block, 0, st>>>(h->view, m);
    else if (L <= 16) step_multi_kernel<16, true, 4, LOOP><<<grid, block, 0, st>>>(h->view, m);
    else step_multi_kernel<32, true, 4, LOOP><<<grid, block, 0, st>>>(h->view, m);
  } else {
    if (L <= 8) step_multi_kernel<8, false, 4, false><<<grid, block, 0, st>>>(h->view, m);
    else if (L <= 16) step_multi_kernel<16, false, 4, false><<<grid, block, 0, st>>>(h->view, m);
    else step_multi_kernel<32, false, 4, false><<<grid, block, 0, st>>>(h->view, m);
  }
}

// Host-side bounds on the paths' lengths as they were before a call: put back when the call's
// launch fails, so that an error leaves the handle as it was.
struct LengthBounds {
  csd_index* h;
  int64_t lo, hi;
  explicit LengthBounds(csd_index* index);
  int launched(const char* what);        // CSD_OK, or CSD_ERR_HIP with the bounds restored
};

// Host-side bookkeeping shared by csd_append and csd_step.
int note_append(csd_index* h, bool has_counts, int32_t n) {
  if (!has_counts && h->len_lo + n > h->cfg.max_len) return CSD_ERR_CAPACITY;
  if (!has_counts) h->len_lo += n;
  h->len_hi += n;
  if (h->len_hi > h->cfg.max_len) h->len_hi = h->cfg.max_len;
  return CSD_OK;
}

LengthBounds::LengthBounds(csd_index* index) : h(index), lo(index->len_lo), hi(index->len_hi) {}
int LengthBounds::launched(const char* what) {
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) return CSD_OK;
  h->len_lo = lo;
  h->len_hi = hi;
  return hip_fail(e, what);
}
}  // namespace

extern "C" {

int csd_workspace_bytes(const csd_config* cfg, size_t* out_bytes) {
  if (!out_bytes) return CSD_ERR_INVALID_ARG;
  int rc = validate(cfg);
  if (rc != CSD_OK) return rc;
  *out_bytes = make_layout(cfg).total;
  return CSD_OK;
}

int csd_create(const csd_config* cfg, void* d_workspace, size_t workspace_bytes, void* stream,
               csd_index** out_index) {
  if (!out_index) return CSD_ERR_INVALID_ARG;
  *out_index = nullptr;
  int rc = validate(cfg);
  if (rc != CSD_OK) return rc;
  if (!d_workspace) return CSD_ERR_INVALID_ARG;
  Layout l = make_layout(cfg);
  if (workspace_bytes < l.total || (reinterpret_cast<uintptr_t>(d_workspace) % kAlign) != 0)
    return CSD_ERR_WORKSPACE;
  csd_index* h = new (std::nothrow) csd_index;
  if (!h) return CSD_ERR_INVALID_ARG;
  h->cfg = *cfg;
  char* base = static_cast<char*>(d_workspace);
  size_t rows = (size_t)cfg->n_problems * cfg->n_paths;
  h->view.tok = reinterpret_cast<int32_t*>(base + l.tok);
  h->view.pq = reinterpret_cast<uint32_t*>(base + l.pq);
  h->meta[0] = reinterpret_cast<int32_t*>(base + l.meta);
  h->meta[1] = reinterpret_cast<int32_t*>(base + l.meta +
                                          align_up(rows * l.meta_stride * sizeof(int32_t)));
  h->cur = 0;
  h->view.meta_old = h->meta[0];
  h->view.meta_new = h->meta[0];
  h->view.meta_stride = l.meta_stride;
  h->view.tail_len = tail_len_of(cfg);
  h->view.eshift = l.eshift;
  h->view.status = reinterpret_cast<uint32_t*>(base + l.status);
  h->indexed = uses_index(cfg);
  h->view.gram = h->indexed ? reinterpret_cast<int32_t*>(base + l.gram) : nullptr;
  h->view.bucket_mask = h->indexed ? l.n_buckets - 1 : 0;
  h->gram_words = l.gram_words;
  h->slices = ScanSlices{l.n_slices, nullptr, nullptr};
  if (l.n_slices > 1) {
    h->slices.matches = reinterpret_cast<Match*>(base + l.slices);
    h->slices.state = reinterpret_cast<u64*>(base + l.slices +
                                             align_up(rows * LdsScan::kMatch * sizeof(Match)));
  }
  h->view.P = cfg->n_problems;
  h->view.N = cfg->n_paths;
  h->view.max_len = cfg->max_len;
  h->view.vocab = cfg->vocab;
  h->view.kmax = cfg->max_query_len;
  h->view.eps = cfg->max_edits;
  h->view.options = (cfg->flags >> 2) & 3;
  h->alpha_q = to_alpha_q(cfg->alpha);
  h->steps_per_launch = 1;
  rc = csd_reset(h, stream);
  if (rc != CSD_OK) {
    delete h;
    return rc;
  }
  *out_index = h;
  return CSD_OK;
}

int csd_destroy(csd_index* index) {
  if (!index) return CSD_ERR_INVALID_ARG;
  delete index;
  return CSD_OK;
}

int csd_reset(csd_index* h, void* stream) {
  if (!h) return CSD_ERR_INVALID_ARG;
  int64_t work = (int64_t)h->view.P * h->view.N * h->view.meta_stride;
  if ((int64_t)h->gram_words > work) work = (int64_t)h->gram_words;
  int64_t blocks = (work + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  reset_kernel<<<(uint32_t)blocks, 256, 0, as_stream(stream)>>>(view_in_place(h),
                                                                 (int64_t)h->gram_words, h->slices);
  CSD_HIP(hipGetLastError());
  h->len_lo = h->len_hi = 0;
  return CSD_OK;
}

int csd_append(csd_index* h, const int32_t* d_tokens, const float* d_probs,
               const int32_t* d_counts, int32_t n, void* stream) {
  if (!h || !d_tokens || n < 0) return CSD_ERR_INVALID_ARG;
  if (n == 0) return CSD_OK;
  LengthBounds before(h);
  int rc = note_append(h, d_counts != nullptr, n);
  if (rc != CSD_OK) return rc;
  int64_t rows = (int64_t)h->view.P * h->view.N;
  append_kernel<<<(uint32_t)rows, 256, 0, as_stream(stream)>>>(
      view_in_place(h), StepIn{d_tokens, d_probs, d_counts, n});
  return before.launched("csd_append");
}

int csd_draft(csd_index* h, int32_t query_len, int32_t draft_len, int32_t* d_draft_tokens,
              int32_t* d_draft_len, float* d_token_scores, float* d_path_scores, void* stream) {
  if (!h || !d_draft_tokens || !d_draft_len) return CSD_ERR_INVALID_ARG;
  int rc = check_draft_args(h, query_len, draft_len);
  if (rc != CSD_OK) return rc;
  DraftArgs a{query_len, draft_len, h->alpha_q, h->cfg.score_mode, h->cfg.pool_mode,
              d_draft_tokens, d_draft_len,
              d_token_scores, d_path_scores, nullptr, nullptr};
  launch_draft(h, view_in_place(h), StepIn{nullptr, nullptr, nullptr, 0}, a, as_stream(stream));
  CSD_HIP(hipGetLastError());
  return CSD_OK;
}

int csd_accept(csd_index* h, const int32_t* d_draft_tokens, const int32_t* d_draft_len,
               const int32_t* d_targets, int32_t draft_len, int32_t* d_accept_len, void* stream) {
  if (!h || !d_draft_tokens || !d_draft_len || !d_targets || !d_accept_len)
    return CSD_ERR_INVALID_ARG;
  if (draft_len < 1 || draft_len > h->cfg.max_draft_len) return CSD_ERR_INVALID_ARG;
  int64_t rows = (int64_t)h->view.P * h->view.N;
  accept_kernel<<<(uint32_t)((rows + 255) / 256), 256, 0, as_stream(stream)>>>(
      rows, draft_len, d_draft_tokens, d_draft_len, d_targets, d_accept_len);
  CSD_HIP(hipGetLastError());
  return CSD_OK;
}

int csd_step(csd_index* h, const int32_t* d_tokens, const float* d_probs, const int32_t* d_counts,
             int32_t n, int32_t query_len, int32_t draft_len, int32_t* d_draft_tokens,
             int32_t* d_draft_len, float* d_token_scores, float* d_path_scores,
             const int32_t* d_targets, int32_t* d_accept_len, void* stream) {
  if (!h || !d_tokens || n < 1 || n > CSD_MAX_STEP_TOKENS || !d_draft_tokens || !d_draft_len)
    return CSD_ERR_INVALID_ARG;
  if ((d_targets == nullptr) != (d_accept_len == nullptr)) return CSD_ERR_INVALID_ARG;
  int rc = check_draft_args(h, query_len, draft_len);
  if (rc != CSD_OK) return rc;
  LengthBounds before(h);
  rc = note_append(h, d_counts != nullptr, n);
  if (rc != CSD_OK) return rc;
  DraftArgs a{query_len, draft_len, h->alpha_q, h->cfg.score_mode, h->cfg.pool_mode,
              d_draft_tokens, d_draft_len,
              d_token_scores, d_path_scores, d_targets, d_accept_len};
  if (h->indexed && n != 1 && (h->view.eps > 0 || n > kFusedStepTokens)) {
    // the one-wave kernels fuse the append of a few tokens per path (exact matching) or of
    // one (one-edit matching); longer steps append first, with a workgroup per row
    int64_t rows = (int64_t)h->view.P * h->view.N;
    append_kernel<<<(uint32_t)rows, 256, 0, as_stream(stream)>>>(
        view_in_place(h), StepIn{d_tokens, d_probs, d_counts, n});
    launch_draft(h, view_in_place(h), StepIn{nullptr, nullptr, nullptr, 0}, a, as_stream(stream));
    return before.launched("csd_step");
  }
  IndexView v = h->view;
  v.meta_old = h->meta[h->cur];
  v.meta_new = h->meta[h->cur ^ 1];
  launch_draft(h, v, StepIn{d_tokens, d_probs, d_counts, n}, a, as_stream(stream));
  rc = before.launched("csd_step");
  if (rc == CSD_OK) h->cur ^= 1;
  return rc;
}

int csd_replay(csd_index* h, int32_t n_steps, const int32_t* d_tokens, const float* d_probs,
               int32_t query_len, int32_t draft_len, int32_t* d_draft_tokens, int32_t* d_draft_len,
               float* d_token_scores, float* d_path_scores, const int32_t* d_targets,
               int32_t* d_accept_len, int32_t fused, void* stream) {
  if (!h || n_steps < 0 || !d_tokens || !d_draft_tokens || !d_draft_len)
    return CSD_ERR_INVALID_ARG;
  if ((d_targets == nullptr) != (d_accept_len == nullptr)) return CSD_ERR_INVALID_ARG;
  int rc = check_draft_args(h, query_len, draft_len);
  if (rc != CSD_OK) return rc;
  if (h->len_lo + n_steps > h->cfg.max_len) return CSD_ERR_CAPACITY;
  size_t rows = (size_t)h->view.P * h->view.N;
  size_t L = (size_t)draft_len;
  if (fused && h->steps_per_launch > 1 && multi_step_ok(h)) {
    // the device-side loop: up to steps_per_launch steps per launch
    const bool general = h->cfg.pool_mode != CSD_POOL_DAG || h->view.options != 0;
    for (int32_t t = 0; t < n_steps;) {
      const int32_t chunk = n_steps - t < h->steps_per_launch ? n_steps - t : h->steps_per_launch;
      MultiArgs m{};
      m.n_steps = chunk;
      m.cur = h->cur;
      m.meta[0] = h->meta[0];
      m.meta[1] = h->meta[1];
      m.tokens = d_tokens + t * rows;
      m.probs = d_probs ? d_probs + t * rows : nullptr;
      m.a = DraftArgs{query_len, draft_len, h->alpha_q, h->cfg.score_mode, h->cfg.pool_mode,
                      d_draft_tokens + t * rows * L, d_draft_len + t * rows,
                      d_token_scores ? d_token_scores + t * rows * L : nullptr,
                      d_path_scores ? d_path_scores + t * rows : nullptr,
                      d_targets ? d_targets + t * rows * L : nullptr,
                      d_accept_len ? d_accept_len + t * rows : nullptr};
      LengthBounds before(h);
      h->len_lo += chunk;
      h->len_hi = h->len_hi + chunk > h->cfg.max_len ? h->cfg.max_len : h->len_hi + chunk;
      launch_multi<false>(h, m, general, as_stream(stream));
      rc = before.launched("csd_replay");
      if (rc != CSD_OK) return rc;
      h->cur ^= chunk & 1;
      t += chunk;
    }
    return CSD_OK;
  }
  for (int32_t t = 0; t < n_steps; ++t) {
    const int32_t* tk = d_tokens + t * rows;
    const float* pr = d_probs ? d_probs + t * rows : nullptr;
    int32_t* dt = d_draft_tokens + t * rows * L;
    int32_t* dl = d_draft_len + t * rows;
    float* ts = d_token_scores ? d_token_scores + t * rows * L : nullptr;
    float* ps = d_path_scores ? d_path_scores + t * rows : nullptr;
    const int32_t* tg = d_targets ? d_targets + t * rows * L : nullptr;
    int32_t* al = d_accept_len ? d_accept_len + t * rows : nullptr;
    if (fused) {
      rc = csd_step(h, tk, pr, nullptr, 1, query_len, draft_len, dt, dl, ts, ps, tg, al, stream);
    } else {
      rc = csd_append(h, tk, pr, nullptr, 1, stream);
      if (rc == CSD_OK) rc = csd_draft(h, query_len, draft_len, dt, dl, ts, ps, stream);
      if (rc == CSD_OK && tg) rc = csd_accept(h, dt, dl, tg, draft_len, al, stream);
    }
    if (rc != CSD_OK) return rc;
  }
  return CSD_OK;
}

static int accept_loop(csd_index* h, int32_t n_steps, const int32_t* d_future_tokens,
                       const float* d_future_probs, int32_t query_len, int32_t draft_len,
                       void* d_scratch, size_t scratch_bytes, int32_t* d_draft_tokens,
                       int32_t* d_draft_len, int32_t* d_accept_len, int32_t* d_path_len, void* stream) {
  if (!h || n_steps < 0 || !d_future_tokens || !d_scratch || !d_draft_tokens || !d_draft_len ||
      !d_accept_len || !d_path_len)
    return CSD_ERR_INVALID_ARG;
  int rc = check_draft_args(h, query_len, draft_len);
  if (rc != CSD_OK) return rc;
  const size_t rows = (size_t)h->view.P * h->view.N;
  const size_t L = (size_t)draft_len, n = L + 1;
  if (scratch_bytes < rows * (2 * n + L + 1) * 4 || (reinterpret_cast<uintptr_t>(d_scratch) & 3))
    return CSD_ERR_WORKSPACE;
  int32_t* step_tok = static_cast<int32_t*>(d_scratch);
  float* step_prob = reinterpret_cast<float*>(step_tok + rows * n);
  int32_t* targets = reinterpret_cast<int32_t*>(step_prob + rows * n);
  int32_t* step_cnt = targets + rows * L;
  hipStream_t st = as_stream(stream);
  if (h->indexed && h->view.eps == 0 && h->view.kmax <= 4 && n_steps > 0 &&
      scratch_bytes >= 2 * rows * (2 * n + L + 1) * 4) {
    // one launch per step: the fused step of up to L + 1 tokens per path, whose tail works out
    // the next step's input into the other half of the scratch memory
    int32_t* half[2] = {step_tok, step_tok + rows * (2 * n + L + 1)};
    auto tok_of = [&](int x) { return half[x]; };
    auto prob_of = [&](int x) { return reinterpret_cast<float*>(half[x] + rows * n); };
    auto targets_of = [&](int x) { return half[x] + rows * 2 * n; };
    auto cnt_of = [&](int x) { return half[x] + rows * (2 * n + L); };
    advance_kernel<<<(uint32_t)((rows + 255) / 256), 256, 0, st>>>(
        (int64_t)rows, h->cfg.max_len, (int32_t)n, draft_len, h->meta[h->cur], h->view.meta_stride,
        nullptr, d_future_tokens, d_future_probs, tok_of(0), d_future_probs ? prob_of(0) : nullptr,
        cnt_of(0), targets_of(0), d_path_len);
    CSD_HIP(hipGetLastError());
    if (h->steps_per_launch > 1 && multi_step_ok(h)) {
      // the device-side loop: up to steps_per_launch steps per launch (an even number, so
      // that every launch starts with the first set of step buffers)
      const int32_t most = h->steps_per_launch & ~1;
      for (int32_t s = 0; s < n_steps;) {
        const int32_t chunk = n_steps - s < most ? n_steps - s : most;
        MultiArgs m{};
        m.n_steps = chunk;
        m.cur = h->cur;
        m.meta[0] = h->meta[0];
        m.meta[1] = h->meta[1];
        for (int x = 0; x < 2; ++x) {
          m.step_tok[x] = tok_of(x);
          m.step_prob[x] = d_future_probs ? prob_of(x) : nullptr;
          m.step_cnt[x] = cnt_of(x);
          m.step_targets[x] = targets_of(x);
        }
        m.future_tok = d_future_tokens;
        m.future_prob = d_future_probs;
        m.path_len = d_path_len + (size_t)s * rows;
        m.n = (int32_t)n;
        m.a = DraftArgs{query_len, draft_len, h->alpha_q, h->cfg.score_mode, h->cfg.pool_mode,
                        d_draft_tokens + (size_t)s * rows * L, d_draft_len + (size_t)s * rows,
                        nullptr, nullptr, targets_of(0), d_accept_len + (size_t)s * rows};
        LengthBounds before(h);
        h->len_hi = h->len_hi + (int64_t)chunk * (int64_t)n > h->cfg.max_len
                        ? h->cfg.max_len : h->len_hi + (int64_t)chunk * (int64_t)n;
        launch_multi<true>(h, m, true, st);
        rc = before.launched("csd_accept_loop");
        if (rc != CSD_OK) return rc;
        h->cur ^= chunk & 1;
        s += chunk;
      }
      return CSD_OK;
    }
    const uint32_t grid = xcd_grid((int64_t)rows);
    for (int32_t s = 0; s < n_steps; ++s) {
      const int x = s & 1;
      LengthBounds before(h);
      rc = note_append(h, true, (int32_t)n);
      if (rc != CSD_OK) return rc;
      IndexView v = h->view;
      v.meta_old = h->meta[h->cur];
      v.meta_new = h->meta[h->cur ^ 1];
      const StepIn in{tok_of(x), d_future_probs ? prob_of(x) : nullptr, cnt_of(x), (int32_t)n};
      DraftArgs a{query_len, draft_len, h->alpha_q, h->cfg.score_mode, h->cfg.pool_mode,
                  d_draft_tokens + (size_t)s * rows * L, d_draft_len + (size_t)s * rows,
                  nullptr, nullptr, targets_of(x), d_accept_len + (size_t)s * rows};
      const LoopTail tail{d_future_tokens, d_future_probs, tok_of(x ^ 1),
                          d_future_probs ? prob_of(x ^ 1) : nullptr, cnt_of(x ^ 1), targets_of(x ^ 1),
                          d_path_len + (size_t)s * rows, (int32_t)n, h->cfg.max_len};
      if (draft_len <= 8) step_loop_kernel<8, 4><<<grid, step_wave_threads(false), 0, st>>>(v, in, a, tail);
      else if (draft_len <= 16) step_loop_kernel<16, 4><<<grid, step_wave_threads(false), 0, st>>>(v, in, a, tail);
      else step_loop_kernel<32, 4><<<grid, step_wave_threads(false), 0, st>>>(v, in, a, tail);
      rc = before.launched("csd_accept_loop");
      if (rc != CSD_OK) return rc;
      h->cur ^= 1;
    }
    return CSD_OK;
  }
  for (int32_t s = 0; s < n_steps; ++s) {
    const int32_t* settled = s > 0 ? d_accept_len + (size_t)(s - 1) * rows : nullptr;
    if (h->indexed) {                   // two launches: step input + append, then the draft
      LengthBounds before(h);
      rc = note_append(h, true, (int32_t)n);
      if (rc != CSD_OK) return rc;
      advance_append_kernel<<<(uint32_t)rows, 256, 0, st>>>(
          view_in_place(h), (int32_t)n, draft_len, settled, d_future_tokens, d_future_probs, step_tok,
          d_future_probs ? step_prob : nullptr, step_cnt, targets, d_path_len + (size_t)s * rows);
      DraftArgs a{query_len, draft_len, h->alpha_q, h->cfg.score_mode, h->cfg.pool_mode,
                  d_draft_tokens + (size_t)s * rows * L, d_draft_len + (size_t)s * rows,
                  nullptr, nullptr, targets, d_accept_len + (size_t)s * rows};
      launch_draft(h, view_in_place(h), StepIn{nullptr, nullptr, nullptr, 0}, a, st);
      rc = before.launched("csd_accept_loop");
      if (rc != CSD_OK) return rc;
      continue;
    }
    advance_kernel<<<(uint32_t)((rows + 255) / 256), 256, 0, st>>>(
        (int64_t)rows, h->cfg.max_len, (int32_t)n, draft_len, h->meta[h->cur], h->view.meta_stride,
        settled, d_future_tokens, d_future_probs, step_tok, d_future_probs ? step_prob : nullptr,
        step_cnt, targets, d_path_len + (size_t)s * rows);
    CSD_HIP(hipGetLastError());
    rc = csd_step(h, step_tok, d_future_probs ? step_prob : nullptr, step_cnt, (int32_t)n, query_len,
                  draft_len, d_draft_tokens + (size_t)s * rows * L, d_draft_len + (size_t)s * rows,
                  nullptr, nullptr, targets, d_accept_len + (size_t)s * rows, stream);
    if (rc != CSD_OK) return rc;
  }
  return CSD_OK;
}

int csd_accept_loop(csd_index* h, int32_t n_steps, const int32_t* d_future_tokens,
                    const float* d_future_probs, int32_t query_len, int32_t draft_len,
                    void* d_scratch, size_t scratch_bytes, int32_t* d_draft_tokens,
                    int32_t* d_draft_len, int32_t* d_accept_len, int32_t* d_path_len, void* stream) {
  return accept_loop(h, n_steps, d_future_tokens, d_future_probs, query_len, draft_len, d_scratch,
                     scratch_bytes, d_draft_tokens, d_draft_len, d_accept_len, d_path_len, stream);
}

// Device address of `scratch` on the current device, looked up once per device (each GPU
// holds its own copy of the array at its own address).
static int scratch_on_this_device(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex lock;
  static void* known[kMaxDevices] = {};
  int dev = -1;
  CSD_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return CSD_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> guard(lock);
  if (!known[dev]) {
    void* ptr = nullptr;
    CSD_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return CSD_ERR_HIP;
    known[dev] = ptr;
  }
  *out = known[dev];
  return CSD_OK;
}

int csd_accept_loop_noalloc(csd_index* h, int32_t n_steps, const int32_t* d_future_tokens,
                            const float* d_future_probs, int32_t query_len, int32_t draft_len,
                            int32_t* d_draft_tokens, int32_t* d_draft_len, int32_t* d_accept_len,
                            int32_t* d_path_len, void* stream) {
  if (!h) return CSD_ERR_INVALID_ARG;
  int rc = check_draft_args(h, query_len, draft_len);
  if (rc != CSD_OK) return rc;
  // two sets of step buffers (one launch per step); every word of a set is written by the
  // launch before the one that reads it, so nothing of an earlier call's contents is seen
  const size_t rows = (size_t)h->view.P * h->view.N;
  const size_t need = 2 * rows * (3 * (size_t)draft_len + 3) * 4;
  if (need > kStaticScratchBytes) return CSD_ERR_SCRATCH_LIMIT;
  void* ptr = nullptr;
  rc = scratch_on_this_device(&ptr);
  if (rc != CSD_OK) return rc;
  return accept_loop(h, n_steps, d_future_tokens, d_future_probs, query_len, draft_len, ptr, need,
                     d_draft_tokens, d_draft_len, d_accept_len, d_path_len, stream);
}

int csd_set_steps_per_launch(csd_index* h, int32_t steps) {
  if (!h || steps < 1) return CSD_ERR_INVALID_ARG;
  h->steps_per_launch = steps;
  return CSD_OK;
}

int csd_status(csd_index* h, uint32_t* host_flags, void* stream) {
  if (!h || !host_flags) return CSD_ERR_INVALID_ARG;
  CSD_HIP(hipMemcpyAsync(host_flags, h->view.status, sizeof(uint32_t), hipMemcpyDeviceToHost,
                         as_stream(stream)));
  CSD_HIP(hipStreamSynchronize(as_stream(stream)));
  return CSD_OK;
}

int csd_dump_matches(csd_index* h, int32_t query_len, int32_t* d_match_je, int32_t* d_match_off,
                     int64_t cap, void* stream) {
  if (!h || !d_match_off || cap < 0 || (cap > 0 && !d_match_je)) return CSD_ERR_INVALID_ARG;
  if (query_len < 1 || query_len > h->cfg.max_query_len) return CSD_ERR_INVALID_ARG;
  hipStream_t st = as_stream(stream);
  int32_t rows = h->view.P * h->view.N;
  int32_t words = (int32_t)(((int64_t)h->view.N * h->view.max_len + 31) / 32);
  uint32_t* bits = nullptr;
  int32_t* counts = nullptr;
  CSD_HIP(hipMalloc(&bits, (size_t)rows * words * sizeof(uint32_t)));
  hipError_t e = hipMalloc(&counts, ((size_t)rows + 1) * sizeof(int32_t));
  if (e != hipSuccess) { (void)hipFree(bits); return hip_fail(e, "hipMalloc"); }
  int rc = CSD_OK;
  int32_t total = 0;
  IndexView v = view_in_place(h);
  const StepIn no_step{nullptr, nullptr, nullptr, 0};
  do {
    e = hipMemsetAsync(bits, 0, (size_t)rows * words * sizeof(uint32_t), st);
    if (e != hipSuccess) break;
    if (h->indexed && v.eps > 0)
      dump_match_bits_wave_kernel<true><<<xcd_grid(rows), kWave, 0, st>>>(v, no_step, query_len,
                                                                          bits, words);
    else if (h->indexed)
      dump_match_bits_wave_kernel<false><<<xcd_grid(rows), kWave, 0, st>>>(v, no_step, query_len,
                                                                           bits, words);
    else
      dump_match_bits_scan_kernel<<<xcd_grid(rows), kScanBlock, 0, st>>>(v, no_step, query_len,
                                                                        bits, words);
    count_bits_kernel<<<rows, 256, 0, st>>>(bits, words, counts);
    offsets_kernel<<<1, 1, 0, st>>>(counts, rows, d_match_off, counts + rows);
    expand_bits_kernel<<<rows, 64, 0, st>>>(bits, words, h->view.max_len, d_match_off, d_match_je,
                                            cap);
    e = hipGetLastError();
    if (e != hipSuccess) break;
    e = hipMemcpyAsync(&total, d_match_off + rows, sizeof(int32_t), hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) break;
    e = hipStreamSynchronize(st);
  } while (0);
  (void)hipFree(bits);
  (void)hipFree(counts);
  if (e != hipSuccess) return hip_fail(e, "csd_dump_matches");
  if ((int64_t)total > cap) rc = CSD_ERR_CAPACITY;
  return rc;
}

int csd_dump_edges(csd_index* h, int32_t query_len, int32_t draft_len, int32_t* d_edge_duv,
                   uint64_t* d_edge_cs, int32_t* d_edge_off, int64_t cap, void* stream) {
  if (!h || !d_edge_off || cap < 0 || (cap > 0 && (!d_edge_duv || !d_edge_cs)))
    return CSD_ERR_INVALID_ARG;
  int rc = check_draft_args(h, query_len, draft_len);
  if (rc != CSD_OK) return rc;
  hipStream_t st = as_stream(stream);
  int32_t rows = h->view.P * h->view.N;
  u64* tmp = nullptr;
  int32_t* counts = nullptr;
  size_t tmp_elems = (size_t)rows * kDumpStride;
  CSD_HIP(hipMalloc(&tmp, 2 * tmp_elems * sizeof(u64)));
  hipError_t e = hipMalloc(&counts, ((size_t)rows + 1) * sizeof(int32_t));
  if (e != hipSuccess) { (void)hipFree(tmp); return hip_fail(e, "hipMalloc"); }
  int32_t tail[2] = {0, 0};   // total rows, bad flag
  IndexView v = view_in_place(h);
  const StepIn no_step{nullptr, nullptr, nullptr, 0};
  do {
    if (h->indexed && v.eps > 0)
      dump_edge_rows_wave_kernel<32, true><<<xcd_grid(rows), kWave, 0, st>>>(
          v, no_step, query_len, draft_len, tmp, tmp + tmp_elems, counts);
    else if (h->indexed && draft_len <= 8)
      dump_edge_rows_wave_kernel<8, false><<<xcd_grid(rows), kWave, 0, st>>>(
          v, no_step, query_len, draft_len, tmp, tmp + tmp_elems, counts);
    else if (h->indexed && draft_len <= 16)
      dump_edge_rows_wave_kernel<16, false><<<xcd_grid(rows), kWave, 0, st>>>(
          v, no_step, query_len, draft_len, tmp, tmp + tmp_elems, counts);
    else if (h->indexed)
      dump_edge_rows_wave_kernel<32, false><<<xcd_grid(rows), kWave, 0, st>>>(
          v, no_step, query_len, draft_len, tmp, tmp + tmp_elems, counts);
    else
      dump_edge_rows_scan_kernel<<<xcd_grid(rows), kScanBlock, 0, st>>>(
          v, no_step, query_len, draft_len, tmp, tmp + tmp_elems, counts);
    offsets_kernel<<<1, 1, 0, st>>>(counts, rows, d_edge_off, counts + rows);
    scatter_edges_kernel<<<rows, 256, 0, st>>>(tmp, tmp + tmp_elems, d_edge_off, d_edge_duv,
                                               d_edge_cs, cap);
    e = hipGetLastError();
    if (e != hipSuccess) break;
    e = hipMemcpyAsync(&tail[0], d_edge_off + rows, sizeof(int32_t), hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) break;
    e = hipMemcpyAsync(&tail[1], counts + rows, sizeof(int32_t), hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) break;
    e = hipStreamSynchronize(st);
  } while (0);
  (void)hipFree(tmp);
  (void)hipFree(counts);
  if (e != hipSuccess) return hip_fail(e, "csd_dump_edges");
  if ((int64_t)tail[0] > cap || tail[1] != 0) return CSD_ERR_CAPACITY;
  return CSD_OK;
}

int csd_debug_copy(void* d_dst, const void* d_src, size_t bytes, void* stream) {
  if (!d_dst || !d_src || bytes % 16 != 0) return CSD_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(d_dst) | reinterpret_cast<uintptr_t>(d_src)) % 16 != 0)
    return CSD_ERR_INVALID_ARG;
  int64_t n = (int64_t)(bytes / 16);
  if (n == 0) return CSD_OK;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  copy_kernel<<<(uint32_t)blocks, 256, 0, as_stream(stream)>>>(
      static_cast<const uint4*>(d_src), static_cast<uint4*>(d_dst), n);
  CSD_HIP(hipGetLastError());
  return CSD_OK;
}

#ifdef CSD_STAMPS
// Timing build only: copies the stamps of the last launches to the host (after a device
// synchronisation by the caller).
int csd_read_stamps(unsigned long long* host, size_t count) {
  CSD_HIP(hipMemcpyFromSymbol(host, HIP_SYMBOL(csd::g_stamps), count * sizeof(unsigned long long)));
  return CSD_OK;
}
#endif

const char* csd_strerror(int err) {
  switch (err) {
    case CSD_OK: return "ok";
    case CSD_ERR_INVALID_ARG: return "invalid argument";
    case CSD_ERR_CAPACITY: return "capacity exceeded";
    case CSD_ERR_WORKSPACE: return "workspace too small or misaligned";
    case CSD_ERR_HIP: return g_hip_msg;
    case CSD_ERR_UNIMPLEMENTED: return "configuration not implemented in this build";
    case CSD_ERR_SCRATCH_LIMIT: return "input exceeds the fixed scratch array of the non-allocating entry point";
    default: return "unknown csd error";
  }
}

}  // extern "C"
