// csd — the kernels: reset, append, the decode step (a drafting and an
// appending wave per path in index mode, one 1024-thread workgroup per path —
// or several, sharing its scan — in scan mode), accept, the stand-in model of
// the accept-driven loop, and the kernels behind the debug dumps.
#pragma once

#include "csd_common.cuh"
#include "csd_dag.cuh"
#include "csd_index.cuh"
#include "csd_match.cuh"

namespace csd {

__global__ __launch_bounds__(256) void reset_kernel(IndexView ix, int64_t gram_words, ScanSlices sl) {
  int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * 256;
  int64_t rows = (int64_t)ix.P * ix.N;
  if (sl.n > 1)
    for (int64_t r = t; r < rows; r += stride) sl.state[r] = 0ull;
  for (int64_t r = t; r < rows * ix.meta_stride; r += stride) ix.meta_new[r] = 0;
  for (int64_t w = t; w < gram_words; w += stride) ix.gram[w] = (w & (kBucketWords - 1)) ? -1 : 0;
  if (t == 0) *ix.status = 0u;
}

// Append only: one workgroup per (problem, path); the meta row is updated in place.
__global__ __launch_bounds__(256) void append_kernel(IndexView ix, StepIn in) {
  int32_t row = blockIdx.x;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);
  int32_t old_i = c.y.old_len(c.i);
  int32_t new_i = c.y.new_len(c.i, old_i);
  append_row<256, true>(ix, c.y, p, c.i, old_i, new_i, c.tid);
}

// Draft tokens, scores, length and (optionally) accept length of one row.
// `target` is the lane's target token (lanes < L), loaded by the caller.
template <int BLOCK>
__device__ __forceinline__ void write_outputs(const DraftArgs& a, int32_t row, const DraftOut& o,
                                              int tid) {
  const int32_t L = a.L;
  bool live = tid < o.n;
  if (tid < L) {
    a.draft_tokens[(int64_t)row * L + tid] = live ? o.tok : -1;
    if (a.token_scores) a.token_scores[(int64_t)row * L + tid] = live ? key_to_score(o.key) : 0.0f;
  }
  if (tid == 0) {
    a.draft_len[row] = o.n;
    if (a.path_scores) a.path_scores[row] = key_to_score(o.key_sum);
  }
}

// "Draft acceptance": the first lane whose draft token differs from its target.
// Returns the accept length (the same in every lane).
__device__ __forceinline__ int32_t write_accept(const DraftArgs& a, int32_t row, const DraftOut& o,
                                                int32_t target, int tid) {
  bool same = tid < o.n && target == o.tok;
  u64 differs = wave_ballot(!same);
  const int32_t accepted = differs ? (int32_t)__ffsll((long long)differs) - 1 : kWave;
  if (tid == 0) a.accept_len[row] = accepted;
  return accepted;
}

// Lengths of the first LDS::kLens paths into LDS (the scan reads them per tile).
// The caller synchronises the workgroup before using them.
template <int BLOCK, class LDS>
__device__ __forceinline__ void cache_lens(LDS& s, const Paths& y, int tid) {
  for (int32_t j = tid; j < y.N && j < LDS::kLens; j += BLOCK) {
    int32_t old_j = y.old_len(j);
    s.len_old[j] = old_j;
    s.len_new[j] = y.new_len(j, old_j);
  }
}

// The continuations of the M listed matches into windows of 2 L words (tokens, then
// probabilities), one (match, layer) instance per thread; ends with a workgroup barrier.
template <int BLOCK, class LDS>
__device__ __forceinline__ void fetch_windows(LDS& s, const Ctx& c, int32_t M, int32_t L,
                                              int32_t* windows) {
  for (int32_t idx = c.tid; idx < M * L; idx += BLOCK) {
    const int32_t mi = idx / L, d = idx - mi * L + 1;
    uint32_t u, v;
    u64 w;
    if (layer_instance(c.y, s.match[mi], d, 0u, u, v, w)) {
      windows[mi * 2 * L + d - 1] = (int32_t)v;
      windows[mi * 2 * L + L + d - 1] = (int32_t)cs_sum(w);
    }
  }
  block_sync<BLOCK>();
}

// Scan mode.  One 1024-thread workgroup per (problem, path): [append] -> match
// by scan (Eq. 3, or Eq. 4 with one edit) -> DAG (Eq. 5) -> greedy walk ->
// [accept].  With in.n > 0 the launch also performs the step's append; every
// workgroup then reads the other paths through `Paths`, which never touches
// cells written by this launch.  The histories are read straight from memory:
// the q + 1 tokens a position compares are shared with its neighbours in the
// wave, so all but the first load of a line hit the CU's vector cache, and no
// workgroup barrier is needed per tile as staging through LDS would.
// POOLS: also compiled for the tree and list pools (kept out of the DAG-only
// kernels, whose code and register footprint they would enlarge).
// With sl.n > 1 a row's scan is shared by sl.n workgroups (few rows: the scan is
// bound by instruction issue on the row's CU, and most CUs would be idle); the
// one that finishes last does the rest of the row's work.
// FUZZY: matching tolerates one edit (compiled apart from the exact kernel: code a launch
// does not run still costs it time).
// QC: compile-time bound (4 or 8) of the query length: the comparison loops are unrolled to it.
template <int QC, bool POOLS, bool FUZZY>
__global__ __launch_bounds__(kScanBlock) void step_scan_kernel(IndexView ix, StepIn in,
                                                               DraftArgs a, ScanSlices sl) {
  constexpr int BLOCK = kScanBlock;
  fetch_kernel_arguments<sizeof(IndexView) + sizeof(StepIn) + sizeof(DraftArgs) + sizeof(ScanSlices)>();
  __shared__ LdsScan s;
  __shared__ int32_t sh_base, sh_total, sh_last;
  int32_t row, slice = 0;
  if (sl.n == 1) {
    row = xcd_row(ix.P * ix.N);
  } else {                              // XCD x takes rows x, x + 8, ..: a row's slices share an L2
    int32_t idx = (int32_t)(blockIdx.x >> 3);
    slice = idx & (sl.n - 1);
    row = (idx / sl.n) * 8 + (int32_t)(blockIdx.x & 7);
    if (row >= ix.P * ix.N) row = -1;
  }
  if (row < 0) return;
  const int32_t unit = row * 8 + slice;                  // (timing build only)
  CSD_STAMP(unit, 0, CSD_CLOCK());
  CSD_STAMP(unit, 6, 0ull);
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);
#ifdef CSD_STAMPS
  c.unit = unit;
#endif
  int32_t st_i = in.n == 1 ? c.y.st[c.i] : 0;           // (first: the head's lengths wait for its load)
  Head me = load_head(c.y, ix.tail_len, c.i);           // length and newest tokens in one read
  const int32_t old_i = me.old_len;
  c.len_i = me.new_len;
  cache_lens<BLOCK>(s, c.y, c.tid);
  if (in.n > 0 && slice == 0) append_row<BLOCK, true>(ix, c.y, p, c.i, old_i, c.len_i, c.tid);
  if (in.n <= 1) {                                       // the query follows from what is loaded
    int32_t cnt_i = c.len_i - old_i;
    c.q = a.k < c.len_i ? a.k : c.len_i;
#pragma unroll
    for (int x = 0; x < CSD_MAX_QUERY_LEN; ++x) {
      int32_t v = 0;
      if (x < c.q) v = x < cnt_i ? st_i : pick(me.tail, x - cnt_i);
      c.Q[x] = v;
    }
  } else {
    load_query(c, a.k, old_i);
  }
  if (c.tid == 0) s.n_match = 0;
  lds_barrier<BLOCK>();                 // lengths and the empty list are in LDS; the append's stores,
                                        // which nothing in this launch reads, need not have landed
  DraftOut o;
  const int32_t L = a.L;
  CSD_STAMP(unit, 1, CSD_CLOCK());
  if (c.q > 0) {
    ListSink<LdsScan> sink{&s};
    match_scan<BLOCK, FUZZY, QC>(s, c, sink, slice, sl.n);
    block_sync<BLOCK>();
    int32_t M = s.n_match;
    CSD_STAMP(unit, 2, CSD_CLOCK());
    CSD_STAMP(unit, 8, (unsigned long long)M);
    if (POOLS && (ix.options & 2)) {
      // query back-off (never with slices): no match, so the query loses its oldest token and
      // the scan runs again; every thread sees the same M and q, so the barriers pair up
      while (M == 0 && c.q > 1) {
        block_sync<BLOCK>();            // everybody has read the count before anybody pushes again
        --c.q;
        match_scan<BLOCK, FUZZY, QC>(s, c, sink);
        block_sync<BLOCK>();
        M = s.n_match;
      }
    }
    if (sl.n > 1) {
      // hand this slice's matches to the row's list in memory.  One 64-bit word per row
      // holds the matches listed so far (low half) and the slices finished, over all
      // launches (high half): a slice reserves its part of the list with one atomic and
      // signs off with a second one, whose result tells the last slice the row's total
      Match* listed = sl.matches + (int64_t)row * LdsScan::kMatch;
      if (c.tid == 0) sh_base = (int32_t)(uint32_t)atomicAdd(&sl.state[row], (u64)(uint32_t)M);
      block_sync<BLOCK>();
      for (int32_t m = c.tid; m < M && m < LdsScan::kMatch; m += BLOCK)
        if (sh_base + m < LdsScan::kMatch) listed[sh_base + m] = s.match[m];
      block_sync<BLOCK>();              // every wave's stores have left the CU
      // (while wave 0 signs off, the others prepare the tables of the walk that rows of
      // 65 .. 1024 matches take: wasted on all slices but the last, which would wait here anyway)
      if (!POOLS || a.pool_mode == CSD_POOL_DAG) walk_tab_clear<BLOCK>(s, c.tid, kWave);
      if (c.tid == 0) {
        // one wave fences for the workgroup (a device-scope fence writes the L2 back: sixteen
        // of them in a row cost more than the scan): list entries before the sign-off, the
        // sign-off before the reads below
        __threadfence();
        const u64 seen = atomicAdd(&sl.state[row], 1ull << 32);
        sh_last = ((uint32_t)(seen >> 32) & (uint32_t)(sl.n - 1)) == (uint32_t)(sl.n - 1);
        sh_total = (int32_t)(uint32_t)seen;   // every slice has reserved before it signs off
        // the next launch starts with an empty list (nobody else touches the word any more)
        if (sh_last) sl.state[row] = ((seen >> 32) + 1ull) << 32;
        __threadfence();
      }
      block_sync<BLOCK>();
      CSD_STAMP(unit, 3, CSD_CLOCK());
      if (!sh_last) return;             // the last slice goes on with all matches of the row
      M = sh_total;
      for (int32_t m = c.tid; m < M && m < LdsScan::kMatch; m += BLOCK) s.match[m] = listed[m];
      if (c.tid == 0) s.n_match = M;
      block_sync<BLOCK>();
    }
    CSD_STAMP(unit, 4, CSD_CLOCK());
    CSD_STAMP(unit, 9, (unsigned long long)M);
    if (POOLS && M > 0 && a.pool_mode != CSD_POOL_DAG) {
      auto each = [&](auto f) {
        if (M <= LdsScan::kMatch) {
          for (int32_t m = c.tid; m < M; m += BLOCK) f(s.match[m], m);
        } else {
          auto g = [&](Match found) { f(found, -1); };
          FnSink<decltype(g)> fs{g};
          match_scan<BLOCK, FUZZY, QC>(s, c, fs);
        }
      };
      if (a.pool_mode == CSD_POOL_TREE && M <= kWave) {
        int32_t* windows = reinterpret_cast<int32_t*>(s.table);
        fetch_windows<BLOCK>(s, c, M, L, windows);
        if (c.tid < kWave)
          walk_matches<true>(s, c, M, L, WinInfo{0, M}, windows, a.alpha_q, a.score_mode, o);
      } else if (a.pool_mode == CSD_POOL_TREE) {
        walk_tree<BLOCK>(s, c, WinInfo{M, 0}, M, L, a.alpha_q, ix.status, o, each);
      } else {
        walk_list<BLOCK>(s, c, WinInfo{M, 0}, L, a.alpha_q, o, each);
      }
    } else if (M > 0) {
      // up to a wave's worth of matches: a lane per match; up to a workgroup's worth: a thread
      // per match; else streaming
      bool done = false;
      if (M <= kWave) {
        // one lane of wave 0 per match, no tables: all threads fetch the continuations into
        // windows (laid over the unused table), one (match, layer) instance each.  (More matches
        // per lane do not pay here: with one-edit matching most continuations differ, and a
        // layer then costs one round per match.)
        int32_t* windows = reinterpret_cast<int32_t*>(s.table);
        fetch_windows<BLOCK>(s, c, M, L, windows);
        if (c.tid < kWave) walk_matches(s, c, M, L, WinInfo{0, M}, windows, a.alpha_q, a.score_mode, o);
        done = true;
      } else if (M <= BLOCK) {
        // one thread per match: node weights tabulated first, or layer by layer
        // (the second where the first does not apply or finds too many distinct continuations)
        if (!walk_tab_fits<BLOCK>(M, L, ix.vocab, a.score_mode) ||
            !walk_tab<BLOCK>(s, c, M, L, a.alpha_q, o, sl.n > 1))
          walk_wide<BLOCK>(s, c, M, L, a.alpha_q, a.score_mode, o);
        done = true;
      }
      if (!done)
        walk_streaming<BLOCK>(s, c, WinInfo{M, 0}, M, L, a.alpha_q, a.score_mode, ix.status, o, [&](auto f) {
          if (M <= LdsScan::kMatch) {
            for (int32_t m = c.tid; m < M; m += BLOCK) f(s.match[m], m);
          } else {
            auto g = [&](Match found) { f(found, -1); };
            FnSink<decltype(g)> fs{g};
            match_scan<BLOCK, FUZZY, QC>(s, c, fs);
          }
        });
    }
  }
  CSD_STAMP(unit, 5, CSD_CLOCK());
  write_outputs<BLOCK>(a, row, o, c.tid);
  if (a.targets && c.tid < kWave) {
    int32_t target = c.tid < L ? a.targets[(int64_t)row * L + c.tid] : 0;
    write_accept(a, row, o, target, c.tid);
  }
  CSD_STAMP(unit, 6, CSD_CLOCK());
}

// Index mode.  Per (problem, path) one wave64 runs the front end (matches with
// their continuations in LDS), the DAG and its walk in one of three forms
// (lanes = instances, lanes = matches, LDS tables), outputs and accept; the
// append and the split-phase index insert are done by the same wave (one-edit
// matching) or by a second one (exact matching, see below).
// FUZZY: the index files every position under its gram's variants and matching tolerates
// one edit (Eq. 4).
// QC: compile-time bound (4 or 8) of the index's gram length.
// Two waves per row (on two SIMDs of the CU): the second does the row's append and index
// insert, which the draft does not depend on, so that they leave the critical path of the
// first.  The two never meet at a barrier.
constexpr int step_wave_threads(bool) { return 2 * kWave; }

// The accept-driven loop's stand-in model as the tail of a step (see advance_kernel): the row
// that has just drafted and counted its accepted tokens works out what it appends at the NEXT
// step — those tokens plus the one the model emits itself, from the path's own future — and
// the targets of the next draft, into buffers that the next launch reads (not the ones this
// launch reads: the caller alternates between two sets).
struct NoTail {};
struct LoopTail {
  const int32_t* future_tok;    // [rows][max_len]
  const float* future_prob;     // [rows][max_len] or null
  int32_t* next_tok;            // [rows][n]
  float* next_prob;             // [rows][n] or null
  int32_t* next_cnt;            // [rows]
  int32_t* next_targets;        // [rows][L]
  int32_t* path_len;            // [rows] output: lengths after this step's append
  int32_t n, max_len;
};

// One decode step of one row by one wave: front end, DAG, walk, outputs, accept, tail.
// APPENDS: the wave also appends the row's tokens and files them in the index (false: another
// wave of the workgroup does, see wave_append).  s: the row's on-chip state.
template <int LCAP, bool POOLS, class LDS, bool FUZZY, int QC, bool APPENDS, class TAIL>
__device__ __forceinline__ void row_step(LDS& s, const IndexView& ix, const StepIn& in,
                                         const DraftArgs& a, const TAIL& tail, int32_t row, int lane) {
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);
  c.tid = lane;
#ifdef CSD_STAMPS
  c.unit = row;
  if (lane == 0 && row < (1 << 14)) {
    g_stamps[row * kStampSlots + 0] = CSD_CLOCK();
    g_stamps[row * kStampSlots + 6] = 0ull;
  }
#endif
  const int32_t L = a.L;
  int32_t target = (a.targets && c.tid < L) ? a.targets[(int64_t)row * L + c.tid] : 0;
  WinInfo wi;
  InsertTicket ticket;
  VariantTicket tickets;
  bool ticket_used;
  int32_t M = FUZZY ? wave_front_end_fuzzy<LCAP, QC, APPENDS>(s, c, ix, p, a.k, L, wi, tickets, ticket_used)
                    : wave_front_end<LCAP, QC, APPENDS, POOLS>(s, c, ix, p, a.k, L, wi, ticket, ticket_used);
  block_sync<kWave>();
#ifdef CSD_STAMPS
  if (lane == 0 && row < (1 << 14)) {
    g_stamps[row * kStampSlots + 1] = CSD_CLOCK();
    g_stamps[row * kStampSlots + 9] = (unsigned long long)M;
  }
#endif
  if (APPENDS && POOLS && !FUZZY && in.n > 1) {
    // a step of several tokens appended by the drafting wave itself (nothing this step's
    // drafts read is written here)
    const int32_t old_i = c.y.old_len(c.i);
    append_row<kWave, true>(ix, c.y, p, c.i, old_i, c.y.new_len(c.i, old_i), lane);
  }
  // the loop's tail needs the path's future from its new end on (lane x: x tokens further):
  // requested here, so that the load travels during the walk
  int32_t future_a = 0, future_b = 0;
  float future_p = 0.0f;
  if constexpr (std::is_same<TAIL, LoopTail>::value) {
    const int64_t base = (int64_t)row * tail.max_len;
    const int32_t xa = c.len_i + c.tid, xb = xa + kWave;
    future_a = tail.future_tok[base + (xa < tail.max_len ? xa : 0)];
    future_b = tail.future_tok[base + (xb < tail.max_len ? xb : 0)];
    if (tail.future_prob) future_p = tail.future_prob[base + (xa < tail.max_len ? xa : 0)];
  }
  if (POOLS && (ix.options & 2)) {
    // query back-off: no match, so the query loses its oldest token and the histories are
    // searched again (position by position: the index holds grams of max_query_len tokens only)
    while (M == 0 && c.q > 1) {
      --c.q;
      WaveListSink<LDS> sink{&s, &M, c.tid};
      match_plain<FUZZY>(s, c, sink);
      wi = WinInfo{M, 0};
      if (c.tid == 0) s.n_match = M;
      block_sync<kWave>();
    }
  }

  DraftOut o;
  if (POOLS && M > 0 && a.pool_mode != CSD_POOL_DAG) {
    auto each = [&](auto f) {
      if (M <= LDS::kMatch) {
        for (int32_t m = c.tid; m < M; m += kWave) f(s.match[m], m);
      } else {
        auto g = [&](Match found) { f(found, -1); };
        FnSink<decltype(g)> fs{g};
        match_plain<FUZZY>(s, c, fs);
      }
    };
    if (a.pool_mode == CSD_POOL_TREE && M <= kWave && M <= LDS::kWin / (2 * L))
      walk_matches<true>(s, c, M, L, wi, s.win, a.alpha_q, a.score_mode, o);   // one lane per match
    else if (a.pool_mode == CSD_POOL_TREE)
      walk_tree<kWave>(s, c, wi, M, L, a.alpha_q, ix.status, o, each);
    else
      walk_list<kWave>(s, c, wi, L, a.alpha_q, o, each);
  } else if (M > 0 && M <= 8 && (L << lanes_log2(M)) <= kWave) {                   // few matches: no tables
    switch (lanes_log2(M)) {
      case 0: walk_instances<1>(s, c, M, L, wi, a.alpha_q, a.score_mode, o); break;
      case 1: walk_instances<2>(s, c, M, L, wi, a.alpha_q, a.score_mode, o); break;
      case 2: walk_instances<4>(s, c, M, L, wi, a.alpha_q, a.score_mode, o); break;
      default: walk_instances<8>(s, c, M, L, wi, a.alpha_q, a.score_mode, o); break;
    }
  } else if (M > 0 && M <= kWave &&
             (M - LDS::kWin / (2 * L)) * 2 * L * (int32_t)sizeof(int32_t) <= (int32_t)sizeof(s.table)) {
    // one lane per match; with more matches than the layout has windows, the others' windows
    // are laid over the table, which this walk does not use
    walk_matches(s, c, M, L, wi, s.win, a.alpha_q, a.score_mode, o, reinterpret_cast<int32_t*>(s.table),
                 LDS::kWin / (2 * L));
  } else if (M > 0 && M <= 2 * kWave && M <= LDS::kWin / (2 * L)) {
    walk_matches<false, 2>(s, c, M, L, wi, s.win, a.alpha_q, a.score_mode, o);   // two matches per lane
  } else if (M > 0 && walk_tab_wave_fits<LDS>(M, ix.vocab, a.score_mode) &&
             walk_tab_wave(s, c, wi, M, L, a.alpha_q, o)) {
    // node weights of all layers tabulated first, then the walk
  } else if (M > 0) {
    bool streaming = M > LDS::kMatch;
    if (!streaming) {
      Tier1 t1 = build_dag<kWave>(s, c, M, L, wi, a.alpha_q);
      streaming = s.overflow != 0;
      if (!streaming) walk_dag<kWave, LCAP>(s, c, t1, L, a.alpha_q, a.score_mode, o);
    }
    if (streaming)
      walk_streaming<kWave>(s, c, wi, M, L, a.alpha_q, a.score_mode, ix.status, o, [&](auto f) {
        if (M <= LDS::kMatch) {
          for (int32_t m = c.tid; m < M; m += kWave) f(s.match[m], m);
        } else {
          auto g = [&](Match found) { f(found, -1); };
          FnSink<decltype(g)> fs{g};
          match_plain<FUZZY>(s, c, fs);
        }
      });
  }
#ifdef CSD_STAMPS
  if (lane == 0 && row < (1 << 14)) g_stamps[row * kStampSlots + 5] = CSD_CLOCK();
#endif
  // the posting stores wait on atomics issued long ago: do them before the output stores
  if (ticket_used && FUZZY)
    variants_finish(tickets, const_cast<int32_t*>(c.gram), c.bucket_mask, c.y.pos(c.i, c.len_i - 1),
                    c.tid);
  else if (ticket_used)
    insert_finish(ticket, const_cast<int32_t*>(c.gram), c.bucket_mask,
                  c.y.pos(c.i, c.len_i - 1), c.tid);
  write_outputs<kWave>(a, row, o, c.tid);
  int32_t accepted = 0;
  if (a.targets) accepted = write_accept(a, row, o, target, c.tid);
#ifdef CSD_STAMPS
  if (lane == 0 && row < (1 << 14)) g_stamps[row * kStampSlots + 6] = CSD_CLOCK();
#endif
  if constexpr (std::is_same<TAIL, LoopTail>::value) {
    const int32_t len = c.len_i;                        // after this step's append
    int32_t grow = accepted + 1;
    grow = grow > tail.n ? tail.n : grow;
    const int32_t room = tail.max_len - len;
    grow = grow < room ? grow : room;
    const int64_t r = row;
    static_assert(CSD_MAX_DRAFT_LEN + 1 <= kWave && 2 * CSD_MAX_DRAFT_LEN < 2 * kWave,
                  "a lane per step token; the targets lie within two waves' worth of the future");
    if (c.tid == 0) {
      tail.next_cnt[r] = grow;
      tail.path_len[r] = len;
    }
    if (c.tid < tail.n) {
      const bool in_path = len + c.tid < tail.max_len;
      tail.next_tok[r * tail.n + c.tid] = in_path ? future_a : 0;
      if (tail.next_prob) tail.next_prob[r * tail.n + c.tid] = in_path ? future_p : 0.0f;
    }
    // target d of the next draft is the future token grow + d places beyond the new end
    const int32_t x = grow + c.tid;
    const int32_t from_a = __shfl(future_a, x & (kWave - 1));
    const int32_t from_b = __shfl(future_b, x & (kWave - 1));
    if (c.tid < L)
      tail.next_targets[r * L + c.tid] = len + x < tail.max_len ? (x < kWave ? from_a : from_b) : -1;
  }
}

// The row of this workgroup: its first wave drafts, a second wave appends.
template <int LCAP, bool POOLS, class LDS, bool FUZZY, int QC, class TAIL>
__device__ __forceinline__ void step_wave_body(const IndexView& ix, const StepIn& in,
                                               const DraftArgs& a, const TAIL& tail) {
  constexpr bool SPLIT = step_wave_threads(FUZZY) > kWave;
  __shared__ LDS s;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  const int lane = (int)(threadIdx.x & (kWave - 1));
  if (SPLIT && __builtin_amdgcn_readfirstlane((int)threadIdx.x) >= kWave) {
    int32_t p;
    Ctx c = make_ctx(ix, in, row, p);
    c.tid = lane;
    if (FUZZY) wave_append_fuzzy(c, ix, p);
    else wave_append<QC, POOLS, std::is_same<LDS, LdsWaveSmall>::value ? 1 : kInsertLanes>(c, ix, p);
    return;
  }
  row_step<LCAP, POOLS, LDS, FUZZY, QC, !SPLIT>(s, ix, in, a, tail, row, lane);
}

template <int LCAP, bool POOLS, class LDS, bool FUZZY, int QC>
__global__ __launch_bounds__(step_wave_threads(FUZZY)) void step_wave_kernel(IndexView ix, StepIn in,
                                                                             DraftArgs a) {
  fetch_kernel_arguments<sizeof(IndexView) + sizeof(StepIn) + sizeof(DraftArgs)>();
  step_wave_body<LCAP, POOLS, LDS, FUZZY, QC>(ix, in, a, NoTail{});
}

// The same for launches of thousands of rows (exact matching, drafts of up to 8 tokens), where
// the number of rows resident on a CU bounds the throughput: compiled for eight waves per SIMD
// (at most 64 registers per lane), with the small on-chip layout: sixteen rows per CU.
template <int QC>
__global__ __launch_bounds__(step_wave_threads(false)) __attribute__((amdgpu_waves_per_eu(8, 8)))
void step_wave_many_kernel(IndexView ix, StepIn in, DraftArgs a) {
  fetch_kernel_arguments<sizeof(IndexView) + sizeof(StepIn) + sizeof(DraftArgs)>();
  step_wave_body<8, false, LdsWaveSmall, false, QC>(ix, in, a, NoTail{});
}

// One step of the accept-driven loop in one launch: a step of up to L + 1 tokens per path
// (general instantiation, exact matching), then the tail that prepares the next step.
template <int LCAP, int QC>
__global__ __launch_bounds__(step_wave_threads(false)) void step_loop_kernel(IndexView ix, StepIn in,
                                                                             DraftArgs a,
                                                                             LoopTail tail) {
  fetch_kernel_arguments<sizeof(IndexView) + sizeof(StepIn) + sizeof(DraftArgs) + sizeof(LoopTail)>();
  step_wave_body<LCAP, true, LdsWave, false, QC>(ix, in, a, tail);
}

// Many steps per launch (the device-side form of the host loops csd_replay and
// csd_accept_loop, where nothing happens on the host between two steps): one workgroup per
// problem, one wave per path (at most 16), exact matching through the index.  A step's rows
// only read what earlier steps wrote, so one workgroup barrier between steps orders
// everything; no launch, no cold cache and no argument fetch per step.
struct MultiArgs {
  int32_t n_steps, cur;         // cur: which meta buffer holds the paths' ends on entry
  int32_t* meta[2];
  // replay: step t appends tokens[t] (one token per path) and drafts into slice t
  const int32_t* tokens;        // [n_steps][P][N], or null (the accept-driven loop)
  const float* probs;           // [n_steps][P][N] or null
  const int32_t* targets;       // [n_steps][P][N][L] or null
  float* token_scores;          // [n_steps][P][N][L] or null
  float* path_scores;           // [n_steps][P][N] or null
  // accept-driven loop: the two sets of step buffers (see LoopTail); step t reads set t & 1
  int32_t* step_tok[2];
  float* step_prob[2];
  int32_t* step_cnt[2];
  int32_t* step_targets[2];
  const int32_t* future_tok;
  const float* future_prob;
  int32_t* path_len;            // [n_steps][P][N]
  int32_t n;                    // tokens per path and step the loop offers (L + 1)
  // both
  DraftArgs a;                  // outputs of step 0; step t writes slice t
};

template <int LCAP, bool POOLS, int QC, bool LOOP>
__global__ __launch_bounds__(16 * kWave) void step_multi_kernel(IndexView ix, MultiArgs m) {
  __shared__ LdsMulti rows_lds[16];
  const int wave = (int)(threadIdx.x >> 6), lane = (int)(threadIdx.x & (kWave - 1));
  const int32_t row = (int32_t)blockIdx.x * ix.N + wave;    // the block has N waves
  const int64_t rows = (int64_t)ix.P * ix.N;
  const int64_t L = m.a.L;
  for (int32_t t = 0; t < m.n_steps; ++t) {
    IndexView v = ix;
    v.meta_old = m.meta[(m.cur + t) & 1];
    v.meta_new = m.meta[(m.cur + t + 1) & 1];
    DraftArgs a = m.a;
    a.draft_tokens += t * rows * L;
    a.draft_len += t * rows;
    if (a.accept_len) a.accept_len += t * rows;
    if constexpr (LOOP) {
      const int x = t & 1;
      const StepIn in{m.step_tok[x], m.step_prob[x], m.step_cnt[x], m.n};
      a.targets = m.step_targets[x];
      const LoopTail tail{m.future_tok, m.future_prob, m.step_tok[x ^ 1], m.step_prob[x ^ 1],
                          m.step_cnt[x ^ 1], m.step_targets[x ^ 1], m.path_len + t * rows, m.n, ix.max_len};
      row_step<LCAP, true, LdsMulti, false, QC, true>(rows_lds[wave], v, in, a, tail, row, lane);
    } else {
      const StepIn in{m.tokens + t * rows, m.probs ? m.probs + t * rows : nullptr, nullptr, 1};
      if (a.targets) a.targets += t * rows * L;
      if (a.token_scores) a.token_scores += t * rows * L;
      if (a.path_scores) a.path_scores += t * rows;
      row_step<LCAP, POOLS, LdsMulti, false, QC, true>(rows_lds[wave], v, in, a, NoTail{}, row, lane);
    }
    // what this step wrote (histories, path ends, index, the loop's next input) before what
    // the next step reads: the waves of a workgroup share their CU's vector cache, which is
    // dropped here all the same (index buckets are also written by atomics, which work in
    // the L2)
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
}

__global__ __launch_bounds__(256) void accept_kernel(int64_t rows, int32_t L,
                                                     const int32_t* draft_tokens,
                                                     const int32_t* draft_len,
                                                     const int32_t* targets, int32_t* accept_len) {
  int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (r >= rows) return;
  int32_t n = draft_len[r];
  n = n < 0 ? 0 : (n > L ? L : n);
  int32_t a = 0;
  while (a < n && draft_tokens[r * L + a] == targets[r * L + a]) ++a;
  accept_len[r] = a;
}

// The stand-in model of the accept-driven loop: what the model samples for a
// path is the path's own future.  Per row: the step's input — the tokens the
// previous step settled (its accepted draft tokens plus the one token the model
// emits itself), i.e. the next n of the path's future with a count, clipped at
// max_len — and the targets the coming draft will be checked against, the L
// future tokens behind them (-1 beyond the end).
__global__ __launch_bounds__(256) void advance_kernel(int64_t rows, int32_t max_len, int32_t n,
                                                      int32_t L, const int32_t* meta,
                                                      int32_t meta_stride, const int32_t* settled,
                                                      const int32_t* future_tok,
                                                      const float* future_prob, int32_t* step_tok,
                                                      float* step_prob, int32_t* step_cnt,
                                                      int32_t* targets, int32_t* path_len) {
  int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (r >= rows) return;
  int32_t len = meta[r * meta_stride];
  int32_t grow = (settled ? settled[r] : 0) + 1;
  grow = grow < 1 ? 1 : (grow > n ? n : grow);
  int32_t room = max_len - len;
  grow = grow < room ? grow : room;
  step_cnt[r] = grow;
  path_len[r] = len + grow;
  const int32_t* ft = future_tok + r * max_len;
  for (int32_t t = 0; t < n; ++t) {
    bool in = len + t < max_len;
    step_tok[r * n + t] = in ? ft[len + t] : 0;
    if (step_prob) step_prob[r * n + t] = in ? future_prob[r * max_len + len + t] : 0.0f;
  }
  for (int32_t d = 0; d < L; ++d) {
    int32_t t = len + grow + d;
    targets[r * L + d] = t < max_len ? ft[t] : -1;
  }
}

// advance_kernel and append_kernel in one launch (index mode): one workgroup per row works out
// the row's step input, writes it where the draft launch behind it finds the targets, and
// appends it.  The meta row is read before, and updated after, the workgroup's barrier.
__global__ __launch_bounds__(256) void advance_append_kernel(
    IndexView ix, int32_t n, int32_t L, const int32_t* settled, const int32_t* future_tok,
    const float* future_prob, int32_t* step_tok, float* step_prob, int32_t* step_cnt,
    int32_t* targets, int32_t* path_len) {
  fetch_kernel_arguments<sizeof(IndexView) + 2 * sizeof(int32_t) + 9 * sizeof(void*)>();
  const int64_t r = blockIdx.x;
  const int tid = threadIdx.x;
  const int32_t max_len = ix.max_len;
  const int32_t len = ix.meta_old[r * ix.meta_stride];
  int32_t grow = (settled ? settled[r] : 0) + 1;
  grow = grow < 1 ? 1 : (grow > n ? n : grow);
  const int32_t room = max_len - len;
  grow = grow < room ? grow : room;
  if (tid == 0) {
    step_cnt[r] = grow;
    path_len[r] = len + grow;
  }
  const int32_t* ft = future_tok + r * max_len;
  for (int32_t t = tid; t < n; t += 256) {
    bool in = len + t < max_len;
    step_tok[r * n + t] = in ? ft[len + t] : 0;
    if (step_prob) step_prob[r * n + t] = in ? future_prob[r * max_len + len + t] : 0.0f;
  }
  for (int32_t d = tid; d < L; d += 256) {
    int32_t t = len + grow + d;
    targets[r * L + d] = t < max_len ? ft[t] : -1;
  }
  __syncthreads();                      // the step input is read back by this workgroup below
  int32_t p;
  Ctx c = make_ctx(ix, StepIn{step_tok, step_prob, step_cnt, n}, (int32_t)r, p);
  int32_t old_i = c.y.old_len(c.i);
  int32_t new_i = c.y.new_len(c.i, old_i);
  append_row<256, true>(ix, c.y, p, c.i, old_i, new_i, c.tid);
}

// Plain copy of n 16-byte words: the known-size kernel that hardware traffic
// counters are calibrated against.
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src,
                                                   uint4* __restrict__ dst, int64_t n) {
  int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x; x < n; x += stride) dst[x] = src[x];
}

// ---- debug dumps ------------------------------------------------------------

// Scan mode: marks every match of every row in a bitmap [rows][words].
__global__ __launch_bounds__(kScanBlock) void dump_match_bits_scan_kernel(IndexView ix, StepIn in,
                                                                          int32_t k, uint32_t* bits,
                                                                          int32_t words) {
  __shared__ LdsScan s;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);   // in.n == 0: nothing is being appended
  int32_t old_i = c.y.old_len(c.i);
  c.len_i = old_i;
  load_query(c, k, old_i);
  cache_lens<kScanBlock>(s, c.y, c.tid);
  block_sync<kScanBlock>();
  if (c.q <= 0) return;
  BitmapSink sink{bits + (int64_t)row * words};
  match_scan_any<kScanBlock>(s, c, sink);
}

// Index mode: the matches as the step kernel's own front end finds them.
template <bool FUZZY>
__global__ __launch_bounds__(kWave) void dump_match_bits_wave_kernel(IndexView ix, StepIn in,
                                                                     int32_t k, uint32_t* bits,
                                                                     int32_t words) {
  __shared__ LdsWave s;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);   // in.n == 0: nothing is being appended
  WinInfo wi;
  InsertTicket ticket;
  VariantTicket tickets;
  bool ticket_used;
  int32_t M = FUZZY ? wave_front_end_fuzzy<8>(s, c, ix, p, k, 1, wi, tickets, ticket_used)
                    : wave_front_end<8, CSD_MAX_QUERY_LEN, true, true>(s, c, ix, p, k, 1, wi, ticket, ticket_used);
  block_sync<kWave>();
  BitmapSink sink{bits + (int64_t)row * words};
  if (M <= LdsWave::kMatch) {
    for (int32_t m = c.tid; m < M; m += kWave) sink.push(c.y, true, s.match[m]);
  } else if (c.q > 0) {
    match_plain<FUZZY>(s, c, sink);
  }
}

// counts[row] = number of set bits of the row (one workgroup per row)
__global__ __launch_bounds__(256) void count_bits_kernel(const uint32_t* bits, int32_t words,
                                                         int32_t* counts) {
  __shared__ int total;
  if (threadIdx.x == 0) total = 0;
  __syncthreads();
  const uint32_t* b = bits + (int64_t)blockIdx.x * words;
  int n = 0;
  for (int32_t w = threadIdx.x; w < words; w += 256) n += __popc(b[w]);
  atomicAdd(&total, n);
  __syncthreads();
  if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

// off[0] = 0, off[r+1] = off[r] + max(counts[r], 0); *bad = 1 if any count < 0
__global__ void offsets_kernel(const int32_t* counts, int32_t rows, int32_t* off, int32_t* bad) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  int32_t acc = 0, any_bad = 0;
  off[0] = 0;
  for (int32_t r = 0; r < rows; ++r) {
    int32_t n = counts[r];
    if (n < 0) { any_bad = 1; n = 0; }
    acc += n;
    off[r + 1] = acc;
  }
  *bad = any_bad;
}

// Expands each row's bitmap into ascending (j, e) pairs (one wave per row).
__global__ __launch_bounds__(64) void expand_bits_kernel(const uint32_t* bits, int32_t words,
                                                         int32_t max_len, const int32_t* off,
                                                         int32_t* out_je, int64_t cap) {
  const uint32_t* b = bits + (int64_t)blockIdx.x * words;
  int64_t base = off[blockIdx.x];
  int lane = threadIdx.x;
  for (int32_t w0 = 0; w0 < words; w0 += 64) {
    int32_t w = w0 + lane;
    uint32_t x = w < words ? b[w] : 0u;
    int n = __popc(x);
    int incl = n;                                     // inclusive prefix sum over lanes
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      int y = __shfl_up(incl, o);
      if (lane >= o) incl += y;
    }
    int64_t at = base + incl - n;
    while (x) {
      int bit = __ffs(x) - 1;
      x &= x - 1;
      int32_t pos = w * 32 + bit;
      if (at < cap) {
        out_je[2 * at] = pos / max_len;
        out_je[2 * at + 1] = pos % max_len;
      }
      ++at;
    }
    base += __shfl(incl, 63);
  }
}

// Scan mode: builds the tier-1 DAG tables of a row exactly as step_scan_kernel
// does and writes the edge entries, sorted by key, to tmp rows of kDumpStride
// entries.  counts[row] = number of edges, or -1 if the row's DAG does not fit
// the table as a whole.
__global__ __launch_bounds__(kScanBlock) void dump_edge_rows_scan_kernel(
    IndexView ix, StepIn in, int32_t k, int32_t L, u64* tmp_keys, u64* tmp_vals, int32_t* counts) {
  constexpr int BLOCK = kScanBlock;
  __shared__ LdsScan s;
  __shared__ int n_edges;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);   // in.n == 0: nothing is being appended
  int32_t old_i = c.y.old_len(c.i);
  c.len_i = old_i;
  load_query(c, k, old_i);
  cache_lens<BLOCK>(s, c.y, c.tid);
  if (c.tid == 0) { s.n_match = 0; n_edges = 0; }
  block_sync<BLOCK>();
  if (c.q <= 0) { if (c.tid == 0) counts[row] = 0; return; }
  ListSink<LdsScan> sink{&s};
  match_scan_any<BLOCK>(s, c, sink);
  block_sync<BLOCK>();
  int32_t M = s.n_match;
  if (M == 0) { if (c.tid == 0) counts[row] = 0; return; }
  if (M > LdsScan::kMatch) { if (c.tid == 0) counts[row] = -1; return; }
  Tier1 t1 = build_dag<BLOCK>(s, c, M, L, WinInfo{M, 0}, 0u);
  if (s.overflow) { if (c.tid == 0) counts[row] = -1; return; }
  emit_sorted_edges<BLOCK>(s, t1.region * (uint32_t)L, c.tid, &n_edges,
                           tmp_keys + (int64_t)row * kDumpStride, tmp_vals + (int64_t)row * kDumpStride);
  block_sync<BLOCK>();
  if (c.tid == 0) counts[row] = n_edges;
}

// Index mode: front end and DAG build of the step kernel itself.
template <int LCAP, bool FUZZY>
__global__ __launch_bounds__(kWave) void dump_edge_rows_wave_kernel(IndexView ix, StepIn in,
                                                                    int32_t k, int32_t L,
                                                                    u64* tmp_keys, u64* tmp_vals,
                                                                    int32_t* counts) {
  __shared__ LdsWave s;
  __shared__ int n_edges;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);   // in.n == 0: nothing is being appended
  if (c.tid == 0) n_edges = 0;
  WinInfo wi;
  InsertTicket ticket;
  VariantTicket tickets;
  bool ticket_used;
  int32_t M = FUZZY ? wave_front_end_fuzzy<LCAP>(s, c, ix, p, k, L, wi, tickets, ticket_used)
                    : wave_front_end<LCAP, CSD_MAX_QUERY_LEN, true, true>(s, c, ix, p, k, L, wi, ticket, ticket_used);
  block_sync<kWave>();
  if (M == 0) { if (c.tid == 0) counts[row] = 0; return; }
  if (M > LdsWave::kMatch) { if (c.tid == 0) counts[row] = -1; return; }
  Tier1 t1 = build_dag<kWave>(s, c, M, L, wi, 0u);
  if (s.overflow) { if (c.tid == 0) counts[row] = -1; return; }
  emit_sorted_edges<kWave>(s, t1.region * (uint32_t)L, c.tid, &n_edges,
                           tmp_keys + (int64_t)row * kDumpStride, tmp_vals + (int64_t)row * kDumpStride);
  block_sync<kWave>();
  if (c.tid == 0) counts[row] = n_edges;
}

__global__ __launch_bounds__(256) void scatter_edges_kernel(const u64* tmp_keys,
                                                            const u64* tmp_vals,
                                                            const int32_t* off, int32_t* out_duv,
                                                            uint64_t* out_cs, int64_t cap) {
  int32_t row = blockIdx.x;
  int64_t base = off[row];
  int32_t n = off[row + 1] - off[row];
  for (int32_t x = threadIdx.x; x < n; x += 256) {
    int64_t at = base + x;
    if (at >= cap) break;
    u64 key = tmp_keys[(int64_t)row * kDumpStride + x];
    u64 val = tmp_vals[(int64_t)row * kDumpStride + x];
    out_duv[3 * at] = (int32_t)(key >> 58);
    out_duv[3 * at + 1] = (int32_t)key_u(key);
    out_duv[3 * at + 2] = (int32_t)key_v(key);
    out_cs[2 * at] = cs_count(val);
    out_cs[2 * at + 1] = cs_sum(val);
  }
}

}  // namespace csd
