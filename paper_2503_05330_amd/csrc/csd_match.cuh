// csd — cross-path suffix matching (Eq. 3): by exhaustive scan, through the
// n-gram index (general form), and the one-wave front end of the decode step
// that needs only three dependent memory round trips.
#pragma once

#include "csd_common.cuh"
#include "csd_dag.cuh"
#include "csd_index.cuh"

namespace csd {

__device__ __forceinline__ void load_query(Ctx& c, int32_t k, int32_t old_i) {
  c.q = k < c.len_i ? k : c.len_i;
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a)
    c.Q[a] = (a < c.q) ? c.y.token(c.i, c.len_i - 1 - a, old_i) : 0;
}

// t[a] = the a-th token before index e of path j for a < min(want, e), else 0.
// All loads are issued together (one memory round trip).  When the tokens of
// every calling lane are history and exist (the rule, unless a path is very
// short or the launch appends several tokens), they come from one address with
// fixed offsets; otherwise each is located on its own.
template <int NT>
__device__ __forceinline__ void tokens_before(const Ctx& c, int32_t j, int32_t e, int32_t old_j,
                                              int32_t want, int32_t (&t)[NT]) {
  bool deep = e <= old_j && e >= NT;
  if (wave_ballot(!deep) == 0) {
    const int32_t* newest = c.y.tok + c.y.cell(j, e - 1);
#pragma unroll
    for (int a = 0; a < NT; ++a) t[a] = newest[-a];
  } else {
#pragma unroll
    for (int a = 0; a < NT; ++a) {                         // every lane loads; unused ones read cell 0
      bool has = a < want && a < e;
      t[a] = c.y.token(has ? j : 0, has ? e - 1 - a : 0, has ? old_j : 1);
    }
  }
#pragma unroll
  for (int a = 0; a < NT; ++a) t[a] = (a < want && a < e) ? t[a] : 0;
}

// Does the q-gram that ends just before index e >= q of path j equal the query?
// QK: compile-time bound of the query length (the loops are unrolled to it).
template <int QK = CSD_MAX_QUERY_LEN>
__device__ __forceinline__ bool gram_equals_query(const Ctx& c, int32_t j, int32_t e,
                                                  int32_t old_j) {
  int32_t t[QK];
  tokens_before(c, j, e, old_j, c.q, t);
  bool hit = true;
#pragma unroll
  for (int a = 0; a < QK; ++a) hit = hit && (a >= c.q || t[a] == c.Q[a]);
  return hit;
}

// Eq. 4 with tolerance 1: is SOME substring of path j that ends just before
// index e within one edit (substitution, insertion or deletion) of the query?
// With t[a] = a-th token before e (newest first, like Q): the tokens newer than
// the edit agree in place, the older ones agree in place (substitution), one
// step further back (the text has an extra token) or one step closer (the text
// lacks a token).
// t[a] = the a-th token before e for a < min(q + 1, e), else 0.
// K: compile-time bound of the query length (the loops are unrolled to it).
template <int K = CSD_MAX_QUERY_LEN>
__device__ __forceinline__ bool near_query(const Ctx& c, int32_t e, const int32_t (&t)[K + 1]) {
  const int32_t q = c.q;
  // pre[p]: t[a] == Q[a] for all a < p.  same/back/fwd[p]: the agreement of the older part
  // a > p (same, fwd) or a >= p (back) at shift 0 / +1 / -1, scanned from the oldest token.
  int32_t Q[K + 1];                                        // Q[K] only pads the unrolled loops
#pragma unroll
  for (int a = 0; a <= K; ++a) Q[a] = a < K ? c.Q[a < K ? a : 0] : 0;
  bool pre[K + 1], same[K + 1], back[K + 1], fwd[K + 1];
  pre[0] = true;
#pragma unroll
  for (int a = 0; a < K; ++a) pre[a + 1] = pre[a] && (a >= q || t[a] == Q[a]);
  same[K] = back[K] = fwd[K] = true;
#pragma unroll
  for (int a = K - 1; a >= 0; --a) {
    same[a] = same[a + 1] && (a + 1 >= q || t[a + 1] == Q[a + 1]);
    back[a] = back[a + 1] && (a >= q || t[a + 1] == Q[a]);
    fwd[a] = fwd[a + 1] && (a + 1 >= q || t[a] == Q[a + 1]);
  }
  bool hit = false;
#pragma unroll
  for (int p = 0; p <= K; ++p) {
    if (p < q) {
      hit = hit || (e >= q && pre[p] && same[p]);          // Q[p] substituted (or kept)
      hit = hit || (e >= q - 1 && pre[p] && fwd[p]);       // the text lacks Q[p]
    }
    if (p <= q) hit = hit || (e >= q + 1 && pre[p] && back[p]);   // extra text token at p
  }
  return hit;
}

template <int QK = CSD_MAX_QUERY_LEN>
__device__ __forceinline__ bool gram_near_query(const Ctx& c, int32_t j, int32_t e, int32_t old_j) {
  int32_t t[QK + 1];
  tokens_before(c, j, e, old_j, c.q + 1, t);
  return near_query<QK>(c, e, t);
}

// Eq. 4 with any tolerance up to CSD_MAX_EDITS: is SOME substring of path j that ends just
// before index e within eps edits of the query?  With both strings read backwards from e
// (Q[a] = a-th query token from its end, t[b] = b-th token before e) the substrings that end
// at e are the prefixes of t, so one dynamic programme answers for all their lengths at once:
// D[i][b] = Levenshtein distance between the first i tokens of Q and the first b of t; the
// position matches when D[q][b] <= eps for some b <= min(e, q + eps).  Column by column
// over b, the column kept in registers.
// t[b] = the b-th token before e for b < min(q + eps, e), else anything.
template <int K = CSD_MAX_QUERY_LEN>
__device__ __forceinline__ bool within_edits(const Ctx& c, int32_t e,
                                             const int32_t (&t)[K + CSD_MAX_EDITS]) {
  const int32_t q = c.q;
  int32_t D[K + 1];
#pragma unroll
  for (int i = 0; i <= K; ++i) D[i] = i;                 // against the empty substring
  int32_t best = q;
  const int32_t longest = q + c.eps < e ? q + c.eps : e;   // substrings of up to this many tokens
#pragma unroll
  for (int b = 1; b <= K + CSD_MAX_EDITS; ++b) {
    int32_t diag = D[0];
    D[0] = b;
#pragma unroll
    for (int i = 1; i <= K; ++i) {
      const int32_t up = D[i];
      int32_t v = diag + ((i <= q && c.Q[i - 1] == t[b - 1]) ? 0 : 1);   // substitute / keep
      v = v < up + 1 ? v : up + 1;                                       // the text has one token more
      v = v < D[i - 1] + 1 ? v : D[i - 1] + 1;                           // the query has one token more
      D[i] = v;
      diag = up;
    }
    const int32_t here = pick(D, q);
    best = (b <= longest && here < best) ? here : best;
  }
  return best <= c.eps;
}

template <int QK = CSD_MAX_QUERY_LEN>
__device__ __forceinline__ bool gram_within_edits(const Ctx& c, int32_t j, int32_t e, int32_t old_j) {
  int32_t t[QK + CSD_MAX_EDITS];
  tokens_before(c, j, e, old_j, c.q + c.eps, t);
  return within_edits<QK>(c, e, t);
}

template <int QC>
__device__ __forceinline__ GramHash query_hash(const Ctx& c) {
  uint32_t acc = kGramSeed;
#pragma unroll
  for (int a = 0; a < QC; ++a)
    if (a < c.q) acc = gram_hash_add(acc, c.Q[a]);
  return gram_hash_end(acc, c.q);
}

// ---------------------------------------------------------------- match sinks

// Compacts hits into the LDS match list with one LDS atomic per wave.
// push() must be reached by all 64 lanes of a wave together.
template <class LDS>
struct ListSink {
  LDS* s;
  __device__ __forceinline__ void push(const Paths&, bool hit, Match m) {
    u64 mask = wave_ballot(hit);
    if (mask == 0) return;
    int lane = __lane_id();
    int base = 0;
    if (lane == 0) base = atomicAdd(&s->n_match, (int)__popcll(mask));
    base = __builtin_amdgcn_readfirstlane(base);
    int slot = base + (int)__popcll(mask & ((1ull << lane) - 1ull));
    if (hit && slot < LDS::kMatch) s->match[slot] = m;
  }
};

// Marks hits in a bitmap over all positions [N][max_len] of the problem (debug dump).
struct BitmapSink {
  uint32_t* bits;
  __device__ __forceinline__ void push(const Paths& y, bool hit, Match m) {
    if (!hit) return;
    int32_t bit = y.cell(y.pos_path(m.pos), y.pos_index(m.pos));
    atomicOr(&bits[bit >> 5], 1u << (bit & 31));
  }
};

// Hands every hit to a callable (streaming tier).
template <class F>
struct FnSink {
  F f;
  __device__ __forceinline__ void push(const Paths&, bool hit, Match m) {
    if (hit) f(m);
  }
};

// ---------------------------------------------------------------- general matchers

// Lengths of path j: from the LDS cache for the first LDS::kLens paths.
template <class LDS>
__device__ __forceinline__ void lens_of(const LDS& s, const Paths& y, int32_t j, int32_t& old_j,
                                        int32_t& new_j) {
  if (j < LDS::kLens) {
    old_j = s.len_old[j];
    new_j = s.len_new[j];
  } else {
    old_j = y.old_len(j);
    new_j = y.new_len(j, old_j);
  }
}

// The scan's filter: can a position match at all, judged by the three newest
// tokens before it (t[0] newest; all three exist)?
//   Exact: they must equal the query's newest tokens; for q <= 3 that already
//   is the answer.
//   One edit, q >= 3: the edit touches at most one of the three newest query
//   tokens, so two of them survive, in place or one place off.  The cases: no
//   edit among the newest two (t0=Q0, t1=Q1); Q0 or Q1 substituted (t1=Q1,
//   t2=Q2 / t0=Q0, t2=Q2); the text lacks Q0 or Q1 (t0=Q1, t1=Q2 / t0=Q0,
//   t1=Q2); the text has an extra token before Q0 or between Q0 and Q1
//   (t1=Q0, t2=Q1 / t0=Q0, t2=Q1).  Shorter queries get a weaker test or none.
constexpr int kFilterTokens = 3;
template <bool FUZZY>
__device__ __forceinline__ bool may_match(const Ctx& c, const int32_t (&t)[kFilterTokens]) {
  if (!FUZZY) {
    bool ok = true;
#pragma unroll
    for (int a = 0; a < kFilterTokens; ++a) ok = ok && (a >= c.q || t[a] == c.Q[a]);
    return ok;
  }
  if (c.q < 2 || c.eps > 1) return true;                   // (more than one edit: no filter)
  if (c.q < 3) return t[0] == c.Q[0] || t[0] == c.Q[1] || t[1] == c.Q[0] || t[1] == c.Q[1];
  bool c0 = t[0] == c.Q[0], c1 = t[1] == c.Q[1], c2 = t[2] == c.Q[2];
  bool a01 = t[0] == c.Q[1], a12 = t[1] == c.Q[2], b10 = t[1] == c.Q[0], b21 = t[2] == c.Q[1];
  return (c0 && (c1 || c2 || a12 || b21)) || (c1 && c2) || (a01 && a12) || (b10 && b21);
}

// Eq. 3 (FUZZY = false) or Eq. 4 with one edit (FUZZY = true) by exhaustive
// comparison: every position e of every other path j with q - eps <= e <=
// len_j - 1 is tested.  s.len_old / s.len_new hold the lengths of the first
// LDS::kLens paths.
//
// A row's positions all pass through one CU, and what bounds the scan there is
// instruction issue, so the common case is kept lean.  The paths are cut into
// spans of 256 positions, dealt round-robin to the workgroup's waves; a lane
// takes four consecutive positions and fetches the six tokens they look at
// (three before the first .. the one before the last) with two 12-byte loads,
// outside any branch; the loads of four spans travel together.  A position
// with three history tokens before it is filtered on those; where the filter
// does not settle the answer, and for the few positions it does not cover (the
// first three of a path, which are only pre-filtered, and those that touch
// tokens this launch appends), the full comparison runs once per round for the
// lanes' next candidate, until no lane of the wave has one left.  Hits are
// pushed in no particular order; every wave runs its own trip counts (push() is
// a wave-level operation).  A row's scan can be shared by n_slices workgroups:
// this one, number `slice`, takes every n_slices-th share of the spans.
// QK: compile-time bound of the query length.
template <int BLOCK, bool FUZZY, int QK = CSD_MAX_QUERY_LEN, class LDS, class Sink>
__device__ __forceinline__ void match_scan(const LDS& s, const Ctx& c, Sink& sink, int32_t slice = 0,
                                           int32_t n_slices = 1) {
  const int32_t n_waves = (BLOCK / kWave) * n_slices;       // waves that share the row
  constexpr int kPerLane = 4;                              // consecutive positions of a lane
  constexpr int kSpan = kWave * kPerLane;                  // positions of a span
  constexpr int kSpans = 4;                                // spans in flight: 16 candidate bits
  // (consecutive spans go to different slices: a row with fewer spans than waves still keeps
  // all its workgroups busy)
  const int lane = c.tid & 63, wave = (c.tid >> 6) * n_slices + slice;
  const int32_t first_e = c.q > c.eps ? c.q - c.eps : 0;          // shortest substring that can match
  const int32_t spans_per_path = (c.y.max_len + kSpan - 1) / kSpan;
  const int32_t spans = c.y.N * spans_per_path;            // < 2^24
  const float inv_spp = 1.0f / (float)spans_per_path;
  const bool filter_decides = !FUZZY && c.q <= kFilterTokens;
  // span number g -> its path and the first position of this lane in it
  auto locate = [&](int32_t g, int32_t& j, int32_t& e0) {
    j = (int32_t)((float)g * inv_spp);                     // g / spans_per_path, fixed up below
    j += (j + 1) * spans_per_path <= g;
    j -= j * spans_per_path > g;
    e0 = (g - j * spans_per_path) * kSpan + lane * kPerLane;
  };
  for (int32_t g0 = wave; g0 < spans; g0 += n_waves * kSpans) {
    int32_t w[kSpans][2 * kFilterTokens];                  // tokens e0 - 3 .. e0 + 2 (first lane: 0 .. 5)
    // bit 4u + r, for position r of span u: is a candidate / was filtered / lies among the
    // first three of its path; bit u of firsts: this lane starts span u's path
    uint32_t todo = 0, filtered = 0, early = 0, firsts = 0;
#pragma unroll
    for (int u = 0; u < kSpans; ++u) {
      int32_t g = g0 + u * n_waves, j, e0, old_j = 0, new_j = 0;
      if (g >= spans) {                                    // uniform over the wave: no such span
#pragma unroll
        for (int x = 0; x < 2 * kFilterTokens; ++x) w[u][x] = 0;
        continue;
      }
      locate(g, j, e0);
      bool on = j != c.skip;                               // uniform over the wave
      if (on) lens_of(s, c.y, j, old_j, new_j);
      // the lane that starts a path has no three tokens before its positions: it reads the
      // path's first six instead, which serve its fourth position and pre-filter the others
      bool first = on && e0 == 0 && old_j >= kFilterTokens;
      bool lane_ok = on && (first || (e0 >= kFilterTokens && e0 < new_j));
      // lanes without filtered positions read the first six cells of path 0 (the token
      // array is padded for that, and for the two cells a span may read past its path)
      const int32_t* at = c.y.tok + (lane_ok ? c.y.cell(j, first ? kFilterTokens : e0) : kFilterTokens);
#pragma unroll
      for (int x = 0; x < 2 * kFilterTokens; ++x) w[u][x] = at[x - kFilterTokens];
      firsts |= first ? (1u << u) : 0u;
#pragma unroll
      for (int r = 0; r < kPerLane; ++r) {
        int32_t e = e0 + r;
        bool live = on && e >= first_e && e < new_j;
        bool lean = live && lane_ok && e >= kFilterTokens && e <= old_j;   // its three tokens are history
        bool head = live && first && r < kFilterTokens;
        filtered |= lean ? (1u << (4 * u + r)) : 0u;
        early |= head ? (1u << (4 * u + r)) : 0u;
        todo |= (live && !lean && !head) ? (1u << (4 * u + r)) : 0u;
      }
    }
#pragma unroll
    for (int u = 0; u < kSpans; ++u) {
      if (g0 + u * n_waves >= spans) continue;             // uniform over the wave
      const bool fs = (firsts >> u & 1u) != 0;
#pragma unroll
      for (int r = 0; r < kPerLane; ++r) {
        const uint32_t bit = 1u << (4 * u + r);
        int32_t t[kFilterTokens] = {w[u][2 + r], w[u][1 + r], w[u][r]};   // newest first
        if (r == kFilterTokens) {                          // position 3 of a first lane: tokens 2, 1, 0
          t[0] = fs ? w[u][2] : t[0];
          t[1] = fs ? w[u][1] : t[1];
          t[2] = fs ? w[u][0] : t[2];
        }
        todo |= ((filtered & bit) && may_match<FUZZY>(c, t)) ? bit : 0u;
        if (r < kFilterTokens) {                           // position r < 3 of a first lane: tokens r-1 .. 0
          int32_t t0 = w[u][r >= 1 ? r - 1 : 0], t1 = w[u][r >= 2 ? r - 2 : 0];
          bool pass = r == 0;
          if (r >= 1) {
            pass = t0 == c.Q[0];
            if (FUZZY) pass = pass || c.q < 2 || c.eps > 1 || t0 == c.Q[1] || (r >= 2 && (t1 == c.Q[0] || t1 == c.Q[1]));
          }
          todo |= ((early & bit) && pass) ? bit : 0u;
        }
      }
    }
    while (wave_ballot(todo != 0) != 0) {                     // uniform over the wave
      bool have = todo != 0;
      int32_t bit = have ? (int32_t)__ffs(todo) - 1 : 0;
      todo &= todo - 1u;                                   // 0 stays 0
      int32_t j, e, old_j = 1, new_j = 1;
      locate(g0 + (bit >> 2) * n_waves, j, e);
      e += bit & 3;
      bool hit = have;
      if (have) lens_of(s, c.y, j, old_j, new_j);
      if (have && !(filter_decides && (filtered >> bit & 1u)))
        hit = !FUZZY ? gram_equals_query<QK>(c, j, e, old_j)
                     : (c.eps > 1 ? gram_within_edits<QK>(c, j, e, old_j)     // uniform over the launch
                                  : gram_near_query<QK>(c, j, e, old_j));
      sink.push(c.y, hit, make_match(c.y, j, e, old_j, new_j));
    }
  }
}

// The scan with the configured tolerance.
template <int BLOCK, class LDS, class Sink>
__device__ __forceinline__ void match_scan_any(const LDS& s, const Ctx& c, Sink& sink,
                                               int32_t slice = 0, int32_t n_slices = 1) {
  if (c.eps == 0) match_scan<BLOCK, false>(s, c, sink, slice, n_slices);
  else match_scan<BLOCK, true>(s, c, sink, slice, n_slices);
}

// Eq. 3 / Eq. 4 by ONE wave, position by position, in as little code as
// possible.  The one-wave kernels use it where they cannot use the index: for
// queries shorter than the indexed grams (a path's first steps) and to re-find
// matches that did not fit the on-chip list.  Both are rare, and the code of a
// kernel that every launch fetches through cold caches is worth keeping small:
// with the tiled scan inlined in these places the common step was 8 % slower.
template <bool FUZZY, class LDS, class Sink>
__device__ __forceinline__ void match_plain(const LDS& s, const Ctx& c, Sink& sink) {
  const int lane = c.tid & 63;
  const int32_t first_e = c.q > c.eps ? c.q - c.eps : 0;          // shortest substring that can match
  for (int32_t j = 0; j < c.y.N; ++j) {
    if (j == c.skip) continue;
    int32_t old_j, new_j;
    lens_of(s, c.y, j, old_j, new_j);
    for (int32_t e0 = first_e; e0 < new_j; e0 += kWave) {  // trip counts are uniform over the wave
      int32_t e = e0 + lane;
      bool hit = false;
      if (e < new_j)
        hit = !FUZZY ? gram_equals_query(c, j, e, old_j)
                     : (c.eps > 1 ? gram_within_edits(c, j, e, old_j) : gram_near_query(c, j, e, old_j));
      sink.push(c.y, hit, make_match(c.y, j, e, old_j, new_j));
    }
  }
}

// ---------------------------------------------------------------- the one-wave front end
//
// In index mode one wave64 drafts for a (problem, path).  The step is a chain of
// dependent memory round trips, and every launch starts with a cold L2, so the
// front end is laid out to need only three of them before the walk:
//   1. the meta rows (length + last tokens) of all paths and the step's input:
//      the query, the index hashes, the own append and the matches among the
//      newest positions all follow from these without touching the histories;
//   2. the index buckets of the query, and the fill counts for the insert;
//   3. for every posting found, its verify tokens together with its whole
//      continuation (tokens and probabilities), kept in LDS for the DAG;
//      the insert's atomic travels with these.
// It is laid out for steps that append at most one token per path (in.n <= 1); the general
// kernels also take longer steps, at the price of one more round trip (the query then comes
// from the step's input, and the appended positions are matched one lane per position).  With
// exact matching the append and the insert are another wave's (wave_append).


struct Head {                   // a path's end before this step
  int32_t old_len, new_len;
  int32_t tail[kTailCap];       // tail[a] = a-th token from the old end (tail_len of them are kept)
};

// QC: compile-time bound of tail_len (the words beyond it are not looked at).
template <int QC = kTailCap>
__device__ __forceinline__ Head load_head(const Paths& y, int32_t tail_len, int32_t j) {
  Head h;
  const int32_t* row = y.meta_old + (int64_t)j * y.meta_stride;
  const int4* m = reinterpret_cast<const int4*>(row);
  // words the row does not have are not read: their loads go to word 0 instead, so that no
  // load sits behind a branch and all of them travel together
  int4 a = m[0];
  int4 b = QC > 3 ? m[tail_len > 3 ? 1 : 0] : int4{0, 0, 0, 0};
  int32_t c8 = QC > 7 ? row[tail_len > 7 ? 8 : 0] : 0;
  int32_t c9 = QC > 8 ? row[tail_len > 8 ? 9 : 0] : 0;
  if (tail_len <= 3) b = int4{0, 0, 0, 0};
  if (tail_len <= 7) c8 = 0;
  if (tail_len <= 8) c9 = 0;
  h.old_len = a.x;
  h.tail[0] = a.y; h.tail[1] = a.z; h.tail[2] = a.w;
  h.tail[3] = b.x; h.tail[4] = b.y; h.tail[5] = b.z; h.tail[6] = b.w;
  h.tail[7] = c8;
  h.tail[8] = c9;
  h.new_len = y.new_len(j, h.old_len);
  return h;
}

// Appends the hits of all 64 lanes to the match list (one wave: the count lives
// in a register).  Returns each hit's slot, -1 for lanes without one.
template <class LDS>
__device__ __forceinline__ int32_t wave_push(LDS& s, int32_t& n_match, bool hit, Match m, int lane) {
  u64 mask = wave_ballot(hit);
  int32_t slot = n_match + (int32_t)__popcll(mask & ((1ull << lane) - 1ull));
  n_match += (int32_t)__popcll(mask);
  if (!hit) return -1;
  if (slot < LDS::kMatch) s.match[slot] = m;
  return slot;
}

template <class LDS>
struct WaveListSink {           // match list of a one-wave row; push() by all 64 lanes together
  LDS* s;
  int32_t* n_match;
  int lane;
  __device__ __forceinline__ void push(const Paths&, bool hit, Match m) {
    wave_push(*s, *n_match, hit, m, lane);
  }
};

// The own row's append when the step carries one token per path, from values
// already in registers (no further loads).
template <int QC = kTailCap>
__device__ __forceinline__ void append_own_single(const IndexView& ix, const Paths& y, int64_t row,
                                                  int32_t i, const Head& me, int32_t st_i,
                                                  float sp_i, int lane) {
  int32_t cnt = me.new_len - me.old_len;                 // 0 or 1
  if (lane <= ix.tail_len) {
    int32_t a = lane - 1;
    int32_t v = 0;
    if (lane == 0) v = me.new_len;
    else if (a < cnt) v = st_i;
    else if (a < me.new_len) v = pick_n<QC>(me.tail, a - cnt);
    ix.meta_new[row * ix.meta_stride + lane] = v;
  }
  if (lane == 0) {
    uint32_t flags = 0;
    if (cnt == 1) {
      ix.tok[row * ix.max_len + me.old_len] = st_i;
      ix.pq[row * ix.max_len + me.old_len] = y.sp ? quantize_prob(sp_i) : 65536u;
      if (st_i < 0 || st_i >= ix.vocab) flags |= CSD_STATUS_TOKEN_RANGE;
    } else if (!y.sc || y.sc[i] >= 1) {
      flags |= CSD_STATUS_CAPACITY;                      // a token was offered but the path is full
    }
    if (flags) atomicOr(ix.status, flags);
  }
}

// Eq. 3 through the hash index with the continuations fetched in the same
// round trip as the verification.  `word` is the lane's word of the first batch
// of 4 buckets, already requested.  Adds its hits behind the matches already
// listed; match number x of the list gets window x (if x < win_cap).
// GENERAL: also compiled for the options (own history searched): kept out of the usual kernels.
// FIRST: buckets of the first batch (4, or 1 where fetched lines count for more than a row's
// latency: `word` is then requested by the first 16 lanes only); later batches have 4.
template <int LCAP, int QC, bool GENERAL = false, int FIRST = 4, class LDS>
__device__ __forceinline__ void lookup_with_windows(LDS& s, const Ctx& c, int32_t L,
                                                    int32_t win_cap, int32_t& n_match,
                                                    GramHash gh, int32_t word) {
  const int lane = c.tid;
  const Paths& y = c.y;
  int32_t* tbl = const_cast<int32_t*>(c.gram);
  const int sub = lane & 15;          // word of the bucket this lane reads
  const int grp = lane >> 4;          // which of the 4 buckets of a batch
  const uint32_t n_buckets = c.bucket_mask + 1;
  int32_t query_oldest_first[QC];     // [x] = Q[q - 1 - x]
#pragma unroll
  for (int x = 0; x < QC; ++x) query_oldest_first[x] = pick_n<QC>(c.Q, c.q - 1 - x);
  uint32_t width = FIRST;             // buckets of this batch
  for (uint32_t r0 = 0; r0 < n_buckets; r0 += width, width = 4) {
    consume_here(word);
    const bool in_batch = (uint32_t)grp < width;
    if (!in_batch || r0 + grp >= n_buckets) word = -1;
    int32_t count = __shfl(word, lane & ~15);
    bool full = count >= kBucketSlots;
    bool seq_ends = wave_ballot(in_batch && (!full || r0 + grp >= n_buckets)) != 0;
    int32_t next_word = -1;           // next batch: in flight while this one is processed
    if (!seq_ends) {
      uint32_t r = r0 + width + grp;
      next_word = gram_bucket(tbl, gh, r < n_buckets ? r : 0u, c.bucket_mask)[sub];
    }
    bool cand = sub >= 1 && word >= 0 && (sub - 1) < (full ? kBucketSlots : count);
    int32_t j = y.pos_path(word), e = y.pos_index(word), old_j = 0, new_j = 0;
    cand = cand && j != (GENERAL ? c.skip : c.i) && j < y.N;
    if (cand) {
      lens_of(s, y, j, old_j, new_j);
      cand = e < old_j;               // newer positions are matched directly, not looked up
    }
    int32_t wv[LCAP];
    uint32_t wp[LCAP];
#pragma unroll
    for (int d = 0; d < LCAP; ++d) {
      wv[d] = 0;
      wp[d] = 0;
    }
    bool hit = cand;
    int32_t rem = 0, n_hist = 0;
    if (cand) {
      const int32_t* hrow = y.tok + y.cell(j, e);        // history of path j at the posting
      const uint32_t* prow = y.pq + y.cell(j, e);
      // the gram before the posting as ONE run of QC tokens from e - q on (e >= q: inside the
      // path; the run may reach into the continuation, which is padded): loaded token by token
      // behind the comparisons, every token was a dependent fetch of its own
      int32_t gram_at[QC];
#pragma unroll
      for (int x = 0; x < QC; ++x) gram_at[x] = hrow[x - c.q];
      rem = new_j - e;
      rem = rem < L ? rem : L;
      n_hist = old_j - e;             // >= 1: continuation tokens that are already history
      n_hist = n_hist < rem ? n_hist : rem;
      // the whole window with a few wide loads, whatever part of it is valid: what lies
      // beyond n_hist is replaced below or never looked at (the arrays are padded for it)
#pragma unroll
      for (int d = 0; d < LCAP; ++d) {
        wv[d] = hrow[d];
        wp[d] = prow[d];
      }
      int32_t differ = 0;             // (OR of differences: no comparison behind a branch)
#pragma unroll
      for (int x = 0; x < QC; ++x) differ |= x < c.q ? (gram_at[x] ^ query_oldest_first[x]) : 0;
      hit = differ == 0;
    }
    if (wave_ballot(hit && rem > n_hist) != 0) {            // rare: runs into this step's new tokens
#pragma unroll
      for (int d = 0; d < LCAP; ++d)
        if (hit && d >= n_hist && d < rem) {
          wv[d] = y.token(j, e + d, old_j);
          wp[d] = y.prob(j, e + d, old_j);
        }
    }
    int32_t slot = wave_push(s, n_match, hit, make_match(y, j, e, old_j, new_j), lane);
    int32_t w = slot;                 // a match's window has the match's number
    if (slot >= 0 && w < win_cap) {
      int32_t* win = s.win + w * 2 * L;
      if (L == LCAP) {                // the whole window at once; entries beyond rem are never read
#pragma unroll
        for (int d = 0; d < LCAP; ++d) {
          win[d] = wv[d];
          win[LCAP + d] = (int32_t)wp[d];
        }
      } else {
#pragma unroll
        for (int d = 0; d < LCAP; ++d)
          if (d < rem) {
            win[d] = wv[d];
            win[L + d] = (int32_t)wp[d];
          }
      }
    }
    if (seq_ends) break;
    word = next_word;
  }
}

// The front end of a row handled by one wave: round trip 1 (heads, query, own
// append), matches among the newest positions, index lookup with windows.
// Returns the number of matches; wi tells build_dag which of them have windows;
// the ticket, if used, must be finished with insert_finish by the caller.
// QC: compile-time bound of the index's gram length kmax (4 or 8): the loops
// over query tokens are unrolled to it, and the common step is bound by the
// instructions one wave issues.
// APPENDS: the wave also appends the row's token and files it in the index (false: another
// wave of the workgroup does, see wave_append).
template <int LCAP, int QC, bool APPENDS = true, bool GENERAL = false, class LDS>
__device__ __forceinline__ int32_t wave_front_end(LDS& s, Ctx& c, const IndexView& ix, int32_t p,
                                                  int32_t k, int32_t L, WinInfo& wi,
                                                  InsertTicket& ticket, bool& ticket_used) {
  const int lane = c.tid;
  const Paths& y = c.y;
  const int64_t row = (int64_t)p * ix.N + c.i;
  int32_t* gram = const_cast<int32_t*>(c.gram);
  // ---- round trip 1: every load here has an address known from the kernel arguments.  They
  // are per-lane loads issued together; the row's own head and step token are then read from
  // lane i (a load of their own, with the same address in every lane, would be a scalar one
  // whose round trip the compiler puts BEFORE these)
  const int32_t jl = lane < y.N ? lane : 0;
  int32_t st_j = y.n == 1 ? y.st[jl] : 0;               // (before the head: its lengths wait for it)
  Head hj = load_head<QC>(y, ix.tail_len, jl);
  // a step of several tokens per path (general kernels): the step's tokens and the paths' old
  // tails go to LDS (laid over the table, which nothing uses before the walk) when they fit, so
  // that the query and the matches among the appended positions need no further round trip
  const bool multi = GENERAL && y.n > 1;
  constexpr int kStageWords = (int)(sizeof(s.table) / (sizeof(int32_t)));
  const bool staged = multi && y.N * (y.n + QC) <= kStageWords;
  int32_t* stage = reinterpret_cast<int32_t*>(s.table);   // [N][n] the step's tokens
  int32_t* tails = stage + y.N * y.n;                     // [N][QC] tokens before the old ends
  if (GENERAL && staged)
    for (int32_t x = lane; x < y.N * y.n; x += kWave) stage[x] = y.st[x];
  Head me;
  int32_t st_i;
  if (c.i < kWave) {
    me.old_len = __builtin_amdgcn_readlane(hj.old_len, c.i);
    me.new_len = __builtin_amdgcn_readlane(hj.new_len, c.i);
#pragma unroll
    for (int a = 0; a < kTailCap; ++a) me.tail[a] = a < QC ? __builtin_amdgcn_readlane(hj.tail[a], c.i) : 0;
    st_i = __builtin_amdgcn_readlane(st_j, c.i);
  } else {
    me = load_head<QC>(y, ix.tail_len, c.i);
    st_i = y.n == 1 ? y.st[c.i] : 0;
  }
  float sp_i = 1.0f;
  if (APPENDS && y.n == 1 && y.sp) sp_i = y.sp[c.i];
  const int32_t old_i = me.old_len, cnt_i = me.new_len - me.old_len;
  c.len_i = me.new_len;
  c.q = k < c.len_i ? k : c.len_i;
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a) {
    int32_t v = 0;
    if (a < QC && a < c.q) v = a < cnt_i ? st_i : pick_n<QC>(me.tail, a - cnt_i);
    c.Q[a] = v;
  }
  if (GENERAL && staged) {
    block_sync<kWave>();                                // the staged tokens are in LDS
#pragma unroll
    for (int a = 0; a < QC; ++a)
      if (a < c.q && a < cnt_i) c.Q[a] = stage[c.i * y.n + cnt_i - 1 - a];
  } else if (multi) {
    load_query(c, k, old_i);                            // (one more round trip: from the step's input)
  }
  const bool use_index = c.q == ix.kmax;                // shorter queries: scan (short paths)
  // ---- round trip 2 is requested: fill counts for the insert, first buckets of the query
  // (four of each; one with the layout of launches of thousands of rows, whose time is set by
  // what all rows together fetch and issue, not by a row's latency)
  constexpr int kFirst = std::is_same<LDS, LdsWaveSmall>::value ? 1 : 4;
  ticket_used = APPENDS && y.n == 1 && cnt_i == 1;   // (longer steps are appended by append_row)
  if (ticket_used) ticket = insert_begin<QC, kFirst>(gram, c.bucket_mask, ix.kmax, me.tail, old_i, lane);
  GramHash gh{0u, 1u};
  int32_t word = -1;
  if (use_index) {
    gh = query_hash<QC>(c);
    uint32_t r = (uint32_t)(lane >> 4);
    if (kFirst == 4 || r == 0)
      word = gram_bucket(gram, gh, r <= c.bucket_mask ? r : 0u, c.bucket_mask)[lane & 15];
  }
  // ---- while it travels: own append, lengths into LDS, matches among the new positions
  if (APPENDS && y.n == 1) append_own_single<QC>(ix, y, row, c.i, me, st_i, sp_i, lane);
  int32_t n_match = 0;
  for (int32_t j0 = 0; j0 < y.N; j0 += kWave) {
    int32_t j = j0 + lane;
    bool have = j < y.N;
    if (j0 > 0) hj = load_head<QC>(y, ix.tail_len, have ? j : 0);
    if (have && j < LDS::kLens) {
      s.len_old[j] = hj.old_len;
      s.len_new[j] = hj.new_len;
    }
    if (GENERAL && staged && have) {
#pragma unroll
      for (int a = 0; a < QC; ++a) tails[j * QC + a] = hj.tail[a];
    }
    // a position appended by this very launch matches when the old tail before it is the query
    bool hit = use_index && !multi && have && j != (GENERAL ? c.skip : c.i) &&
               hj.new_len > hj.old_len && hj.old_len >= c.q;
#pragma unroll
    for (int a = 0; a < QC; ++a) hit = hit && (a >= c.q || hj.tail[a] == c.Q[a]);
    wave_push(s, n_match, hit, make_match(y, j, hj.old_len, hj.old_len, hj.new_len), lane);
  }
  if (GENERAL && multi && use_index) {
    // every position this launch appends, a lane per (path, offset): its gram runs through
    // the old tail and the step's input
    block_sync<kWave>();                                // the lengths are in LDS
    const int32_t pairs = y.N * y.n;
    for (int32_t x0 = 0; x0 < pairs; x0 += kWave) {
      const int32_t x = x0 + lane;
      const int32_t j = x < pairs ? x % y.N : 0;        // (offset-major: the first offsets, which
      int32_t old_j, new_j;                             // most paths have, fill the first rounds)
      lens_of(s, y, j, old_j, new_j);
      const int32_t e = old_j + x / y.N;
      bool hit = x < pairs && j != c.skip && e < new_j && e >= c.q;
      if (wave_ballot(hit) == 0) continue;              // no path has that many new tokens
      if (staged) {
        const int32_t off = hit ? e - old_j : 0;        // new tokens before the position
#pragma unroll
        for (int a = 0; a < QC; ++a) {
          const int32_t t = a < off ? stage[j * y.n + off - 1 - a] : tails[j * QC + (a - off)];
          hit = hit && (a >= c.q || t == c.Q[a]);
        }
      } else {
        // (idle lanes look at the row's own end, where every token of the gram exists)
        hit = gram_equals_query(c, hit ? j : c.i, hit ? e : c.len_i, hit ? old_j : old_i) && hit;
      }
      wave_push(s, n_match, hit, make_match(y, j, e, old_j, new_j), lane);
    }
  }
  if (ticket_used) insert_claim(ticket, gram, c.bucket_mask, lane);   // round trip 3 starts
  wi.n_fresh = n_match;
  wi.win_cap = use_index ? LDS::kWin / (2 * L) : 0;
  if (use_index) {
    lookup_with_windows<LCAP, QC, GENERAL, kFirst>(s, c, L, wi.win_cap, n_match, gh, word);
  } else if (c.q > 0) {
    WaveListSink<LDS> sink{&s, &n_match, lane};
    match_plain<false>(s, c, sink);                     // covers old and new positions alike
    wi.n_fresh = n_match;
  }
  if (lane == 0) s.n_match = n_match;
  return n_match;
}

// The writing half of a step that appends one token per path, run by a wave of its own beside
// the one that drafts: the row's token goes to the history and the meta row, its position to
// the index.  Nothing the drafting waves of this launch read is written here: they take
// positions from the old lengths on from the step's input, and ignore newer postings.
// GENERAL: also compiled for steps of several tokens per path.
// LANES: buckets of the insert's chain whose fill counts are read up front.
template <int QC, bool GENERAL = false, int LANES = kInsertLanes>
__device__ __forceinline__ void wave_append(const Ctx& c, const IndexView& ix, int32_t p) {
  const int lane = c.tid;
  const Paths& y = c.y;
  if (GENERAL && y.n > 1) {
    const int32_t old_i = y.old_len(c.i);
    append_row<kWave, true>(ix, y, p, c.i, old_i, y.new_len(c.i, old_i), lane);
    return;
  }
  if (y.n != 1) return;
  const int64_t row = (int64_t)p * ix.N + c.i;
  int32_t* gram = const_cast<int32_t*>(c.gram);
  Head me = load_head<QC>(y, ix.tail_len, c.i);
  const int32_t st_i = y.st[c.i];
  const float sp_i = y.sp ? y.sp[c.i] : 1.0f;
  const bool ticket_used = me.new_len - me.old_len == 1;
  InsertTicket ticket;
  if (ticket_used) ticket = insert_begin<QC, LANES>(gram, c.bucket_mask, ix.kmax, me.tail, me.old_len, lane);
  append_own_single<QC>(ix, y, row, c.i, me, st_i, sp_i, lane);
  if (ticket_used) {
    insert_claim(ticket, gram, c.bucket_mask, lane);
    insert_finish(ticket, gram, c.bucket_mask, y.pos(c.i, me.new_len - 1), lane);
  }
}

// ---------------------------------------------------------------- one edit through the index

// Does a posting found in the chain of the query's variant u — filed there as
// variant v of the gram G[0 .. q) before its position (newest first, like Q) —
// count?  It does if the two variants are the same string (chains can share a
// bucket, and hashes collide) and no earlier variant of the query is a variant
// of G as well: a position is filed under every distinct variant of its gram,
// so it turns up once for every variant it shares with the query, and is
// counted for the first.  (Variant 0: the string itself; w >= 1: without its
// token w-1.)
//   Q - a == G - b  (a <= b)  <=>  Q, G agree before a and after b, and
//                                  Q[x+1] == G[x] for a <= x < b;
//   Q - a == G - b  (a >  b)  <=>  they agree before b and after a, and
//                                  Q[x] == G[x+1] for b <= x < a.
// With P / S the first / last index where Q and G differ, the b that asks
// least of a given a is max(a, S) in the first case, min(a - 1, P) in the second.
// K: compile-time bound of the query length (the loops are unrolled to it).
template <int K = CSD_MAX_QUERY_LEN>
__device__ __forceinline__ bool variant_counts(const Ctx& c, const int32_t (&G)[K + 1], int32_t u, int32_t v) {
  const int32_t q = c.q;
  int32_t P = q, S = -1;                                 // first / last mismatch
  int32_t up[K + 1], down[K + 1];      // failures of Q[x+1]==G[x] / Q[x]==G[x+1] among x < index
  up[0] = down[0] = 0;
#pragma unroll
  for (int x = 0; x < K; ++x) {
    bool differ = x < q && c.Q[x] != G[x];
    P = (differ && P == q) ? x : P;
    S = differ ? x : S;
    bool in = x + 1 < q;
    up[x + 1] = up[x] + ((in && c.Q[x + 1 < K ? x + 1 : x] != G[x]) ? 1 : 0);
    down[x + 1] = down[x] + ((in && c.Q[x] != G[x + 1]) ? 1 : 0);
  }
  if (S < 0) return u == 0 && v == 0;                    // the gram is the query: counted there
  if (u == 0 || v == 0 || v > q) return false;           // strings of different lengths
  // the same string?
  const int32_t a0 = u - 1, b0 = v - 1;
  bool same = a0 <= b0 ? (a0 <= P && b0 >= S && pick(up, b0) == pick(up, a0))
                       : (b0 <= P && a0 >= S && pick(down, a0) == pick(down, b0));
  // an earlier variant of the query that G shares?
  bool earlier = false;
#pragma unroll
  for (int a = 0; a < K; ++a) {
    if (a >= q) continue;
    int32_t b1 = a > S ? a : S;                          // Q - a == G - b1 ?
    bool first = a <= P && pick(up, b1) == up[a];
    int32_t b2 = a - 1 < P ? a - 1 : P;                  // Q - a == G - b2 ?
    bool second = a >= 1 && a >= S && down[a] == pick(down, b2);
    earlier = earlier || (a < a0 && (first || second));
  }
  return same && !earlier;
}

// One batch of the variant lookup: this lane's word of a bucket (word 0 = fill
// count, held by the first lane of each group of 16; -1 everywhere for an idle
// group).  Every posting fetches the tokens the predicate looks at together
// with its continuation (one round trip, as in lookup_with_windows); a verified
// position counts once, whichever variants led to it (my_u: the variant whose
// chain this bucket belongs to).  Returns whether the group's bucket was full
// (its chain goes on).
// Which lanes of a batch hold a posting (word 0 of a bucket is its fill count, held by the
// first lane of each group of 16; -1 everywhere for an idle group), and is the group's bucket
// full (its chain goes on)?
__device__ __forceinline__ bool bucket_has_posting(int32_t word, int lane, bool& full) {
  const int sub = lane & 15;          // word of the bucket this lane reads
  const int32_t count = __shfl(word, lane & ~15);
  full = count >= kBucketSlots;
  return sub >= 1 && word >= 0 && (sub - 1) < (full ? kBucketSlots : count);
}

// The postings of a batch, one per lane (`cand`: this lane has one; `my_u`: the query variant
// whose chain it was found in).
template <int LCAP, int K, class LDS>
__device__ __forceinline__ void consume_variant_postings(LDS& s, const Ctx& c, int32_t L,
                                                         int32_t win_cap, int32_t& n_match,
                                                         int32_t my_u, int32_t word, bool cand) {
  const int lane = c.tid;
  const Paths& y = c.y;
  const int32_t filed_as = word >> kVariantShift;       // variant of its gram the posting stands for
  const int32_t pos = word & ((1 << kVariantShift) - 1);
  int32_t j = y.pos_path(pos), e = y.pos_index(pos), old_j = 0, new_j = 0;
  cand = cand && j != c.skip && j < y.N && e >= c.q;    // postings are filed for e >= kmax only
  if (cand) {
    lens_of(s, y, j, old_j, new_j);
    cand = e < old_j;                 // newer positions are matched directly, not looked up
  }
  int32_t tv[K + 1];
  int32_t wv[LCAP];
  uint32_t wp[LCAP];
#pragma unroll
  for (int a = 0; a <= K; ++a) tv[a] = 0;
#pragma unroll
  for (int d = 0; d < LCAP; ++d) {
    wv[d] = 0;
    wp[d] = 0;
  }
  int32_t rem = 0, n_hist = 0;
  if (cand) {
    const int32_t* hrow = y.tok + y.cell(j, e);          // history of path j at the posting
    const uint32_t* prow = y.pq + y.cell(j, e);
#pragma unroll
    for (int a = 0; a <= K; ++a)                         // e >= q: only token q may not exist
      if (a <= c.q) tv[a] = hrow[a < e ? -1 - a : -1];
    rem = new_j - e;
    rem = rem < L ? rem : L;
    n_hist = old_j - e;               // >= 1: continuation tokens that are already history
    n_hist = n_hist < rem ? n_hist : rem;
    // the whole window with a few wide loads, whatever part of it is valid: what lies beyond
    // n_hist is replaced below or never looked at (the arrays are padded for it)
#pragma unroll
    for (int d = 0; d < LCAP; ++d) {
      wv[d] = hrow[d];
      wp[d] = prow[d];
    }
#pragma unroll
    for (int a = 0; a <= K; ++a) tv[a] = (a <= c.q && a < e) ? tv[a] : 0;
  }
  // each position once: for the first variant it shares with the query
  bool hit = cand && near_query<K>(c, e, tv) && variant_counts<K>(c, tv, my_u, filed_as);
  if (wave_ballot(hit && rem > n_hist) != 0) {              // rare: runs into this step's new tokens
#pragma unroll
    for (int d = 0; d < LCAP; ++d)
      if (hit && d >= n_hist && d < rem) {
        wv[d] = y.token(j, e + d, old_j);
        wp[d] = y.prob(j, e + d, old_j);
      }
  }
  int32_t slot = wave_push(s, n_match, hit, make_match(y, j, e, old_j, new_j), lane);
  int32_t w = slot;                   // a match's window has the match's number
  if (slot >= 0 && w < win_cap) {
    int32_t* win = s.win + w * 2 * L;
    if (L == LCAP) {                  // the whole window at once; entries beyond rem are never read
#pragma unroll
      for (int d = 0; d < LCAP; ++d) {
        win[d] = wv[d];
        win[LCAP + d] = (int32_t)wp[d];
      }
    } else {
#pragma unroll
      for (int d = 0; d < LCAP; ++d)
        if (d < rem) {
          win[d] = wv[d];
          win[L + d] = (int32_t)wp[d];
        }
    }
  }
}

// One batch by position: this lane's word of its group's bucket.  Returns whether the
// group's bucket was full.
template <int LCAP, int K, class LDS>
__device__ __forceinline__ bool consume_variant_bucket(LDS& s, const Ctx& c, int32_t L,
                                                       int32_t win_cap, int32_t& n_match,
                                                       int32_t my_u, int32_t word) {
  bool full;
  const bool cand = bucket_has_posting(word, c.tid, full);
  consume_variant_postings<LCAP, K>(s, c, L, win_cap, n_match, my_u, word, cand);
  return full;
}

// Eq. 4 (one edit) through the index.  Bucket 0 of the chains of the query's variants is
// read in batches of four, one variant per group of 16 lanes; a chain that goes on is then
// walked by the whole wave, four buckets per batch with the next batch in flight (reading
// past the end of a chain is harmless: buckets behind the first one that is not full are
// empty).  `word` / `word_beyond`: the lane's word of bucket 0 of its group's variant in the
// first batch (variants 0 .. 3) / the second (4 .. 7), both already requested.
template <int LCAP, int K, class LDS>
__device__ __forceinline__ void lookup_variants_with_windows(LDS& s, const Ctx& c, int32_t L,
                                                             int32_t win_cap, int32_t& n_match,
                                                             int32_t word, int32_t word_beyond) {
  const int lane = c.tid;
  int32_t* tbl = const_cast<int32_t*>(c.gram);
  const int sub = lane & 15;
  const int grp = lane >> 4;
  const uint32_t n_buckets = c.bucket_mask + 1;
  // variants 0 .. 3 and 4 .. 7: both batches of first buckets were requested together.  Buckets
  // are a third full on average, so the postings of the second batch nearly always find a
  // lane of their own among those that hold none of the first, and both are looked through at
  // once (through a small LDS array: the x-th posting of the second batch goes to the x-th
  // such lane).  Queries of 8 tokens have a ninth variant: a batch of its own.
  const int32_t u_a = grp, u_b = 4 + grp, u_c = 8 + grp;
  const bool active_a = u_a <= c.q && variant_is_new(c.Q, u_a);
  const bool active_b = u_b <= c.q && variant_is_new(c.Q, u_b);
  const bool active_c = K >= 8 && u_c <= c.q && variant_is_new(c.Q, 8);
  consume_here(word);
  consume_here(word_beyond);
  if (!active_a) word = -1;           // idle groups see an empty bucket
  if (!active_b) word_beyond = -1;
  int32_t word_ninth = -1;
  if (K >= 8 && c.q >= 8)             // (travels while the others are looked through)
    word_ninth = gram_bucket(tbl, variant_hash(c.Q, c.q, 8), 0u, c.bucket_mask)[sub];
  bool full_a, full_b, full_c = false;
  const bool has_a = bucket_has_posting(word, lane, full_a);
  const bool has_b = bucket_has_posting(word_beyond, lane, full_b);
  const u64 mask_a = wave_ballot(has_a), mask_b = wave_ballot(has_b);
  const u64 below = (1ull << lane) - 1ull;
  const bool together = mask_b != 0 && __popcll(mask_b) <= kWave - __popcll(mask_a);   // uniform over the wave
  int32_t posting = word, my_u = u_a;
  bool cand = has_a;
  if (together) {
    int32_t* moved = reinterpret_cast<int32_t*>(s.link);              // (the links are not in use yet)
    static_assert(sizeof(s.link) >= 2 * kWave * sizeof(int32_t), "room for a batch of postings");
    if (has_b) {
      const int x = (int)__popcll(mask_b & below);
      moved[2 * x] = word_beyond;
      moved[2 * x + 1] = u_b;
    }
    lds_barrier<kWave>();
    const int x = (int)__popcll(~mask_a & below);                     // this lane's number among the free ones
    const bool takes = !has_a && x < (int)__popcll(mask_b);
    posting = takes ? moved[2 * x] : word;
    my_u = takes ? moved[2 * x + 1] : u_a;
    cand = has_a || takes;
  }
  // the batches of first buckets: both at once, or one after the other; then the ninth variant's
#pragma unroll 1
  for (int batch = 0; batch < 3; ++batch) {
    if (batch == 1) {
      if (together || mask_b == 0) continue;             // uniform over the wave
      posting = word_beyond;
      my_u = u_b;
      cand = has_b;
    } else if (batch == 2) {
      if (!(K >= 8 && c.q >= 8)) break;
      consume_here(word_ninth);
      if (!active_c) word_ninth = -1;
      posting = word_ninth;
      my_u = u_c;
      cand = bucket_has_posting(word_ninth, lane, full_c);
    }
    consume_variant_postings<LCAP, K>(s, c, L, win_cap, n_match, my_u, posting, cand);
  }
  // a chain that goes on beyond its first bucket: walked by the whole wave, four buckets per
  // batch with the next batch in flight
  const u64 on_a = wave_ballot(active_a && full_a && sub == 0);       // bit 16 g: group g's chain
  const u64 on_b = wave_ballot(active_b && full_b && sub == 0);
  const u64 on_c = wave_ballot(active_c && full_c && sub == 0);
#pragma unroll 1
  for (int chain = 0; chain < 12; ++chain) {
    const u64 goes_on = chain < 4 ? on_a : chain < 8 ? on_b : on_c;
    if ((goes_on >> (16 * (chain & 3)) & 1ull) == 0) continue;        // uniform over the wave
    const GramHash gh = variant_hash(c.Q, c.q, chain);                // the same in every lane
    uint32_t r0 = 1;
    int32_t tail = gram_bucket(tbl, gh, r0 + grp < n_buckets ? r0 + grp : 0u, c.bucket_mask)[sub];
    for (; r0 < n_buckets; r0 += 4) {
      consume_here(tail);
      if (r0 + grp >= n_buckets) tail = -1;
      uint32_t rn = r0 + 4 + grp;                                     // next batch: in flight meanwhile
      int32_t next_tail = gram_bucket(tbl, gh, rn < n_buckets ? rn : 0u, c.bucket_mask)[sub];
      bool tail_full = consume_variant_bucket<LCAP, K>(s, c, L, win_cap, n_match, chain, tail);
      if (wave_ballot(!tail_full) != 0) break;                         // the chain ends in this batch
      tail = next_tail;
    }
  }
}

// The writing half of a one-token step when the index files every position under its gram's
// variants: as wave_append, by a wave of its own beside the one that drafts.
__device__ __forceinline__ void wave_append_fuzzy(const Ctx& c, const IndexView& ix, int32_t p) {
  const int lane = c.tid;
  const Paths& y = c.y;
  if (y.n != 1) return;
  const int64_t row = (int64_t)p * ix.N + c.i;
  int32_t* gram = const_cast<int32_t*>(c.gram);
  Head me = load_head(y, ix.tail_len, c.i);
  const int32_t st_i = y.st[c.i];
  const float sp_i = y.sp ? y.sp[c.i] : 1.0f;
  const bool ticket_used = me.new_len - me.old_len == 1;
  VariantTicket ticket;
  if (ticket_used) ticket = variants_begin(gram, c.bucket_mask, ix.kmax, me.tail, me.old_len, lane);
  append_own_single(ix, y, row, c.i, me, st_i, sp_i, lane);
  if (ticket_used) {
    variants_claim(ticket, gram, c.bucket_mask, lane);
    variants_beyond_four(ticket, gram, c.bucket_mask, ix.kmax, me.tail, y.pos(c.i, me.old_len), lane);
    variants_finish(ticket, gram, c.bucket_mask, y.pos(c.i, me.new_len - 1), lane);
  }
}

// The front end of a row handled by one wave when matching tolerates one edit
// and the index files every position under its gram's variants.  Same three
// round trips as wave_front_end.  Matched directly, without the index: the
// position this launch appends to each other path (from the old tails, which
// keep kmax + 1 tokens for that) and position kmax - 1 of each other path (the
// only one with fewer than kmax tokens before it that can match a kmax-token
// query).  Returns the number of matches.
// K: compile-time bound (4 or 8) of the index's gram length: the predicates are unrolled to it.
// APPENDS: this wave also appends the row's token and files it (false: another wave does, see
// wave_append_fuzzy).
template <int LCAP, int K = CSD_MAX_QUERY_LEN, bool APPENDS = true, class LDS>
__device__ __forceinline__ int32_t wave_front_end_fuzzy(LDS& s, Ctx& c, const IndexView& ix,
                                                        int32_t p, int32_t k, int32_t L, WinInfo& wi,
                                                        VariantTicket& ticket, bool& ticket_used) {
  const int lane = c.tid;
  const Paths& y = c.y;
  const int64_t row = (int64_t)p * ix.N + c.i;
  int32_t* gram = const_cast<int32_t*>(c.gram);
  // ---- round trip 1: every load here has an address known from the kernel arguments
  Head me = load_head(y, ix.tail_len, c.i);             // same address in every lane
  Head hj = load_head(y, ix.tail_len, lane < y.N ? lane : 0);
  int32_t first_tokens[K];                              // tokens kmax-2 .. 0 of path `lane`, newest first
#pragma unroll
  for (int a = 0; a < K; ++a)
    first_tokens[a] = y.tok[y.cell(lane < y.N ? lane : 0, a < ix.kmax - 1 ? ix.kmax - 2 - a : 0)];
  int32_t st_i = 0;
  float sp_i = 1.0f;
  if (y.n == 1) {
    st_i = y.st[c.i];
    if (y.sp) sp_i = y.sp[c.i];
  }
  const int32_t old_i = me.old_len, cnt_i = me.new_len - me.old_len;
  c.len_i = me.new_len;
  c.q = k < c.len_i ? k : c.len_i;
#pragma unroll
  for (int a = 0; a < K; ++a) {
    int32_t v = 0;
    if (a < c.q) v = a < cnt_i ? st_i : pick(me.tail, a - cnt_i);
    c.Q[a] = v;
  }
  const bool use_index = c.q == ix.kmax;                // shorter queries: scan (short paths)
  // ---- round trip 2 is requested: fill counts for the insert, bucket 0 of the first 4 variants
  ticket_used = APPENDS && cnt_i == 1;
  if (ticket_used) ticket = variants_begin(gram, c.bucket_mask, ix.kmax, me.tail, old_i, lane);
  int32_t word = -1, word_beyond = -1;
  if (use_index) {
    word = gram_bucket(gram, variant_hash(c.Q, c.q, lane >> 4), 0u, c.bucket_mask)[lane & 15];
    const int32_t u_b = 4 + (lane >> 4);                // variants 4 .. 7 (queries of 4 tokens and more)
    word_beyond = gram_bucket(gram, variant_hash(c.Q, c.q, u_b <= c.q ? u_b : 0), 0u, c.bucket_mask)[lane & 15];
  }
  // ---- while it travels: own append, lengths into LDS, matches that need no index
  if (APPENDS && y.n == 1) append_own_single(ix, y, row, c.i, me, st_i, sp_i, lane);
  int32_t n_match = 0;
  for (int32_t j0 = 0; j0 < y.N; j0 += kWave) {
    int32_t j = j0 + lane;
    bool have = j < y.N;
    if (j0 > 0) {
      hj = load_head(y, ix.tail_len, have ? j : 0);
#pragma unroll
      for (int a = 0; a < K; ++a)
        first_tokens[a] = y.tok[y.cell(have ? j : 0, a < ix.kmax - 1 ? ix.kmax - 2 - a : 0)];
    }
    if (have && j < LDS::kLens) {
      s.len_old[j] = hj.old_len;
      s.len_new[j] = hj.new_len;
    }
    const bool other = use_index && have && j != c.skip;
    int32_t t[K + 1];
    // the position appended by this very launch: the tokens before it are the old tail
#pragma unroll
    for (int a = 0; a <= K; ++a) t[a] = (a <= c.q && a < hj.old_len) ? hj.tail[a] : 0;
    bool hit = other && hj.new_len > hj.old_len && near_query<K>(c, hj.old_len, t);
    wave_push(s, n_match, hit, make_match(y, j, hj.old_len, hj.old_len, hj.new_len), lane);
    // position kmax - 1, if it is history: no posting exists for it
#pragma unroll
    for (int a = 0; a <= K; ++a) t[a] = (a < K && a < ix.kmax - 1) ? first_tokens[a < K ? a : 0] : 0;
    hit = other && ix.kmax - 1 < hj.old_len && near_query<K>(c, ix.kmax - 1, t);
    wave_push(s, n_match, hit, make_match(y, j, ix.kmax - 1, hj.old_len, hj.new_len), lane);
  }
  if (ticket_used) {
    variants_claim(ticket, gram, c.bucket_mask, lane);                  // round trip 3 starts
    variants_beyond_four(ticket, gram, c.bucket_mask, ix.kmax, me.tail, y.pos(c.i, old_i), lane);
  }
  wi.n_fresh = n_match;
  wi.win_cap = use_index ? LDS::kWin / (2 * L) : 0;
  if (use_index) {
    lookup_variants_with_windows<LCAP, K>(s, c, L, wi.win_cap, n_match, word, word_beyond);
  } else if (c.q > 0) {
    WaveListSink<LDS> sink{&s, &n_match, lane};
    match_plain<true>(s, c, sink);                      // covers old and new positions alike
    wi.n_fresh = n_match;
  }
  if (lane == 0) s.n_match = n_match;
  return n_match;
}

}  // namespace csd
