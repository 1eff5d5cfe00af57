// csd — consensus speculative drafting for N parallel sampling paths on gfx950.
//
// Device kernels and the C-ABI entry points declared in csd.h.  The method is
// the one of "Speculative Decoding for Multi-Sample Inference": suffix match
// across paths (Eq. 3), layered token DAG with aggregated edge weights (Eq. 5),
// greedy layer-wise extraction (rule after Eq. 5, Algorithm 1), and the greedy
// acceptance check ("Draft acceptance").
//
// Nothing here is a dense contraction, so there is no MFMA: the work is
// integer compares, hash lookups, LDS hash-histogram atomics and wavefront
// reductions.  The step is latency-bound (a chain of a few dependent memory
// round trips per path), so the design minimises round trips and barriers:
//   * one launch per decode step (append + draft + accept fused),
//   * one wave64 per (problem, path): no workgroup barriers on the hot path,
//   * matches come from an incrementally updated n-gram hash index,
//   * DAG tables live in LDS, argmax reductions use DPP lane moves.
//
// Exactness: every weight is an integer (probabilities are quantised to
// 1/65536 at append), so atomics may accumulate in any order and the result is
// still unique.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "csd.h"

namespace {

typedef unsigned long long u64;

constexpr int kWave = 64;
constexpr int kScanBlock = 256;             // threads per row when matches come from a scan
constexpr int kMatchCap = 1024;             // matches kept in LDS; beyond -> streaming tier
constexpr int kTableCap = 1024;             // LDS hash slots for DAG edges + nodes
constexpr int kWinWords = 2048;             // LDS words for cached continuations of matches
constexpr int kLenCache = 256;              // path lengths cached in LDS (more paths: read from memory)
constexpr uint32_t kTokMask = (1u << 29) - 1;
constexpr uint32_t kAnyTok = kTokMask;      // "any predecessor": marks node (in-weight) entries
constexpr u64 kEmpty = ~0ull;
constexpr int kMaxClassBits = 20;           // streaming tier: at most 2^20 token classes
constexpr int kBucketWords = 16;            // one 64-byte line: [count, 15 postings]
constexpr int kBucketSlots = kBucketWords - 1;

// ---------------------------------------------------------------- small helpers

__device__ __forceinline__ uint32_t mix_u64(u64 k) {
  k *= 0x9E3779B97F4A7C15ull;
  k ^= k >> 29;
  k *= 0xBF58476D1CE4E5B9ull;
  return (uint32_t)(k >> 32);
}

// DAG table key: layer d (6 bits) | predecessor u (29) | token v (29).
__device__ __forceinline__ u64 dag_key(int d, uint32_t u, uint32_t v) {
  return ((u64)d << 58) | ((u64)(u & kTokMask) << 29) | (u64)(v & kTokMask);
}
// Eq. 5's two sums in one word: count C (high 24 bits) and probability sum S
// in 1/65536 units (low 40 bits).  N*max_len <= 2^24 keeps both in range.
__device__ __forceinline__ u64 pack_cs(uint32_t c, u64 s) { return ((u64)c << 40) | s; }
__device__ __forceinline__ u64 cs_count(u64 w) { return w >> 40; }
__device__ __forceinline__ u64 cs_sum(u64 w) { return w & ((1ull << 40) - 1); }

// weight * 2^32 = alpha_q * S + (65536 - alpha_q) * C * 65536   (Eq. 5, fixed point)
__device__ __forceinline__ u64 weight_key(u64 w, uint32_t alpha_q) {
  return (u64)alpha_q * cs_sum(w) + (u64)(65536u - alpha_q) * (cs_count(w) << 16);
}
__device__ __forceinline__ float key_to_score(u64 key) {
  return (float)((double)key * (1.0 / 4294967296.0));
}

// Probability -> multiple of 1/65536, round to nearest even, clamped, NaN -> 0.
__device__ __forceinline__ uint32_t quantize_prob(float p) {
  if (!(p == p)) return 0u;
  float x = rintf(p * 65536.0f);   // power-of-two scaling is exact; rintf is half-to-even
  x = fminf(fmaxf(x, 0.0f), 65536.0f);
  return (uint32_t)x;
}

// ---------------------------------------------------------------- argmax reductions

struct Cand {      // a successor proposed for the greedy step
  u64 key;         // its weight * 2^32
  int32_t v;       // its token id; INT_MAX = none
};
__device__ __forceinline__ Cand cand_none() { return Cand{0ull, INT_MAX}; }
// larger weight wins, equal weights go to the lower token id
__device__ __forceinline__ Cand cand_best(Cand a, Cand b) {
  bool take_b = (b.key > a.key) || (b.key == a.key && b.v < a.v);
  return take_b ? b : a;
}

// One DPP step: every lane combines its candidate with the one the lane-move
// pattern CTRL delivers; lanes the pattern does not reach combine with "none".
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ Cand dpp_step(Cand c) {
  const Cand none = cand_none();
  Cand x;
  uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)none.key, (int)(uint32_t)c.key,
                                                      CTRL, ROW_MASK, 0xF, false);
  uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)(none.key >> 32),
                                                      (int)(uint32_t)(c.key >> 32), CTRL, ROW_MASK,
                                                      0xF, false);
  x.key = ((u64)hi << 32) | lo;
  x.v = __builtin_amdgcn_update_dpp(none.v, c.v, CTRL, ROW_MASK, 0xF, false);
  return cand_best(c, x);
}

// Argmax over the 64 lanes of a wave; every lane gets the result.  Four
// row_shr steps scan each row of 16 lanes, row_bcast:15 and row_bcast:31 carry
// the row results up, lane 63 ends with the total.
__device__ __forceinline__ Cand wave_argmax(Cand c) {
  c = dpp_step<0x111, 0xF>(c);   // row_shr:1
  c = dpp_step<0x112, 0xF>(c);   // row_shr:2
  c = dpp_step<0x114, 0xF>(c);   // row_shr:4
  c = dpp_step<0x118, 0xF>(c);   // row_shr:8
  c = dpp_step<0x142, 0xA>(c);   // row_bcast:15 into rows 1 and 3
  c = dpp_step<0x143, 0xC>(c);   // row_bcast:31 into rows 2 and 3
  Cand r;
  uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)c.key, 63);
  uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(c.key >> 32), 63);
  r.key = ((u64)hi << 32) | lo;
  r.v = __builtin_amdgcn_readlane(c.v, 63);
  return r;
}

// ---------------------------------------------------------------- device state

struct IndexView {              // device state inside the caller's workspace
  int32_t* tok;                 // [P][N][max_len] token histories
  uint32_t* pq;                 // [P][N][max_len] quantised generation probabilities
  const int32_t* meta_old;      // [P][N][meta_stride] before this launch: {length, last kmax
                                //   tokens newest first}: one aligned load tells a path's end
  int32_t* meta_new;            // same rows after it (may alias meta_old when nothing else reads)
  int32_t meta_stride;          // ints per row: 1 + kmax rounded up to a multiple of 4
  uint32_t* status;             // sticky CSD_STATUS_* bits
  int32_t* gram;                // n-gram index [P][kmax][n_buckets][16], or null (scan mode)
  uint32_t bucket_mask;         // n_buckets - 1 (power of two)
  int32_t P, N, max_len, vocab, kmax;
};

struct StepIn {                 // tokens a step appends; n == 0: none
  const int32_t* tok;           // [P][N][n]
  const float* prob;            // [P][N][n] or null
  const int32_t* counts;        // [P][N] or null
  int32_t n;
};

// One problem's paths as they are AFTER this step's append, readable while the
// append is still in flight: positions below the old length come from the
// history, newer ones straight from the step's input.  No workgroup ever reads
// history cells that another workgroup of the same launch writes.
struct Paths {
  const int32_t* tok;
  const uint32_t* pq;
  const int32_t* meta_old;
  const int32_t* st;
  const float* sp;
  const int32_t* sc;
  int32_t n, N, max_len, meta_stride;

  __device__ __forceinline__ int32_t old_len(int32_t j) const {
    return meta_old[(int64_t)j * meta_stride];
  }
  __device__ __forceinline__ int32_t new_len(int32_t j, int32_t old_j) const {
    if (n == 0) return old_j;
    int32_t c = sc ? sc[j] : n;
    c = c < 0 ? 0 : (c > n ? n : c);
    int32_t room = max_len - old_j;
    return old_j + (c < room ? c : room);
  }
  __device__ __forceinline__ int32_t token(int32_t j, int32_t t, int32_t old_j) const {
    return t < old_j ? tok[(int64_t)j * max_len + t] : st[(int64_t)j * n + (t - old_j)];
  }
  __device__ __forceinline__ uint32_t prob(int32_t j, int32_t t, int32_t old_j) const {
    if (t < old_j) return pq[(int64_t)j * max_len + t];
    return sp ? quantize_prob(sp[(int64_t)j * n + (t - old_j)]) : 65536u;
  }
};

struct Match {                  // one element of the candidate pool (Eq. 3)
  int32_t off;                  // j * max_len + e: first continuation token
  int16_t rem_new;              // new_len_j - e: continuation tokens that exist, clipped to 63
  int16_t rel_old;              // old_len_j - e, clipped to [-32767, 63]; < 0: e itself is new
};

struct Slot {
  u64 key;
  u64 val;
};

struct Lds {
  Slot table[kTableCap];
  Match match[kMatchCap];
  int32_t win[kWinWords];       // per cached match: L continuation tokens, then their L probabilities
  int32_t len_old[kLenCache];
  int32_t len_new[kLenCache];
  Cand red[2][kScanBlock / kWave];
  int n_match;                  // total matches found (may exceed kMatchCap)
  int n_keys;                   // distinct keys in the table
  int overflow;                 // table ran out of room
};

struct Ctx {                    // one (problem, query path)
  Paths y;
  const int32_t* gram;          // this problem's index tables, or null
  uint32_t bucket_mask;
  int32_t kmax;
  int32_t i;                    // query path
  int32_t len_i;                // its length after the append
  int32_t q;                    // effective query length min(k, len_i)
  int32_t Q[CSD_MAX_QUERY_LEN]; // Q[a] = a-th token from the end of path i
  int tid;
};

// ---------------------------------------------------------------- n-gram hash index
//
// For every gram length g = 1..kmax one table of 64-byte buckets.  A posting
// (j, e) — "the g tokens before index e of path j" — is stored under the hash of
// those g tokens when token e is appended, so a query finds its matches (Eq. 3)
// without touching the histories.  Bucket r of a gram's probe sequence is
// (h + r * step) mod n_buckets with an odd step; an insert goes into the first
// bucket of the sequence that is not full, so a lookup may stop at the first
// bucket that is not full.  Hash collisions are harmless: every posting is
// verified against the history before it counts.

struct GramHash {
  uint32_t h, step;
};
// The hash folds the gram's tokens newest first, so the hashes of all gram
// lengths that end at one position come from one pass over the tokens.
constexpr u64 kGramSeed = 0x243F6A8885A308D3ull;
__device__ __forceinline__ u64 gram_hash_add(u64 acc, int32_t token) {
  acc = (acc ^ (u64)(uint32_t)token) * 0xD6E8FEB86659FD93ull;
  return acc ^ (acc >> 32);
}
__device__ __forceinline__ GramHash gram_hash_end(u64 acc, int g) {
  acc ^= (u64)g * 0x9E3779B97F4A7C15ull;
  uint32_t a = mix_u64(acc);
  uint32_t b = mix_u64(acc ^ 0xA5A5A5A5A5A5A5A5ull);
  return GramHash{a, (b << 1) | 1u};
}
__device__ __forceinline__ int32_t* gram_table(int32_t* gram, int g, uint32_t mask) {
  return gram + (int64_t)(g - 1) * ((int64_t)mask + 1) * kBucketWords;
}
__device__ __forceinline__ int32_t* gram_bucket(int32_t* tbl, GramHash gh, uint32_t r, uint32_t mask) {
  return tbl + (int64_t)((gh.h + r * gh.step) & mask) * kBucketWords;
}

// Slow path of an insert, by one whole wave: reads the fill counts of 64
// buckets of the sequence per round trip, starting at bucket r0, and claims a
// slot in the first one that is not full.  Bounded by the table size; the
// tables hold more slots than there are positions.
__device__ __forceinline__ void gram_insert_from(int32_t* tbl, uint32_t mask, GramHash gh,
                                                 uint32_t r0, int32_t off, int lane) {
  for (; r0 <= mask; r0 += kWave) {
    uint32_t r = r0 + lane;
    bool open = r <= mask && gram_bucket(tbl, gh, r, mask)[0] < kBucketSlots;
    u64 m = __ballot(open);
    while (m) {
      uint32_t first = (uint32_t)__ffsll((long long)m) - 1u;
      int32_t* b = gram_bucket(tbl, gh, r0 + first, mask);
      int32_t c = 0;
      if (lane == 0) c = atomicAdd(b, 1);
      c = __builtin_amdgcn_readfirstlane(c);
      if (c < kBucketSlots) {
        if (lane == 0) b[1 + c] = off;
        return;
      }
      m &= m - 1;                                   // filled up meanwhile: next open bucket
    }
  }
}

// Inserts the postings of position e of path i for every gram length
// g = 1..kmax at once, by one whole wave.  Common case: two memory round trips
// in total (64 fill counts per gram length in flight together, then one
// atomic per gram length issued from different lanes).
__device__ __forceinline__ void gram_insert_position(int32_t* gram, uint32_t mask, int32_t kmax,
                                                     const Paths& y, int32_t i, int32_t e,
                                                     int32_t old_i, int lane) {
  GramHash gh[CSD_MAX_QUERY_LEN];
  int32_t fill[CSD_MAX_QUERY_LEN];
  u64 acc = kGramSeed;
#pragma unroll
  for (int g = 1; g <= CSD_MAX_QUERY_LEN; ++g) {
    bool live = g <= kmax && g <= e;
    acc = gram_hash_add(acc, live ? y.token(i, e - g, old_i) : 0);
    gh[g - 1] = gram_hash_end(acc, g);
    fill[g - 1] = kBucketSlots;
    if (live && (uint32_t)lane <= mask)
      fill[g - 1] = gram_bucket(gram_table(gram, g, mask), gh[g - 1], (uint32_t)lane, mask)[0];
  }
  // lane g-1 claims the slot for gram length g
  int32_t my_first = -1;
  GramHash my_gh{0u, 1u};
#pragma unroll
  for (int g = 1; g <= CSD_MAX_QUERY_LEN; ++g) {
    u64 m = __ballot(fill[g - 1] < kBucketSlots);
    if (lane == g - 1) {
      my_first = m ? (int32_t)__ffsll((long long)m) - 1 : -1;
      my_gh = gh[g - 1];
    }
  }
  const int32_t off = i * y.max_len + e;
  bool mine = lane < kmax && lane + 1 <= e;         // this lane's gram length exists
  bool placed = !mine;
  if (mine && my_first >= 0) {
    int32_t* b = gram_bucket(gram_table(gram, lane + 1, mask), my_gh, (uint32_t)my_first, mask);
    int32_t c = atomicAdd(b, 1);
    if (c < kBucketSlots) {
      b[1 + c] = off;
      placed = true;
    }
  }
  u64 todo = __ballot(!placed);                     // rare: long sequences, or lost a race
  while (todo) {
    int g = (int)__ffsll((long long)todo);          // lane index + 1 == gram length
    todo &= todo - 1;
    GramHash ghg;
    ghg.h = (uint32_t)__builtin_amdgcn_readlane((int)my_gh.h, g - 1);
    ghg.step = (uint32_t)__builtin_amdgcn_readlane((int)my_gh.step, g - 1);
    int32_t from = __builtin_amdgcn_readlane(my_first, g - 1);
    gram_insert_from(gram_table(gram, g, mask), mask, ghg, from < 0 ? kWave : (uint32_t)from, off,
                     lane);
  }
}

template <int BLOCK>
__device__ __forceinline__ void block_sync() {
  __syncthreads();   // a one-wave workgroup needs no hardware barrier: the compiler drops it
}

// Stores this row's share of the step (tokens, quantised probabilities, index
// postings, new length and tail).  Called by all threads of the row's workgroup.
template <int BLOCK, bool WITH_INDEX>
__device__ __forceinline__ void append_row(const IndexView& ix, const Paths& y, int32_t p,
                                           int32_t i, int32_t old_i, int32_t new_i, int tid) {
  int64_t row = (int64_t)p * ix.N + i;
  int32_t cnt = new_i - old_i;
  uint32_t flags = 0;
  // new meta row: word 0 = length, word 1+a = a-th token from the new end.  Every value is
  // read before the barrier and written after it, so the row may be updated in place.
  int32_t meta_val = 0;
  if (tid == 0) meta_val = new_i;
  else if (tid <= ix.kmax) {
    int32_t a = tid - 1;
    if (a < cnt) meta_val = y.st[(int64_t)i * y.n + cnt - 1 - a];
    else if (a - cnt < ix.kmax && a < new_i) meta_val = y.meta_old[(int64_t)i * y.meta_stride + 1 + a - cnt];
  }
  if (tid == 0) {
    int32_t want = y.sc ? y.sc[i] : y.n;
    want = want < 0 ? 0 : (want > y.n ? y.n : want);
    if (want > cnt) flags |= CSD_STATUS_CAPACITY;
  }
  block_sync<BLOCK>();
  if (tid <= ix.kmax) ix.meta_new[row * ix.meta_stride + tid] = meta_val;
  for (int32_t t = tid; t < cnt; t += BLOCK) {
    int32_t v = y.st[(int64_t)i * y.n + t];
    if (v < 0 || v >= ix.vocab) flags |= CSD_STATUS_TOKEN_RANGE;
    ix.tok[row * ix.max_len + old_i + t] = v;
    ix.pq[row * ix.max_len + old_i + t] = y.sp ? quantize_prob(y.sp[(int64_t)i * y.n + t]) : 65536u;
  }
  if (WITH_INDEX && ix.gram) {
    int32_t* gram = ix.gram + (int64_t)p * ix.kmax * ((int64_t)ix.bucket_mask + 1) * kBucketWords;
    for (int32_t t = tid / kWave; t < cnt; t += BLOCK / kWave)     // one wave per new position
      gram_insert_position(gram, ix.bucket_mask, ix.kmax, y, i, old_i + t, old_i, tid & 63);
  }
  if (flags) atomicOr(ix.status, flags);
}

// ---------------------------------------------------------------- matching (Eq. 3)

__device__ __forceinline__ void load_query(Ctx& c, int32_t k, int32_t old_i) {
  c.q = k < c.len_i ? k : c.len_i;
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a)
    c.Q[a] = (a < c.q) ? c.y.token(c.i, c.len_i - 1 - a, old_i) : 0;
}

// Does the q-gram that ends just before index e of path j equal the query?
// All q tokens are fetched at once (one memory round trip, not q).
__device__ __forceinline__ bool gram_equals_query(const Ctx& c, int32_t j, int32_t e,
                                                  int32_t old_j) {
  int32_t t[CSD_MAX_QUERY_LEN];
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a) t[a] = (a < c.q) ? c.y.token(j, e - 1 - a, old_j) : 0;
  bool hit = true;
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a) hit = hit && (a >= c.q || t[a] == c.Q[a]);
  return hit;
}

__device__ __forceinline__ Match make_match(const Ctx& c, int32_t j, int32_t e, int32_t old_j,
                                            int32_t new_j) {
  int32_t rn = new_j - e, ro = old_j - e;
  Match m;
  m.off = j * c.y.max_len + e;
  m.rem_new = (int16_t)(rn > 63 ? 63 : rn);
  m.rel_old = (int16_t)(ro < -32767 ? -32767 : (ro > 63 ? 63 : ro));
  return m;
}

// Compacts hits into the LDS match list with one LDS atomic per wave.
// push() must be reached by all 64 lanes of a wave together.
struct ListSink {
  Lds* s;
  __device__ __forceinline__ void push(bool hit, Match m) {
    u64 mask = __ballot(hit);
    if (mask == 0) return;
    int lane = __lane_id();
    int base = 0;
    if (lane == 0) base = atomicAdd(&s->n_match, (int)__popcll(mask));
    base = __builtin_amdgcn_readfirstlane(base);
    int slot = base + (int)__popcll(mask & ((1ull << lane) - 1ull));
    if (hit && slot < kMatchCap) s->match[slot] = m;
  }
};

// Marks hits in a bitmap over all positions of the problem (debug dump).
struct BitmapSink {
  uint32_t* bits;
  __device__ __forceinline__ void push(bool hit, Match m) {
    if (hit) atomicOr(&bits[m.off >> 5], 1u << (m.off & 31));
  }
};

// Hands every hit to a callable (streaming tier).
template <class F>
struct FnSink {
  F f;
  __device__ __forceinline__ void push(bool hit, Match m) {
    if (hit) f(m);
  }
};

// Eq. 3 by exhaustive comparison: every position e of every other path j with
// q <= e <= len_j - 1 is tested.  Trip counts are uniform over the workgroup;
// four tiles are in flight at a time.
template <int BLOCK, class Sink>
__device__ __forceinline__ void match_scan(const Ctx& c, Sink& sink) {
  constexpr int kUnroll = 4;
  int32_t tiles_per_path = (c.y.max_len + BLOCK - 1) / BLOCK;
  int32_t tiles = c.y.N * tiles_per_path;
  for (int32_t g0 = 0; g0 < tiles; g0 += kUnroll) {
    bool hit[kUnroll];
    Match m[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      int32_t g = g0 + u;
      int32_t j = g / tiles_per_path;
      int32_t e = c.q + (g - j * tiles_per_path) * BLOCK + c.tid;
      hit[u] = false;
      m[u] = Match{0, 0, 0};
      if (g < tiles && j != c.i) {
        int32_t old_j = c.y.old_len(j);
        int32_t new_j = c.y.new_len(j, old_j);
        if (e < new_j) {
          hit[u] = gram_equals_query(c, j, e, old_j);
          m[u] = make_match(c, j, e, old_j, new_j);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) sink.push(hit[u], m[u]);
  }
}

// Eq. 3 through the hash index, by ONE wave.  Postings of earlier steps come
// from the gram's bucket sequence; positions this very launch appends are not
// looked up (their inserts may be in flight) but tested directly.
template <class Sink>
__device__ __forceinline__ void match_index(const Ctx& c, Sink& sink) {
  const int lane = c.tid & 63;
  // (a) positions appended by this launch: e in [max(old_j, q), new_j)
  if (c.y.n > 0) {
    for (int32_t j0 = 0; j0 < c.y.N; j0 += kWave) {
      int32_t j = j0 + lane;
      bool live = j < c.y.N && j != c.i;
      int32_t old_j = live ? c.y.old_len(j) : 0;
      int32_t new_j = live ? c.y.new_len(j, old_j) : 0;
      for (int32_t t = 0; t < c.y.n; ++t) {
        int32_t e = old_j + t;
        bool hit = live && e < new_j && e >= c.q && gram_equals_query(c, j, e, old_j);
        sink.push(hit, make_match(c, j, e, old_j, new_j));
      }
    }
  }
  // (b) postings of earlier launches
  u64 acc = kGramSeed;
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a)
    if (a < c.q) acc = gram_hash_add(acc, c.Q[a]);
  GramHash gh = gram_hash_end(acc, c.q);
  const int32_t* tbl = gram_table(const_cast<int32_t*>(c.gram), c.q, c.bucket_mask);
  const int sub = lane & 15;          // word of the bucket this lane reads
  const int grp = lane >> 4;          // which of the 4 buckets of a batch
  uint32_t n_buckets = c.bucket_mask + 1;
  int per_round = 1;                  // batches of 4 buckets in flight per round trip
  for (uint32_t r0 = 0; r0 < n_buckets; r0 += 4u * per_round, per_round = 4) {
    bool seq_ends = false;
    for (int u = 0; u < per_round; ++u) {   // independent loads: one round trip
      uint32_t r = r0 + 4u * u + grp;
      int32_t word = -1;
      if (r < n_buckets)
        word = tbl[(int64_t)((gh.h + r * gh.step) & c.bucket_mask) * kBucketWords + sub];
      int32_t count = __shfl(word, lane & ~15);
      bool full = count >= kBucketSlots;
      bool cand = sub >= 1 && word >= 0 && (sub - 1) < (full ? kBucketSlots : count);
      int32_t j = 0, e = 0, old_j = 0, new_j = 0;
      bool hit = false;
      if (cand) {
        j = word / c.y.max_len;
        e = word - j * c.y.max_len;
        if (j != c.i && j < c.y.N) {
          old_j = c.y.old_len(j);
          if (e < old_j) {               // postings at or beyond old_j belong to case (a)
            new_j = c.y.new_len(j, old_j);
            hit = gram_equals_query(c, j, e, old_j);
          }
        }
      }
      sink.push(hit, make_match(c, j, e, old_j, new_j));
      if (__ballot(!full || r >= n_buckets) != 0) seq_ends = true;
    }
    if (seq_ends) break;
  }
}

// ---------------------------------------------------------------- LDS hash table

template <int BLOCK>
__device__ __forceinline__ void table_clear(Lds& s, uint32_t mask, int tid) {
  for (uint32_t h = tid; h <= mask; h += BLOCK) s.table[h] = Slot{kEmpty, 0ull};
  if (tid == 0) {
    s.n_keys = 0;
    s.overflow = 0;
  }
}

// table[key] += delta, inserting the key if new.  Sets s.overflow when the
// table is more than 3/4 full (the caller then falls back) — never spins.
__device__ __forceinline__ void table_add(Lds& s, uint32_t mask, u64 key, u64 delta) {
  uint32_t h = mix_u64(key) & mask;
  for (uint32_t probe = 0; probe <= mask; ++probe) {
    u64 cur = s.table[h].key;
    if (cur == kEmpty) {
      cur = atomicCAS(&s.table[h].key, kEmpty, key);
      if (cur == kEmpty) {
        int n = atomicAdd(&s.n_keys, 1) + 1;
        if ((uint32_t)n > (mask + 1) - ((mask + 1) >> 2)) s.overflow = 1;
        cur = key;
      }
    }
    if (cur == key) {
      atomicAdd(&s.table[h].val, delta);
      return;
    }
    h = (h + 1) & mask;
  }
  s.overflow = 1;
}

__device__ __forceinline__ u64 table_get(const Lds& s, uint32_t mask, u64 key) {
  uint32_t h = mix_u64(key) & mask;
  for (uint32_t probe = 0; probe <= mask; ++probe) {
    Slot x = s.table[h];
    if (x.key == key) return x.val;
    if (x.key == kEmpty) return 0ull;
    h = (h + 1) & mask;
  }
  return 0ull;
}

// Workgroup-wide argmax of the per-thread candidates; every thread gets the result.
template <int BLOCK>
__device__ __forceinline__ Cand block_argmax(Lds& s, Cand c, int tid, int parity) {
  c = wave_argmax(c);
  if (BLOCK == kWave) return c;
  if ((tid & 63) == 0) s.red[parity][tid >> 6] = c;
  __syncthreads();
  Cand r = s.red[parity][0];
#pragma unroll
  for (int w = 1; w < BLOCK / kWave; ++w) r = cand_best(r, s.red[parity][w]);
  return r;
}

// Successors of `cur` in layer d as held by the table, best one per thread.
template <int BLOCK>
__device__ __forceinline__ Cand scan_successors(const Lds& s, uint32_t mask, int d, int32_t cur,
                                                uint32_t alpha_q, int score_mode, int tid,
                                                Cand best) {
  u64 want = dag_key(d, (uint32_t)cur, 0) >> 29;
  for (uint32_t h = tid; h <= mask; h += BLOCK) {
    Slot x = s.table[h];
    if ((x.key >> 29) != want) continue;
    uint32_t v = (uint32_t)(x.key & kTokMask);
    u64 w = score_mode ? x.val : table_get(s, mask, dag_key(d, kAnyTok, v));
    best = cand_best(best, Cand{weight_key(w, alpha_q), (int32_t)v});
  }
  return best;
}

struct DraftOut {               // what one thread contributes to the outputs
  int32_t tok = -1;             // thread t keeps layer t+1
  u64 key = 0;
  u64 key_sum = 0;
  int32_t n = 0;
};

// The (u, v, p) instance that match m contributes to layer d, if it reaches it.
__device__ __forceinline__ bool layer_instance(const Ctx& c, Match m, int32_t d, uint32_t& u,
                                               uint32_t& v, u64& w) {
  if (d > (int32_t)m.rem_new) return false;        // the candidate has ended
  int32_t j = m.off / c.y.max_len;
  int32_t e = m.off - j * c.y.max_len;
  // rel_old is exact unless clipped at 63 (a step appends at most 32767 tokens), and
  // d <= 32 < 63: every index read below is then on the history side either way
  int32_t old_j = e + (int32_t)m.rel_old;
  u = (uint32_t)c.y.token(j, e + d - 2, old_j);
  v = (uint32_t)c.y.token(j, e + d - 1, old_j);
  w = pack_cs(1u, c.y.prob(j, e + d - 1, old_j));
  return true;
}

// ---------------------------------------------------------------- tier 1: everything in LDS

// Eq. 5: every (match, layer) instance adds (1, p) to its edge (d,u,v) and to
// its node (d,*,v).  Returns the table mask used.
// Matches n_fresh .. n_fresh + win_cap - 1 of the list have their continuation cached in LDS.
struct WinInfo {
  int32_t n_fresh, win_cap;
};

template <int BLOCK>
__device__ __forceinline__ uint32_t build_dag(Lds& s, const Ctx& c, int32_t M, int32_t L,
                                              WinInfo wi) {
  uint32_t want = 4u * (uint32_t)M * (uint32_t)L;     // <= 50 % load without any merging
  uint32_t size = 64;
  while (size < want && size < (uint32_t)kTableCap) size <<= 1;
  uint32_t mask = size - 1;
  table_clear<BLOCK>(s, mask, c.tid);
  block_sync<BLOCK>();
  int32_t items = M * L;
  for (int32_t idx = c.tid; idx < items; idx += BLOCK) {
    int32_t d = idx / M + 1;
    int32_t mi = idx - (d - 1) * M;
    Match m = s.match[mi];
    uint32_t u, v;
    u64 w;
    bool alive;
    int32_t ws = mi - wi.n_fresh;
    if (ws >= 0 && ws < wi.win_cap) {                 // cached: no memory access
      alive = d <= (int32_t)m.rem_new;
      const int32_t* win = s.win + ws * 2 * L;
      v = (uint32_t)win[d - 1];
      u = d == 1 ? (uint32_t)c.Q[0] : (uint32_t)win[d - 2];
      w = pack_cs(1u, (uint32_t)win[L + d - 1]);
    } else {
      alive = layer_instance(c, m, d, u, v, w);
    }
    if (alive && !s.overflow) {
      table_add(s, mask, dag_key(d, u, v), w);
      table_add(s, mask, dag_key(d, kAnyTok, v), w);
    }
  }
  block_sync<BLOCK>();
  return mask;
}

// Greedy walk over the finished tables (rule after Eq. 5).
template <int BLOCK>
__device__ __forceinline__ void walk_dag(Lds& s, const Ctx& c, uint32_t mask, int32_t L,
                                         uint32_t alpha_q, int score_mode, DraftOut& o) {
  int32_t cur = c.Q[0];
  for (int32_t d = 1; d <= L; ++d) {
    Cand best = scan_successors<BLOCK>(s, mask, d, cur, alpha_q, score_mode, c.tid, cand_none());
    best = block_argmax<BLOCK>(s, best, c.tid, d & 1);
    if (best.v == INT_MAX) break;                     // leaf: no edge leaves cur
    if (c.tid == d - 1) { o.tok = best.v; o.key = best.key; }
    o.key_sum += best.key;
    o.n = d;
    cur = best.v;
  }
}

// ---------------------------------------------------------------- tier 2: streaming, layer by layer

template <int BLOCK, bool INDEXED, class Sink>
__device__ __forceinline__ void find_matches(const Ctx& c, Sink& sink) {
  if (INDEXED) match_index(c, sink);
  else match_scan<BLOCK>(c, sink);
}

// Calls f(match) for every match.  Uses the LDS list when it holds all of
// them, else runs the matcher again.
template <int BLOCK, bool INDEXED, class F>
__device__ __forceinline__ void for_each_match(const Lds& s, const Ctx& c, int32_t M, F f) {
  if (M <= kMatchCap) {
    for (int32_t m = c.tid; m < M; m += BLOCK) f(s.match[m]);
  } else {
    FnSink<F> sink{f};
    find_matches<BLOCK, INDEXED>(c, sink);
  }
}

// Same result as build_dag + walk_dag with bounded memory for any input: one
// layer at a time, and within a layer one class of tokens (by hash residue)
// at a time, doubling the number of classes whenever a class overflows LDS.
template <int BLOCK, bool INDEXED>
__device__ __forceinline__ void walk_streaming(Lds& s, const Ctx& c, int32_t M, int32_t L,
                                               uint32_t alpha_q, int score_mode,
                                               uint32_t* status, DraftOut& o) {
  const uint32_t mask = kTableCap - 1;
  int32_t cur = c.Q[0];
  int class_bits = 0;
  int parity = 0;
  for (int32_t d = 1; d <= L; ++d) {
    Cand best;
    bool failed;
    do {
      failed = false;
      best = cand_none();
      uint32_t n_class = 1u << class_bits;
      for (uint32_t r = 0; r < n_class && !failed; ++r) {
        block_sync<BLOCK>();                           // previous readers are done
        table_clear<BLOCK>(s, mask, c.tid);
        block_sync<BLOCK>();
        for_each_match<BLOCK, INDEXED>(s, c, M, [&](Match m) {
          uint32_t u, v;
          u64 w;
          if (s.overflow || !layer_instance(c, m, d, u, v, w)) return;
          if ((mix_u64(v) & (n_class - 1)) != r) return;
          table_add(s, mask, dag_key(d, kAnyTok, v), w);
          if (u == (uint32_t)cur) table_add(s, mask, dag_key(d, u, v), w);
        });
        block_sync<BLOCK>();
        if (s.overflow) failed = true;                 // uniform: read after the barrier
        else best = scan_successors<BLOCK>(s, mask, d, cur, alpha_q, score_mode, c.tid, best);
      }
      if (failed) ++class_bits;
    } while (failed && class_bits <= kMaxClassBits);
    if (failed) {                                      // 2^20 classes did not suffice
      if (c.tid == 0) atomicOr(status, CSD_STATUS_TABLE_FULL);
      break;
    }
    parity ^= 1;
    best = block_argmax<BLOCK>(s, best, c.tid, parity);
    if (best.v == INT_MAX) break;
    if (c.tid == d - 1) { o.tok = best.v; o.key = best.key; }
    o.key_sum += best.key;
    o.n = d;
    cur = best.v;
  }
}

// ---------------------------------------------------------------- kernels

// Workgroups are dealt round-robin to the 8 XCDs; this maps them back so that
// each XCD works on a contiguous range of (problem, path) rows and the paths of
// one problem share one L2.  The grid is padded to a multiple of 8.
__device__ __forceinline__ int32_t xcd_row(int32_t rows) {
  int32_t per_xcd = (int32_t)(gridDim.x >> 3);
  int32_t r = (int32_t)(blockIdx.x & 7) * per_xcd + (int32_t)(blockIdx.x >> 3);
  return r < rows ? r : -1;
}
inline uint32_t xcd_grid(int64_t rows) { return (uint32_t)((rows + 7) / 8 * 8); }

__device__ __forceinline__ Ctx make_ctx(const IndexView& ix, const StepIn& in, int32_t row,
                                        int32_t& p_out) {
  Ctx c;
  int32_t p = row / ix.N;
  p_out = p;
  int64_t cells = (int64_t)p * ix.N * ix.max_len;
  c.i = row - p * ix.N;
  c.y.tok = ix.tok + cells;
  c.y.pq = ix.pq + cells;
  c.y.meta_old = ix.meta_old + (int64_t)p * ix.N * ix.meta_stride;
  c.y.meta_stride = ix.meta_stride;
  c.y.n = in.n;
  c.y.st = in.n ? in.tok + (int64_t)p * ix.N * in.n : nullptr;
  c.y.sp = (in.n && in.prob) ? in.prob + (int64_t)p * ix.N * in.n : nullptr;
  c.y.sc = (in.n && in.counts) ? in.counts + (int64_t)p * ix.N : nullptr;
  c.y.N = ix.N;
  c.y.max_len = ix.max_len;
  c.gram = ix.gram ? ix.gram + (int64_t)p * ix.kmax * ((int64_t)ix.bucket_mask + 1) * kBucketWords
                   : nullptr;
  c.bucket_mask = ix.bucket_mask;
  c.kmax = ix.kmax;
  c.tid = threadIdx.x;
  return c;
}

__global__ __launch_bounds__(256) void reset_kernel(IndexView ix, int64_t gram_words) {
  int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * 256;
  int64_t rows = (int64_t)ix.P * ix.N;
  for (int64_t r = t; r < rows * ix.meta_stride; r += stride) ix.meta_new[r] = 0;
  for (int64_t w = t; w < gram_words; w += stride) ix.gram[w] = (w & (kBucketWords - 1)) ? -1 : 0;
  if (t == 0) *ix.status = 0u;
}

// Append only: one workgroup per (problem, path).
__global__ __launch_bounds__(256) void append_kernel(IndexView ix, StepIn in) {
  int32_t row = blockIdx.x;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);
  int32_t old_i = c.y.old_len(c.i);
  int32_t new_i = c.y.new_len(c.i, old_i);
  append_row<256, true>(ix, c.y, p, c.i, old_i, new_i, c.tid);   // meta_new aliases meta_old here
}

struct DraftArgs {
  int32_t k, L;
  uint32_t alpha_q;
  int32_t score_mode;
  int32_t* draft_tokens;        // [P][N][L]
  int32_t* draft_len;           // [P][N]
  float* token_scores;          // [P][N][L] or null
  float* path_scores;           // [P][N] or null
  const int32_t* targets;       // [P][N][L] or null
  int32_t* accept_len;          // [P][N] or null
};

// One workgroup per (problem, path): [append] -> match (Eq. 3) -> DAG (Eq. 5)
// -> greedy walk -> [accept].  With in.n > 0 the launch also performs the
// step's append; every workgroup then reads the other paths through `Paths`,
// which never touches cells written by this launch.
template <int BLOCK, bool INDEXED>
__global__ __launch_bounds__(BLOCK) void draft_kernel(IndexView ix, StepIn in, DraftArgs a) {
  __shared__ Lds s;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);
  int32_t old_i = c.y.old_len(c.i);
  c.len_i = c.y.new_len(c.i, old_i);
  if (in.n > 0) append_row<BLOCK, true>(ix, c.y, p, c.i, old_i, c.len_i, c.tid);
  load_query(c, a.k, old_i);
  if (c.tid == 0) s.n_match = 0;
  block_sync<BLOCK>();

  DraftOut o;
  const int32_t L = a.L;
  if (c.q > 0) {
    ListSink sink{&s};
    find_matches<BLOCK, INDEXED>(c, sink);
    block_sync<BLOCK>();
    int32_t M = s.n_match;
    if (M > 0) {
      bool streaming = M > kMatchCap;
      if (!streaming) {
        uint32_t mask = build_dag<BLOCK>(s, c, M, L, WinInfo{M, 0});
        streaming = s.overflow != 0;
        if (!streaming) walk_dag<BLOCK>(s, c, mask, L, a.alpha_q, a.score_mode, o);
      }
      if (streaming)
        walk_streaming<BLOCK, INDEXED>(s, c, M, L, a.alpha_q, a.score_mode, ix.status, o);
    }
  }
  bool live = c.tid < o.n;
  if (c.tid < L) {
    a.draft_tokens[(int64_t)row * L + c.tid] = live ? o.tok : -1;
    if (a.token_scores) a.token_scores[(int64_t)row * L + c.tid] = live ? key_to_score(o.key) : 0.0f;
  }
  if (c.tid == 0) {
    a.draft_len[row] = o.n;
    if (a.path_scores) a.path_scores[row] = key_to_score(o.key_sum);
  }
  if (a.targets && c.tid < kWave) {     // "Draft acceptance": first lane whose token differs
    bool same = live && c.tid < L && a.targets[(int64_t)row * L + c.tid] == o.tok;
    u64 differs = __ballot(!same);
    if (c.tid == 0) a.accept_len[row] = differs ? (int32_t)__ffsll((long long)differs) - 1 : kWave;
  }
}


// ---------------------------------------------------------------- the one-wave step kernel
//
// Index mode runs one wave64 per (problem, path).  The step is a chain of
// dependent memory round trips, and each launch starts with a cold L2 (the XCDs'
// L2s are not coherent with each other across launches), so the kernel is laid
// out to need only three of them before the LDS work:
//   1. the meta rows (length + last tokens) of all paths and the step's input:
//      the query, the index hashes and the matches among the newest positions
//      all follow from these without touching the histories;
//   2. the index buckets of the query (and the fill counts for the inserts);
//   3. for every posting found, its verify tokens together with its whole
//      continuation (tokens and probabilities), kept in LDS for the DAG build.

struct Head {                   // a path's end before this step
  int32_t old_len, new_len;
  int32_t tail[CSD_MAX_QUERY_LEN];   // tail[a] = a-th token from the old end
};

__device__ __forceinline__ int32_t pick(const int32_t (&arr)[CSD_MAX_QUERY_LEN], int32_t idx) {
  int32_t r = 0;
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a) r = (idx == a) ? arr[a] : r;
  return r;
}

__device__ __forceinline__ Head load_head(const Paths& y, int32_t kmax, int32_t j) {
  Head h;
  const int4* m = reinterpret_cast<const int4*>(y.meta_old + (int64_t)j * y.meta_stride);
  int4 a = m[0];
  int4 b = kmax > 3 ? m[1] : int4{0, 0, 0, 0};
  int32_t c = kmax > 7 ? y.meta_old[(int64_t)j * y.meta_stride + 8] : 0;
  h.old_len = a.x;
  h.tail[0] = a.y; h.tail[1] = a.z; h.tail[2] = a.w;
  h.tail[3] = b.x; h.tail[4] = b.y; h.tail[5] = b.z; h.tail[6] = b.w;
  h.tail[7] = c;
  h.new_len = y.new_len(j, h.old_len);
  return h;
}

// Split-phase insert of ONE new position into all kmax tables: lanes 8g-8..8g-1
// look at the first 8 buckets of gram length g's sequence.
struct InsertTicket {
  GramHash gh;                  // of this lane's gram length
  int32_t fill;                 // fill count of bucket (lane & 7) of that sequence
  int32_t first;                // first open bucket among the 8, or -1
  int32_t claimed;              // slot the leader lane got from the atomic, or kBucketSlots
  bool live;                    // this lane's gram length exists at this position
};

// Phase 1: hashes of the grams that end just before the new position (they are
// the old tail) and the fill-count loads.
__device__ __forceinline__ InsertTicket insert_begin(int32_t* gram, uint32_t mask, int32_t kmax,
                                                     const Head& me, int lane) {
  InsertTicket t;
  const int g = (lane >> 3) + 1;
  t.gh = GramHash{0u, 1u};
  u64 acc = kGramSeed;
#pragma unroll
  for (int a = 1; a <= CSD_MAX_QUERY_LEN; ++a) {
    acc = gram_hash_add(acc, me.tail[a - 1]);
    GramHash gh = gram_hash_end(acc, a);
    if (a == g) t.gh = gh;
  }
  t.live = g <= kmax && g <= me.old_len;
  t.fill = kBucketSlots;
  t.first = -1;
  t.claimed = kBucketSlots;
  uint32_t r = (uint32_t)(lane & 7);
  if (t.live && r <= mask) t.fill = gram_bucket(gram_table(gram, g, mask), t.gh, r, mask)[0];
  return t;
}

// Phase 2: the leader lane of each gram length claims a slot in the first open bucket.
__device__ __forceinline__ void insert_claim(InsertTicket& t, int32_t* gram, uint32_t mask,
                                             int lane) {
  u64 open = __ballot(t.fill < kBucketSlots);
  uint32_t mine = (uint32_t)(open >> (lane & ~7)) & 0xFFu;
  t.first = mine ? (int32_t)__ffs((int)mine) - 1 : -1;
  if (t.live && (lane & 7) == 0 && t.first >= 0)
    t.claimed = atomicAdd(gram_bucket(gram_table(gram, (lane >> 3) + 1, mask), t.gh,
                                      (uint32_t)t.first, mask), 1);
}

// Phase 3: store the posting; gram lengths whose first 8 buckets were full (or
// that lost a race for the last slot) take the general wave-wide insert.
__device__ __forceinline__ void insert_finish(const InsertTicket& t, int32_t* gram, uint32_t mask,
                                              int32_t off, int lane) {
  bool leader = t.live && (lane & 7) == 0;
  bool placed = !leader;
  if (leader && t.claimed < kBucketSlots) {
    gram_bucket(gram_table(gram, (lane >> 3) + 1, mask), t.gh, (uint32_t)t.first, mask)[1 + t.claimed] = off;
    placed = true;
  }
  u64 todo = __ballot(!placed);
  while (todo) {
    int src = (int)__ffsll((long long)todo) - 1;     // a leader lane: gram length src/8 + 1
    todo &= todo - 1;
    GramHash gh;
    gh.h = (uint32_t)__builtin_amdgcn_readlane((int)t.gh.h, src);
    gh.step = (uint32_t)__builtin_amdgcn_readlane((int)t.gh.step, src);
    int32_t from = __builtin_amdgcn_readlane(t.first, src);
    gram_insert_from(gram_table(gram, (src >> 3) + 1, mask), mask, gh, from < 0 ? 8u : (uint32_t)from,
                     off, lane);
  }
}

// Lengths of path j: from the LDS cache for the first kLenCache paths.
__device__ __forceinline__ void lens_of(const Lds& s, const Paths& y, int32_t j, int32_t& old_j,
                                        int32_t& new_j) {
  if (j < kLenCache) {
    old_j = s.len_old[j];
    new_j = s.len_new[j];
  } else {
    old_j = y.old_len(j);
    new_j = y.new_len(j, old_j);
  }
}

// Appends the hits of all 64 lanes to the match list (one wave: the count lives
// in a register).  Returns each hit's slot, -1 for lanes without one.
__device__ __forceinline__ int32_t wave_push(Lds& s, int32_t& n_match, bool hit, Match m, int lane) {
  u64 mask = __ballot(hit);
  int32_t slot = n_match + (int32_t)__popcll(mask & ((1ull << lane) - 1ull));
  n_match += (int32_t)__popcll(mask);
  if (!hit) return -1;
  if (slot < kMatchCap) s.match[slot] = m;
  return slot;
}

// Eq. 3 through the hash index with the continuations fetched in the same
// round trip as the verification.  Adds its hits behind the n_fresh matches
// already listed; hit number x (0-based among these) gets window x.
template <int LCAP>
__device__ __forceinline__ void lookup_with_windows(Lds& s, const Ctx& c, int32_t L,
                                                    int32_t win_cap, int32_t n_fresh,
                                                    int32_t& n_match, GramHash gh, int32_t word) {
  const int lane = c.tid;
  const int32_t* tbl = gram_table(const_cast<int32_t*>(c.gram), c.q, c.bucket_mask);
  const int sub = lane & 15;          // word of the bucket this lane reads
  const int grp = lane >> 4;          // which of the 4 buckets of a batch
  const uint32_t n_buckets = c.bucket_mask + 1;
  for (uint32_t r0 = 0; r0 < n_buckets; r0 += 4) {
    int32_t count = __shfl(word, lane & ~15);
    bool full = count >= kBucketSlots;
    bool seq_ends = __ballot(!full || r0 + grp >= n_buckets) != 0;
    int32_t next_word = -1;           // next batch: in flight while this one is processed
    if (!seq_ends && r0 + 4 + grp < n_buckets)
      next_word = gram_bucket(const_cast<int32_t*>(tbl), gh, r0 + 4 + grp, c.bucket_mask)[sub];
    bool cand = sub >= 1 && word >= 0 && (sub - 1) < (full ? kBucketSlots : count);
    int32_t j = 0, e = 0, old_j = 0, new_j = 0;
    if (cand) {
      j = word / c.y.max_len;
      e = word - j * c.y.max_len;
      cand = j != c.i && j < c.y.N;
    }
    if (cand) {
      lens_of(s, c.y, j, old_j, new_j);
      cand = e < old_j;               // newer positions are matched directly, not looked up
    }
    int32_t wv[LCAP];
    uint32_t wp[LCAP];
    bool hit = cand;
    int32_t rem = 0;
    if (cand) {
      const int32_t* row = c.y.tok + (int64_t)j * c.y.max_len;
      int32_t tv[CSD_MAX_QUERY_LEN];
#pragma unroll
      for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a) tv[a] = (a < c.q) ? row[e - 1 - a] : 0;
      rem = new_j - e;
      rem = rem < L ? rem : L;
#pragma unroll
      for (int d = 0; d < LCAP; ++d) {
        wv[d] = 0;
        wp[d] = 0;
        if (d < rem) {
          wv[d] = c.y.token(j, e + d, old_j);
          wp[d] = c.y.prob(j, e + d, old_j);
        }
      }
#pragma unroll
      for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a) hit = hit && (a >= c.q || tv[a] == c.Q[a]);
    }
    int32_t slot = wave_push(s, n_match, hit, make_match(c, j, e, old_j, new_j), lane);
    int32_t w = slot - n_fresh;
    if (slot >= 0 && w < win_cap) {
      int32_t* win = s.win + w * 2 * L;
#pragma unroll
      for (int d = 0; d < LCAP; ++d)
        if (d < rem) {
          win[d] = wv[d];
          win[L + d] = (int32_t)wp[d];
        }
    }
    if (seq_ends) break;
    word = next_word;
  }
}

// The front end of a row handled by one wave: round trip 1 (heads, query, own
// append), matches among the newest positions, index lookup with windows.
// Returns the number of matches; wi tells build_dag which of them have windows.
template <int LCAP>
__device__ __forceinline__ int32_t wave_front_end(Lds& s, Ctx& c, const IndexView& ix, int32_t p,
                                                  int32_t k, int32_t L, WinInfo& wi,
                                                  InsertTicket& ticket, bool& ticket_used) {
  const int lane = c.tid;
  const Paths& y = c.y;
  Head me = load_head(y, ix.kmax, c.i);                 // same address in every lane
  const int32_t old_i = me.old_len, cnt_i = me.new_len - me.old_len;
  c.len_i = me.new_len;
  c.q = k < c.len_i ? k : c.len_i;
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a) {
    int32_t v = 0;
    if (a < c.q) v = a < cnt_i ? y.st[(int64_t)c.i * y.n + cnt_i - 1 - a] : pick(me.tail, a - cnt_i);
    c.Q[a] = v;
  }
  int32_t* gram = const_cast<int32_t*>(c.gram);
  ticket_used = false;
  if (y.n > 0) {        // also when this path takes no token: its meta row moves to the new buffer
    append_row<kWave, false>(ix, y, p, c.i, old_i, me.new_len, lane);   // index part: below
    if (cnt_i == 1) {
      ticket = insert_begin(gram, c.bucket_mask, ix.kmax, me, lane);
      ticket_used = true;
    } else {
      for (int32_t t = 0; t < cnt_i; ++t)
        gram_insert_position(gram, c.bucket_mask, ix.kmax, y, c.i, old_i + t, old_i, lane);
    }
  }
  // first batch of index buckets of the query (round trip 2, together with the fill counts)
  GramHash gh{0u, 1u};
  int32_t word = -1;
  if (c.q > 0) {
    u64 acc = kGramSeed;
#pragma unroll
    for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a)
      if (a < c.q) acc = gram_hash_add(acc, c.Q[a]);
    gh = gram_hash_end(acc, c.q);
    if ((uint32_t)(lane >> 4) <= c.bucket_mask)
      word = gram_bucket(gram_table(gram, c.q, c.bucket_mask), gh, (uint32_t)(lane >> 4),
                         c.bucket_mask)[lane & 15];
  }
  // heads of all paths: lengths into LDS, matches among the positions appended by this launch
  int32_t n_match = 0;
  for (int32_t j0 = 0; j0 < y.N; j0 += kWave) {
    int32_t j = j0 + lane;
    bool have = j < y.N;
    Head hj = load_head(y, ix.kmax, have ? j : 0);
    if (have && j < kLenCache) {
      s.len_old[j] = hj.old_len;
      s.len_new[j] = hj.new_len;
    }
    bool live = have && j != c.i && c.q > 0;
    if (y.n == 1) {                         // the usual decode step: compare the old tail
      bool hit = live && hj.new_len > hj.old_len && hj.old_len >= c.q;
#pragma unroll
      for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a) hit = hit && (a >= c.q || hj.tail[a] == c.Q[a]);
      wave_push(s, n_match, hit, make_match(c, j, hj.old_len, hj.old_len, hj.new_len), lane);
    } else {
      for (int32_t t = 0; t < y.n; ++t) {
        int32_t e = hj.old_len + t;
        bool hit = live && e < hj.new_len && e >= c.q && gram_equals_query(c, j, e, hj.old_len);
        wave_push(s, n_match, hit, make_match(c, j, e, hj.old_len, hj.new_len), lane);
      }
    }
  }
  if (ticket_used) insert_claim(ticket, gram, c.bucket_mask, lane);
  wi.n_fresh = n_match;
  wi.win_cap = kWinWords / (2 * L);
  if (c.q > 0) lookup_with_windows<LCAP>(s, c, L, wi.win_cap, wi.n_fresh, n_match, gh, word);
  if (lane == 0) s.n_match = n_match;
  return n_match;
}

template <int LCAP>
__global__ __launch_bounds__(kWave) void step_wave_kernel(IndexView ix, StepIn in, DraftArgs a) {
  __shared__ Lds s;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);
  const int32_t L = a.L;
  int32_t target = (a.targets && c.tid < L) ? a.targets[(int64_t)row * L + c.tid] : 0;
  WinInfo wi;
  InsertTicket ticket;
  bool ticket_used;
  int32_t M = wave_front_end<LCAP>(s, c, ix, p, a.k, L, wi, ticket, ticket_used);
  block_sync<kWave>();

  DraftOut o;
  if (M > 0) {
    bool streaming = M > kMatchCap;
    if (!streaming) {
      uint32_t mask = build_dag<kWave>(s, c, M, L, wi);
      streaming = s.overflow != 0;
      if (!streaming) walk_dag<kWave>(s, c, mask, L, a.alpha_q, a.score_mode, o);
    }
    if (streaming) walk_streaming<kWave, true>(s, c, M, L, a.alpha_q, a.score_mode, ix.status, o);
  }
  bool live = c.tid < o.n;
  if (c.tid < L) {
    a.draft_tokens[(int64_t)row * L + c.tid] = live ? o.tok : -1;
    if (a.token_scores) a.token_scores[(int64_t)row * L + c.tid] = live ? key_to_score(o.key) : 0.0f;
  }
  if (c.tid == 0) {
    a.draft_len[row] = o.n;
    if (a.path_scores) a.path_scores[row] = key_to_score(o.key_sum);
  }
  if (a.targets) {                      // "Draft acceptance": first lane whose token differs
    u64 differs = __ballot(!(live && target == o.tok));
    if (c.tid == 0) a.accept_len[row] = differs ? (int32_t)__ffsll((long long)differs) - 1 : kWave;
  }
  if (ticket_used)
    insert_finish(ticket, const_cast<int32_t*>(c.gram), c.bucket_mask,
                  c.i * ix.max_len + (c.len_i - 1), c.tid);
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

// Plain copy of n 16-byte words: the known-size kernel that hardware traffic
// counters are calibrated against.
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src,
                                                   uint4* __restrict__ dst, int64_t n) {
  int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x; x < n; x += stride) dst[x] = src[x];
}

// ---- debug dumps ------------------------------------------------------------

template <int BLOCK, bool INDEXED>
__global__ __launch_bounds__(BLOCK) void dump_match_bits_kernel(IndexView ix, StepIn in, int32_t k,
                                                                uint32_t* bits, int32_t words) {
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);   // in.n == 0: nothing is being appended
  int32_t old_i = c.y.old_len(c.i);
  c.len_i = old_i;
  load_query(c, k, old_i);
  if (c.q <= 0) return;
  BitmapSink sink{bits + (int64_t)row * words};
  find_matches<BLOCK, INDEXED>(c, sink);
}

// Index mode: the matches as the step kernel's own front end finds them.
__global__ __launch_bounds__(kWave) void dump_match_bits_wave_kernel(IndexView ix, StepIn in,
                                                                     int32_t k, uint32_t* bits,
                                                                     int32_t words) {
  __shared__ Lds s;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);   // in.n == 0: nothing is being appended
  WinInfo wi;
  InsertTicket ticket;
  bool ticket_used;
  int32_t M = wave_front_end<8>(s, c, ix, p, k, 1, wi, ticket, ticket_used);
  block_sync<kWave>();
  BitmapSink sink{bits + (int64_t)row * words};
  if (M <= kMatchCap) {
    for (int32_t m = c.tid; m < M; m += kWave) sink.push(true, s.match[m]);
  } else if (c.q > 0) {
    match_index(c, sink);
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

// Builds the tier-1 DAG tables of a row exactly as draft_kernel does and writes
// the edge entries, sorted by key, to tmp rows of kTableCap entries.
// counts[row] = number of edges, or -1 if the row needs the streaming tier.
// Writes the edge entries of a finished tier-1 table, sorted by key, to the row's tmp slots.
template <int BLOCK>
__device__ __forceinline__ void emit_sorted_edges(Lds& s, uint32_t mask, int tid, int* n_edges,
                                                  u64* ok, u64* ov) {
  for (uint32_t h = tid; h <= mask; h += BLOCK) {
    u64 key = s.table[h].key;
    if (key == kEmpty || ((key >> 29) & kTokMask) == kAnyTok) continue;
    int rank = 0;                                     // keys are distinct: rank = sorted position
    for (uint32_t g = 0; g <= mask; ++g) {
      u64 other = s.table[g].key;
      if (other != kEmpty && ((other >> 29) & kTokMask) != kAnyTok && other < key) ++rank;
    }
    ok[rank] = key;
    ov[rank] = s.table[h].val;
    atomicAdd(n_edges, 1);
  }
}

// Builds the tier-1 DAG tables of a row exactly as the step kernels do and writes
// the edge entries, sorted by key, to tmp rows of kTableCap entries.
// counts[row] = number of edges, or -1 if the row needs the streaming tier.
template <int BLOCK, bool INDEXED>
__global__ __launch_bounds__(BLOCK) void dump_edge_rows_kernel(IndexView ix, StepIn in, int32_t k,
                                                               int32_t L, u64* tmp_keys,
                                                               u64* tmp_vals, int32_t* counts) {
  __shared__ Lds s;
  __shared__ int n_edges;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);   // in.n == 0: nothing is being appended
  int32_t old_i = c.y.old_len(c.i);
  c.len_i = old_i;
  load_query(c, k, old_i);
  if (c.tid == 0) { s.n_match = 0; n_edges = 0; }
  block_sync<BLOCK>();
  if (c.q <= 0) { if (c.tid == 0) counts[row] = 0; return; }
  ListSink sink{&s};
  find_matches<BLOCK, INDEXED>(c, sink);
  block_sync<BLOCK>();
  int32_t M = s.n_match;
  if (M == 0) { if (c.tid == 0) counts[row] = 0; return; }
  if (M > kMatchCap) { if (c.tid == 0) counts[row] = -1; return; }
  uint32_t mask = build_dag<BLOCK>(s, c, M, L, WinInfo{M, 0});
  if (s.overflow) { if (c.tid == 0) counts[row] = -1; return; }
  emit_sorted_edges<BLOCK>(s, mask, c.tid, &n_edges, tmp_keys + (int64_t)row * kTableCap,
                           tmp_vals + (int64_t)row * kTableCap);
  block_sync<BLOCK>();
  if (c.tid == 0) counts[row] = n_edges;
}

// Index mode: front end and DAG build of the step kernel itself.
template <int LCAP>
__global__ __launch_bounds__(kWave) void dump_edge_rows_wave_kernel(IndexView ix, StepIn in,
                                                                    int32_t k, int32_t L,
                                                                    u64* tmp_keys, u64* tmp_vals,
                                                                    int32_t* counts) {
  __shared__ Lds s;
  __shared__ int n_edges;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  int32_t p;
  Ctx c = make_ctx(ix, in, row, p);   // in.n == 0: nothing is being appended
  if (c.tid == 0) n_edges = 0;
  WinInfo wi;
  InsertTicket ticket;
  bool ticket_used;
  int32_t M = wave_front_end<LCAP>(s, c, ix, p, k, L, wi, ticket, ticket_used);
  block_sync<kWave>();
  if (M == 0) { if (c.tid == 0) counts[row] = 0; return; }
  if (M > kMatchCap) { if (c.tid == 0) counts[row] = -1; return; }
  uint32_t mask = build_dag<kWave>(s, c, M, L, wi);
  if (s.overflow) { if (c.tid == 0) counts[row] = -1; return; }
  emit_sorted_edges<kWave>(s, mask, c.tid, &n_edges, tmp_keys + (int64_t)row * kTableCap,
                           tmp_vals + (int64_t)row * kTableCap);
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
    u64 key = tmp_keys[(int64_t)row * kTableCap + x];
    u64 val = tmp_vals[(int64_t)row * kTableCap + x];
    out_duv[3 * at] = (int32_t)(key >> 58);
    out_duv[3 * at + 1] = (int32_t)((key >> 29) & kTokMask);
    out_duv[3 * at + 2] = (int32_t)(key & kTokMask);
    out_cs[2 * at] = cs_count(val);
    out_cs[2 * at + 1] = cs_sum(val);
  }
}

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
  size_t tok, pq, meta, status, gram, total;
  int32_t meta_stride;
  uint32_t n_buckets;           // per (problem, gram length); 0 in scan mode
  size_t gram_words;
};

bool uses_index(const csd_config* c) { return c->flags != CSD_MATCH_SCAN; }

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
  if (c->flags < 0 || c->flags > CSD_MATCH_INDEX) return CSD_ERR_UNIMPLEMENTED;
  return CSD_OK;
}

Layout make_layout(const csd_config* c) {
  Layout l;
  size_t cells = (size_t)c->n_problems * c->n_paths * c->max_len;
  size_t rows = (size_t)c->n_problems * c->n_paths;
  size_t at = 0;
  l.tok = at;    at += align_up(cells * sizeof(int32_t));
  l.pq = at;     at += align_up(cells * sizeof(uint32_t));
  l.meta_stride = (1 + c->max_query_len + 3) / 4 * 4;
  l.meta = at;   at += 2 * align_up(rows * l.meta_stride * sizeof(int32_t));
  l.status = at; at += align_up(4 * sizeof(uint32_t));
  l.n_buckets = 0;
  l.gram_words = 0;
  l.gram = at;
  if (uses_index(c)) {
    // 15 slots per bucket and at least positions/8 buckets: load factor <= 8/15
    uint64_t positions = (uint64_t)c->n_paths * c->max_len;
    uint32_t nb = 4;
    while ((uint64_t)nb * 8 < positions) nb <<= 1;
    l.n_buckets = nb;
    l.gram_words = (size_t)c->n_problems * c->max_query_len * nb * kBucketWords;
    at += align_up(l.gram_words * sizeof(int32_t));
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

struct csd_index {
  csd_config cfg;
  IndexView view;               // meta_old / meta_new are filled per launch
  int32_t* meta[2];             // double-buffered path ends (length + tail); `cur` is valid
  int cur;
  size_t gram_words;
  bool indexed;
  uint32_t alpha_q;
  int64_t len_lo, len_hi;       // host-side bounds on every path's length
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

void launch_draft(const csd_index* h, const IndexView& v, const StepIn& in, const DraftArgs& a,
                  hipStream_t st) {
  int64_t rows = (int64_t)v.P * v.N;
  if (!h->indexed)
    draft_kernel<kScanBlock, false><<<xcd_grid(rows), kScanBlock, 0, st>>>(v, in, a);
  else if (a.L <= 8)
    step_wave_kernel<8><<<xcd_grid(rows), kWave, 0, st>>>(v, in, a);
  else if (a.L <= 16)
    step_wave_kernel<16><<<xcd_grid(rows), kWave, 0, st>>>(v, in, a);
  else
    step_wave_kernel<32><<<xcd_grid(rows), kWave, 0, st>>>(v, in, a);
}

// Host-side bookkeeping shared by csd_append and csd_step.
int note_append(csd_index* h, bool has_counts, int32_t n) {
  if (!has_counts && h->len_lo + n > h->cfg.max_len) return CSD_ERR_CAPACITY;
  if (!has_counts) h->len_lo += n;
  h->len_hi += n;
  if (h->len_hi > h->cfg.max_len) h->len_hi = h->cfg.max_len;
  return CSD_OK;
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
  h->view.status = reinterpret_cast<uint32_t*>(base + l.status);
  h->indexed = uses_index(cfg);
  h->view.gram = h->indexed ? reinterpret_cast<int32_t*>(base + l.gram) : nullptr;
  h->view.bucket_mask = h->indexed ? l.n_buckets - 1 : 0;
  h->gram_words = l.gram_words;
  h->view.P = cfg->n_problems;
  h->view.N = cfg->n_paths;
  h->view.max_len = cfg->max_len;
  h->view.vocab = cfg->vocab;
  h->view.kmax = cfg->max_query_len;
  h->alpha_q = to_alpha_q(cfg->alpha);
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
                                                                 (int64_t)h->gram_words);
  CSD_HIP(hipGetLastError());
  h->len_lo = h->len_hi = 0;
  return CSD_OK;
}

int csd_append(csd_index* h, const int32_t* d_tokens, const float* d_probs,
               const int32_t* d_counts, int32_t n, void* stream) {
  if (!h || !d_tokens || n < 0) return CSD_ERR_INVALID_ARG;
  if (n == 0) return CSD_OK;
  int rc = note_append(h, d_counts != nullptr, n);
  if (rc != CSD_OK) return rc;
  int64_t rows = (int64_t)h->view.P * h->view.N;
  append_kernel<<<(uint32_t)rows, 256, 0, as_stream(stream)>>>(
      view_in_place(h), StepIn{d_tokens, d_probs, d_counts, n});
  CSD_HIP(hipGetLastError());
  return CSD_OK;
}

int csd_draft(csd_index* h, int32_t query_len, int32_t draft_len, int32_t* d_draft_tokens,
              int32_t* d_draft_len, float* d_token_scores, float* d_path_scores, void* stream) {
  if (!h || !d_draft_tokens || !d_draft_len) return CSD_ERR_INVALID_ARG;
  int rc = check_draft_args(h, query_len, draft_len);
  if (rc != CSD_OK) return rc;
  DraftArgs a{query_len, draft_len, h->alpha_q, h->cfg.score_mode, d_draft_tokens, d_draft_len,
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
  rc = note_append(h, d_counts != nullptr, n);
  if (rc != CSD_OK) return rc;
  IndexView v = h->view;
  v.meta_old = h->meta[h->cur];
  v.meta_new = h->meta[h->cur ^ 1];
  DraftArgs a{query_len, draft_len, h->alpha_q, h->cfg.score_mode, d_draft_tokens, d_draft_len,
              d_token_scores, d_path_scores, d_targets, d_accept_len};
  launch_draft(h, v, StepIn{d_tokens, d_probs, d_counts, n}, a, as_stream(stream));
  CSD_HIP(hipGetLastError());
  h->cur ^= 1;
  return CSD_OK;
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
    if (h->indexed)
      dump_match_bits_wave_kernel<<<xcd_grid(rows), kWave, 0, st>>>(v, no_step, query_len, bits,
                                                                    words);
    else
      dump_match_bits_kernel<kScanBlock, false><<<xcd_grid(rows), kScanBlock, 0, st>>>(
          v, no_step, query_len, bits, words);
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
  size_t tmp_elems = (size_t)rows * kTableCap;
  CSD_HIP(hipMalloc(&tmp, 2 * tmp_elems * sizeof(u64)));
  hipError_t e = hipMalloc(&counts, ((size_t)rows + 1) * sizeof(int32_t));
  if (e != hipSuccess) { (void)hipFree(tmp); return hip_fail(e, "hipMalloc"); }
  int32_t tail[2] = {0, 0};   // total rows, bad flag
  IndexView v = view_in_place(h);
  const StepIn no_step{nullptr, nullptr, nullptr, 0};
  do {
    if (h->indexed && draft_len <= 8)
      dump_edge_rows_wave_kernel<8><<<xcd_grid(rows), kWave, 0, st>>>(
          v, no_step, query_len, draft_len, tmp, tmp + tmp_elems, counts);
    else if (h->indexed && draft_len <= 16)
      dump_edge_rows_wave_kernel<16><<<xcd_grid(rows), kWave, 0, st>>>(
          v, no_step, query_len, draft_len, tmp, tmp + tmp_elems, counts);
    else if (h->indexed)
      dump_edge_rows_wave_kernel<32><<<xcd_grid(rows), kWave, 0, st>>>(
          v, no_step, query_len, draft_len, tmp, tmp + tmp_elems, counts);
    else
      dump_edge_rows_kernel<kScanBlock, false><<<xcd_grid(rows), kScanBlock, 0, st>>>(
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

const char* csd_strerror(int err) {
  switch (err) {
    case CSD_OK: return "ok";
    case CSD_ERR_INVALID_ARG: return "invalid argument";
    case CSD_ERR_CAPACITY: return "capacity exceeded";
    case CSD_ERR_WORKSPACE: return "workspace too small or misaligned";
    case CSD_ERR_HIP: return g_hip_msg;
    case CSD_ERR_UNIMPLEMENTED: return "reserved flag bits set";
    default: return "unknown csd error";
  }
}

}  // extern "C"
