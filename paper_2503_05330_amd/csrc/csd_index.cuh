// csd — the incrementally updated n-gram hash index (the "dynamic draft pool"
// of the Method section made searchable) and the append of a step's tokens.
//
// One table of 64-byte buckets [count, 15 postings] per problem, for grams of
// length kmax (the configured maximum query length; shorter queries, which a
// decode loop only issues while a path is shorter than kmax, are matched by
// scan).  A posting (j, e) — "the kmax tokens before index e of path j" — is
// stored under the hash of those tokens when token e is appended, so a query
// finds its matches (Eq. 3) without scanning histories.  Bucket r of a gram's
// probe sequence is (h + r * step) mod n_buckets with an odd step; an insert
// goes into the first bucket of the sequence that is not full, so a lookup may
// stop at the first bucket that is not full.  Hash collisions are harmless:
// every posting is verified against the history before it counts.
#pragma once

#include "csd_common.cuh"

namespace csd {

struct GramHash {
  uint32_t h, step;
};
// The hash folds the gram's tokens newest first, so the hashes of all gram
// lengths that end at one position come from one pass over the tokens.
constexpr uint32_t kGramSeed = 0x243F6A88u;
__device__ __forceinline__ uint32_t gram_hash_add(uint32_t acc, int32_t token) {
  acc = (acc + (uint32_t)token) * 0x9E3779B1u;
  return acc ^ (acc >> 15);
}
__device__ __forceinline__ GramHash gram_hash_end(uint32_t acc, int g) {
  uint32_t x = acc ^ ((uint32_t)g * 0x85EBCA6Bu);
  uint32_t h = x * 0xC2B2AE35u;
  h ^= h >> 16;
  uint32_t step = ((x * 0x27D4EB2Fu) >> 7) | 1u;
  return GramHash{h, step};
}
__device__ __forceinline__ int32_t* gram_bucket(int32_t* tbl, GramHash gh, uint32_t r,
                                                uint32_t mask) {
  return tbl + (int64_t)((gh.h + r * gh.step) & mask) * kBucketWords;
}

// Forces a loaded value to be waited for here and not earlier: everything that
// uses it depends on this statement.  Lets independent loads issued before it
// share one memory round trip.
template <class T>
__device__ __forceinline__ void consume_here(T& v) {
  asm volatile("" : "+v"(v));
}

// General insert, by one whole wave: reads the fill counts of 64 buckets of
// the sequence per round trip, starting at bucket r0, and claims a slot in the
// first one that is not full.  Bounded by the table size; the tables hold more
// slots than there are positions.
__device__ __forceinline__ void gram_insert_from(int32_t* tbl, uint32_t mask, GramHash gh,
                                                 uint32_t r0, int32_t pos, int lane) {
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
        if (lane == 0) b[1 + c] = pos;
        return;
      }
      m &= m - 1;                                   // filled up meanwhile: next open bucket
    }
  }
}

// Inserts the posting of position e of path i (e >= kmax), by one whole wave
// (used for bulk appends).
__device__ __forceinline__ void gram_insert_position(int32_t* gram, uint32_t mask, int32_t kmax,
                                                     const Paths& y, int32_t i, int32_t e,
                                                     int32_t old_i, int lane) {
  if (e < kmax) return;
  uint32_t acc = kGramSeed;
  for (int32_t g = 1; g <= kmax; ++g) acc = gram_hash_add(acc, y.token(i, e - g, old_i));
  gram_insert_from(gram, mask, gram_hash_end(acc, kmax), 0u, y.pos(i, e), lane);
}

// Split-phase insert of ONE new position by one wave, so that its two memory
// round trips overlap the lookup's: lanes 0..15 look at the first 16 buckets of
// the gram's sequence.
constexpr int kInsertLanes = 16;
struct InsertTicket {
  GramHash gh;
  int32_t fill;                 // fill count of bucket `lane` of the sequence (lanes < 16)
  int32_t first;                // first open bucket among the 16, or -1
  int32_t claimed;              // lane 0: slot the atomic returned, or kBucketSlots
  bool live;                    // the position has kmax tokens before it
};

// Phase 1: hash of the gram that ends just before the new position (tail[a] =
// a-th token before it) and the fill-count loads (not waited for here).
__device__ __forceinline__ InsertTicket insert_begin(int32_t* gram, uint32_t mask, int32_t kmax,
                                                     const int32_t (&tail)[CSD_MAX_QUERY_LEN],
                                                     int32_t n_before, int lane) {
  InsertTicket t;
  uint32_t acc = kGramSeed;
#pragma unroll
  for (int a = 1; a <= CSD_MAX_QUERY_LEN; ++a)
    if (a <= kmax) acc = gram_hash_add(acc, tail[a - 1]);
  t.gh = gram_hash_end(acc, kmax);
  t.live = kmax <= n_before;
  t.first = -1;
  t.claimed = kBucketSlots;
  uint32_t r = (uint32_t)(lane & (kInsertLanes - 1));   // every lane loads: no branch, no early wait
  t.fill = gram_bucket(gram, t.gh, r <= mask ? r : 0u, mask)[0];
  return t;
}

// Phase 2: lane 0 claims a slot in the first open bucket.
__device__ __forceinline__ void insert_claim(InsertTicket& t, int32_t* gram, uint32_t mask,
                                             int lane) {
  consume_here(t.fill);
  bool open = t.live && lane < kInsertLanes && (uint32_t)lane <= mask && t.fill < kBucketSlots;
  u64 m = __ballot(open);
  t.first = m ? (int32_t)__ffsll((long long)m) - 1 : -1;
  if (t.live && lane == 0 && t.first >= 0)
    t.claimed = atomicAdd(gram_bucket(gram, t.gh, (uint32_t)t.first, mask), 1);
}

// Phase 3: store the posting; if the first 16 buckets were full (or the last
// slot was lost in a race) take the general insert.
__device__ __forceinline__ void insert_finish(const InsertTicket& t, int32_t* gram, uint32_t mask,
                                              int32_t pos, int lane) {
  if (!t.live) return;
  int32_t claimed = __builtin_amdgcn_readfirstlane(t.claimed);
  if (claimed < kBucketSlots) {
    if (lane == 0) gram_bucket(gram, t.gh, (uint32_t)t.first, mask)[1 + claimed] = pos;
    return;
  }
  gram_insert_from(gram, mask, t.gh, t.first < 0 ? (uint32_t)kInsertLanes : (uint32_t)t.first, pos,
                   lane);
}

// Stores this row's share of the step (tokens, quantised probabilities, index
// postings, new length and tail), reading the step input from memory.  Called
// by all threads of the row's workgroup; handles any number of new tokens.
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
    else if (a < new_i) meta_val = y.meta_old[(int64_t)i * y.meta_stride + 1 + a - cnt];
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
    int32_t* gram = ix.gram + (int64_t)p * ((int64_t)ix.bucket_mask + 1) * kBucketWords;
    for (int32_t t = tid / kWave; t < cnt; t += BLOCK / kWave)     // one wave per new position
      gram_insert_position(gram, ix.bucket_mask, ix.kmax, y, i, old_i + t, old_i, tid & 63);
  }
  if (flags) atomicOr(ix.status, flags);
}

}  // namespace csd
