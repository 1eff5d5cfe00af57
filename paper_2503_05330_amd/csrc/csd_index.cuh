// csd — the incrementally updated n-gram hash index (the "dynamic draft pool"
// of the Method section made searchable) and the append of a step's tokens.
//
// For every gram length g = 1..kmax one table of 64-byte buckets
// [count, 15 postings].  A posting (j, e) — "the g tokens before index e of
// path j" — is stored under the hash of those g tokens when token e is
// appended, so a query finds its matches (Eq. 3) without scanning histories.
// Bucket r of a gram's probe sequence is (h + r * step) mod n_buckets with an
// odd step; an insert goes into the first bucket of the sequence that is not
// full, so a lookup may stop at the first bucket that is not full.  Hash
// collisions are harmless: every posting is verified against the history
// before it counts.
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
__device__ __forceinline__ int32_t* gram_table(int32_t* gram, int g, uint32_t mask) {
  return gram + (int64_t)(g - 1) * ((int64_t)mask + 1) * kBucketWords;
}
__device__ __forceinline__ int32_t* gram_bucket(int32_t* tbl, GramHash gh, uint32_t r,
                                                uint32_t mask) {
  return tbl + (int64_t)((gh.h + r * gh.step) & mask) * kBucketWords;
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

// Inserts the postings of position e of path i for every gram length
// g = 1..kmax, by one whole wave (used for bulk appends).
__device__ __forceinline__ void gram_insert_position(int32_t* gram, uint32_t mask, int32_t kmax,
                                                     const Paths& y, int32_t i, int32_t e,
                                                     int32_t old_i, int lane) {
  uint32_t acc = kGramSeed;
  for (int32_t g = 1; g <= kmax && g <= e; ++g) {
    acc = gram_hash_add(acc, y.token(i, e - g, old_i));
    gram_insert_from(gram_table(gram, g, mask), mask, gram_hash_end(acc, g), 0u, y.pos(i, e), lane);
  }
}

// Split-phase insert of ONE new position into all kmax tables by one wave, so
// that its two memory round trips overlap the lookup's: lanes 8g-8 .. 8g-1 look
// at the first 8 buckets of gram length g's sequence.
struct InsertTicket {
  GramHash gh;                  // of this lane's gram length
  int32_t fill;                 // fill count of bucket (lane & 7) of that sequence
  int32_t first;                // first open bucket among the 8, or -1
  int32_t claimed;              // slot the leader lane got from the atomic, or kBucketSlots
  bool live;                    // this lane's gram length exists at this position
};

// Phase 1: hashes of the grams that end just before the new position (tail[a] =
// a-th token before it) and the fill-count loads.
__device__ __forceinline__ InsertTicket insert_begin(int32_t* gram, uint32_t mask, int32_t kmax,
                                                     const int32_t (&tail)[CSD_MAX_QUERY_LEN],
                                                     int32_t n_before, int lane) {
  InsertTicket t;
  const int g = (lane >> 3) + 1;
  t.gh = GramHash{0u, 1u};
  uint32_t acc = kGramSeed;
#pragma unroll
  for (int a = 1; a <= CSD_MAX_QUERY_LEN; ++a) {
    if (a <= kmax) {                                // uniform: longer grams are not indexed
      acc = gram_hash_add(acc, tail[a - 1]);
      if (a == g) t.gh = gram_hash_end(acc, a);
    }
  }
  t.live = g <= kmax && g <= n_before;
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
// that lost a race for the last slot) take the general insert.
__device__ __forceinline__ void insert_finish(const InsertTicket& t, int32_t* gram, uint32_t mask,
                                              int32_t pos, int lane) {
  bool leader = t.live && (lane & 7) == 0;
  bool placed = !leader;
  if (leader && t.claimed < kBucketSlots) {
    gram_bucket(gram_table(gram, (lane >> 3) + 1, mask), t.gh, (uint32_t)t.first,
                mask)[1 + t.claimed] = pos;
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
    gram_insert_from(gram_table(gram, (src >> 3) + 1, mask), mask, gh,
                     from < 0 ? 8u : (uint32_t)from, pos, lane);
  }
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
    int32_t* gram = ix.gram + (int64_t)p * ix.kmax * ((int64_t)ix.bucket_mask + 1) * kBucketWords;
    for (int32_t t = tid / kWave; t < cnt; t += BLOCK / kWave)     // one wave per new position
      gram_insert_position(gram, ix.bucket_mask, ix.kmax, y, i, old_i + t, old_i, tid & 63);
  }
  if (flags) atomicOr(ix.status, flags);
}

}  // namespace csd
