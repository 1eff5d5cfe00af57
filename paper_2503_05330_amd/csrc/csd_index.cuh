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

// General insert, by one whole wave: reads the fill counts of 64 buckets of
// the sequence per round trip, starting at bucket r0, and claims a slot in the
// first one that is not full.  Bounded by the table size; the tables hold more
// slots than there are positions.
__device__ __forceinline__ void gram_insert_from(int32_t* tbl, uint32_t mask, GramHash gh,
                                                 uint32_t r0, int32_t pos, int lane) {
  for (; r0 <= mask; r0 += kWave) {
    uint32_t r = r0 + lane;
    bool open = r <= mask && gram_bucket(tbl, gh, r, mask)[0] < kBucketSlots;
    u64 m = wave_ballot(open);
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

// Inserts the postings of the cnt <= 64 positions first .. first + cnt - 1 of path i by one
// wave, a lane per position: every lane hashes its gram, reads the fill count of its first
// bucket and claims a slot there — three round trips for all of them together.  A lane whose
// first buckets are full (rare) leaves its posting to the whole wave.
__device__ __forceinline__ void gram_insert_lanes(int32_t* gram, uint32_t mask, int32_t kmax,
                                                  const Paths& y, int32_t i, int32_t old_i,
                                                  int32_t first, int32_t cnt, int lane) {
  const int32_t e = first + lane;
  const bool mine = lane < cnt && e >= kmax;
  uint32_t acc = kGramSeed;
  for (int32_t g = 1; g <= kmax; ++g)                  // (idle lanes read the path's first token)
    acc = gram_hash_add(acc, y.token(i, mine ? e - g : 0, old_i));
  const GramHash gh = gram_hash_end(acc, kmax);
  const int32_t pos = y.pos(i, e);
  bool todo = mine;
  for (uint32_t r = 0; r < 4u && r <= mask; ++r) {
    if (wave_ballot(todo) == 0) return;
    int32_t* b = gram_bucket(gram, gh, r, mask);
    if (todo && b[0] < kBucketSlots) {
      const int32_t c = atomicAdd(b, 1);
      if (c < kBucketSlots) {
        b[1 + c] = pos;
        todo = false;
      }
    }
  }
  u64 left = wave_ballot(todo);
  while (left) {                                       // their first four buckets were full
    const int t = (int)__ffsll((long long)left) - 1;
    left &= left - 1;
    const GramHash g{(uint32_t)__builtin_amdgcn_readlane((int)gh.h, t),
                     (uint32_t)__builtin_amdgcn_readlane((int)gh.step, t)};
    gram_insert_from(gram, mask, g, 4u, __builtin_amdgcn_readlane(pos, t), lane);
  }
}

// Split-phase insert of ONE new position by one wave, so that its two memory
// round trips overlap the lookup's: lanes 0..3 look at the first four buckets of
// the gram's sequence (sixteen were no faster and fetched twelve more lines per row).
// (With thousands of rows per launch the step is bound by what all rows together issue and
// fetch, not by one row's latency: there only the first bucket is looked at up front, LANES = 1.)
constexpr int kInsertLanes = 4;     // buckets of the chain whose fill counts are read up front
struct InsertTicket {
  GramHash gh;
  int32_t fill;                 // fill count of bucket `lane` of the sequence (lanes < LANES)
  int32_t lanes;                // LANES: buckets looked at up front
  int32_t first;                // first open bucket among those looked at, or -1
  int32_t claimed;              // lane 0: slot the atomic returned, or kBucketSlots
  bool live;                    // the position has kmax tokens before it
};

// Phase 1: hash of the gram that ends just before the new position (tail[a] =
// a-th token before it) and the fill-count loads (not waited for here).
template <int QC, int LANES = kInsertLanes>
__device__ __forceinline__ InsertTicket insert_begin(int32_t* gram, uint32_t mask, int32_t kmax,
                                                     const int32_t (&tail)[kTailCap],
                                                     int32_t n_before, int lane) {
  static_assert(LANES >= 1 && (LANES & (LANES - 1)) == 0, "a power of two of buckets");
  InsertTicket t;
  t.lanes = LANES;
  uint32_t acc = kGramSeed;
#pragma unroll
  for (int a = 1; a <= QC; ++a)
    if (a <= kmax) acc = gram_hash_add(acc, tail[a - 1]);
  t.gh = gram_hash_end(acc, kmax);
  t.live = kmax <= n_before;
  t.first = -1;
  t.claimed = kBucketSlots;
  uint32_t r = (uint32_t)(lane & (LANES - 1));          // every lane loads: no branch, no early wait
  t.fill = gram_bucket(gram, t.gh, r <= mask ? r : 0u, mask)[0];
  return t;
}

// Phase 2: lane 0 claims a slot in the first open bucket.
__device__ __forceinline__ void insert_claim(InsertTicket& t, int32_t* gram, uint32_t mask,
                                             int lane) {
  consume_here(t.fill);
  bool open = t.live && lane < t.lanes && (uint32_t)lane <= mask && t.fill < kBucketSlots;
  u64 m = wave_ballot(open);
  t.first = m ? (int32_t)__ffsll((long long)m) - 1 : -1;
  if (t.live && lane == 0 && t.first >= 0)
    t.claimed = atomicAdd(gram_bucket(gram, t.gh, (uint32_t)t.first, mask), 1);
}

// Phase 3: store the posting; if the buckets looked at were full (or the last
// slot was lost in a race) take the general insert.
__device__ __forceinline__ void insert_finish(const InsertTicket& t, int32_t* gram, uint32_t mask,
                                              int32_t pos, int lane) {
  if (!t.live) return;
  int32_t claimed = __builtin_amdgcn_readfirstlane(t.claimed);
  if (claimed < kBucketSlots) {
    if (lane == 0) gram_bucket(gram, t.gh, (uint32_t)t.first, mask)[1 + claimed] = pos;
    return;
  }
  gram_insert_from(gram, mask, t.gh, t.first < 0 ? (uint32_t)t.lanes : (uint32_t)t.first, pos,
                   lane);
}

// ---------------------------------------------------------------- one-edit matching (Eq. 4) through the index
//
// Variant v of a gram G[0 .. kmax) (newest token first): v = 0 is the gram
// itself, v >= 1 the gram without G[v-1].  Two strings within one edit of each
// other share a variant (delete the substituted token from both; delete the
// extra token from the longer one), so a position whose kmax-gram is filed
// under all its kmax + 1 variants is found by looking up the query's variants.
// The converse does not hold, and a position can be found several times:
// candidates are verified and de-duplicated by the matcher.
// A posting of the variant index carries the number of the variant it was
// filed under above the packed position (which needs at most 25 bits): chains
// of different variants can share a bucket, and the matcher must tell them apart.
constexpr int kVariantShift = 26;
__device__ __forceinline__ int32_t variant_posting(int32_t pos, int32_t v) {
  return pos | (v << kVariantShift);
}

template <int SIZE>
__device__ __forceinline__ GramHash variant_hash(const int32_t (&G)[SIZE], int32_t kmax, int32_t v) {
  uint32_t acc = kGramSeed;
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a)
    if (a < kmax && a != v - 1) acc = gram_hash_add(acc, G[a]);
  return gram_hash_end(acc, v == 0 ? kmax : kmax - 1);
}
// Variant v >= 2 is the same string as variant v - 1 when the two dropped tokens are equal.
template <int SIZE>
__device__ __forceinline__ bool variant_is_new(const int32_t (&G)[SIZE], int32_t v) {
  return v < 2 || pick(G, v - 1) != pick(G, v - 2);
}

// Files position e of path i (e >= kmax) under every variant of the gram
// before it, by one whole wave (bulk appends).
__device__ __forceinline__ void gram_insert_variants(int32_t* gram, uint32_t mask, int32_t kmax,
                                                     const Paths& y, int32_t i, int32_t e,
                                                     int32_t old_i, int lane) {
  if (e < kmax) return;
  int32_t G[CSD_MAX_QUERY_LEN];
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a) G[a] = y.token(i, a < kmax ? e - 1 - a : e - 1, old_i);
  for (int32_t v = 0; v <= kmax; ++v)
    if (variant_is_new(G, v))
      gram_insert_from(gram, mask, variant_hash(G, kmax, v), 0u, variant_posting(y.pos(i, e), v), lane);
}

// Split-phase insert of ONE new position under its variants: the four groups
// of 16 lanes take variants 0..3 (fill counts of the first 16 buckets of each
// chain in one round trip, one slot claim per group); further variants
// (kmax >= 4) and groups whose quick claim failed use the general insert.
struct VariantTicket {
  GramHash gh;                  // of this lane's group's variant
  int32_t fill;                 // fill count of bucket (lane & 15) of that chain
  int32_t first;                // first open bucket among those looked at, or -1
  int32_t claimed;              // group leader: slot the atomic returned, or kBucketSlots
  bool live;                    // this group has a variant to file
  bool any;                     // the position has kmax tokens before it
};

__device__ __forceinline__ VariantTicket variants_begin(int32_t* gram, uint32_t mask, int32_t kmax,
                                                        const int32_t (&tail)[kTailCap],
                                                        int32_t n_before, int lane) {
  VariantTicket t;
  const int32_t v = lane >> 4;
  t.gh = variant_hash(tail, kmax, v);
  t.any = kmax <= n_before;
  t.live = t.any && v <= kmax && variant_is_new(tail, v);
  t.first = -1;
  t.claimed = kBucketSlots;
  uint32_t r = (uint32_t)(lane & 15);                   // every lane loads: no branch, no early wait
  t.fill = gram_bucket(gram, t.gh, r <= mask ? r : 0u, mask)[0];
  return t;
}

__device__ __forceinline__ void variants_claim(VariantTicket& t, int32_t* gram, uint32_t mask,
                                               int lane) {
  consume_here(t.fill);
  bool open = t.live && (uint32_t)(lane & 15) <= mask && t.fill < kBucketSlots;
  uint32_t mine = (uint32_t)(wave_ballot(open) >> (lane & 48)) & 0xFFFFu;   // this group's 16 lanes
  t.first = mine ? (int32_t)__ffs(mine) - 1 : -1;
  if (t.live && (lane & 15) == 0 && t.first >= 0)
    t.claimed = atomicAdd(gram_bucket(gram, t.gh, (uint32_t)t.first, mask), 1);
}

// Variants beyond the four the groups take (kmax >= 4): the general insert.
__device__ __forceinline__ void variants_beyond_four(const VariantTicket& t, int32_t* gram,
                                                     uint32_t mask, int32_t kmax,
                                                     const int32_t (&tail)[kTailCap], int32_t pos,
                                                     int lane) {
  if (!t.any) return;
  for (int32_t v = 4; v <= kmax; ++v)
    if (variant_is_new(tail, v))
      gram_insert_from(gram, mask, variant_hash(tail, kmax, v), 0u, variant_posting(pos, v), lane);
}

__device__ __forceinline__ void variants_finish(const VariantTicket& t, int32_t* gram, uint32_t mask,
                                                int32_t pos, int lane) {
  if (!t.any) return;
  bool stored = t.live && (lane & 15) == 0 && t.claimed < kBucketSlots;
  if (stored) gram_bucket(gram, t.gh, (uint32_t)t.first, mask)[1 + t.claimed] = variant_posting(pos, lane >> 4);
  int32_t retry = (t.live && !stored) ? 1 : 0;          // meaningful on the group leaders
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    if (__shfl(retry, 16 * g) == 0) continue;           // uniform over the wave
    GramHash gh{(uint32_t)__shfl((int)t.gh.h, 16 * g), (uint32_t)__shfl((int)t.gh.step, 16 * g)};
    int32_t first = __shfl(t.first, 16 * g);
    gram_insert_from(gram, mask, gh, first < 0 ? 16u : (uint32_t)first, variant_posting(pos, g), lane);
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
  else if (tid <= ix.tail_len) {
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
  if (tid <= ix.tail_len) ix.meta_new[row * ix.meta_stride + tid] = meta_val;
  for (int32_t t = tid; t < cnt; t += BLOCK) {
    int32_t v = y.st[(int64_t)i * y.n + t];
    if (v < 0 || v >= ix.vocab) flags |= CSD_STATUS_TOKEN_RANGE;
    ix.tok[row * ix.max_len + old_i + t] = v;
    ix.pq[row * ix.max_len + old_i + t] = y.sp ? quantize_prob(y.sp[(int64_t)i * y.n + t]) : 65536u;
  }
  if (WITH_INDEX && ix.gram) {
    int32_t* gram = ix.gram + (int64_t)p * ((int64_t)ix.bucket_mask + 1) * kBucketWords;
    if (ix.eps == 0) {                                  // a lane per new position, 64 per wave and round
      for (int32_t t0 = (tid / kWave) * kWave; t0 < cnt; t0 += BLOCK) {
        const int32_t left = cnt - t0;
        gram_insert_lanes(gram, ix.bucket_mask, ix.kmax, y, i, old_i, old_i + t0,
                          left < kWave ? left : kWave, tid & 63);
      }
    } else {
      for (int32_t t = tid / kWave; t < cnt; t += BLOCK / kWave)   // one wave per new position
        gram_insert_variants(gram, ix.bucket_mask, ix.kmax, y, i, old_i + t, old_i, tid & 63);
    }
  }
  if (flags) atomicOr(ix.status, flags);
}

}  // namespace csd
