// csd — shared device definitions: constants, exact fixed-point weights,
// wavefront reductions and the device-side view of the index state.
//
// Method: "Speculative Decoding for Multi-Sample Inference" — suffix match
// across paths (Eq. 3), layered token DAG with aggregated edge weights (Eq. 5),
// greedy layer-wise extraction (rule after Eq. 5, Algorithm 1).
#pragma once

#include <type_traits>

#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>

#include "csd.h"

namespace csd {

typedef unsigned long long u64;

constexpr int kWave = 64;
constexpr int kScanBlock = 1024;            // threads per row when matches come from a scan
constexpr int kDumpStride = 4096;           // debug dump: entries per row of its staging buffers
constexpr int kLenCache = 256;              // path lengths cached in LDS (more paths: read memory)
constexpr uint32_t kTokMask = (1u << 29) - 1;
constexpr uint32_t kAnyTok = kTokMask;      // "any predecessor": marks node (in-weight) entries
constexpr u64 kEmpty = ~0ull;
constexpr int kMaxClassBits = 20;           // streaming tier: at most 2^20 token classes
constexpr int kBucketWords = 16;            // one 64-byte line: [count, 15 postings]
constexpr int kBucketSlots = kBucketWords - 1;
constexpr int kTailCap = CSD_MAX_QUERY_LEN + 1;   // most tokens a meta row keeps

// ---------------------------------------------------------------- timing build
// With -DCSD_STAMPS (never in the shipped library) the first thread of a workgroup writes
// the constant-rate device clock (10 ns units) at marked places of the step kernels into a
// device array that a test harness reads back: where a step's time goes, row by row.
#ifdef CSD_STAMPS
constexpr int kStampSlots = 32;
__device__ unsigned long long g_stamps[(1 << 14) * kStampSlots];
#define CSD_STAMP(unit, n, value)                                                         \
  do {                                                                                    \
    if (threadIdx.x == 0 && (unit) < (1 << 14))                                           \
      csd::g_stamps[(unit) * csd::kStampSlots + (n)] = (value);                           \
  } while (0)
#define CSD_CLOCK() ((unsigned long long)wall_clock64())
#else
#define CSD_STAMP(unit, n, value) do { } while (0)
#define CSD_CLOCK() 0ull
#endif

// ---------------------------------------------------------------- exact weights

// DAG table key: layer d (6 bits) | predecessor u (29) | token v (29).
__device__ __forceinline__ u64 dag_key(int d, uint32_t u, uint32_t v) {
  return ((u64)d << 58) | ((u64)(u & kTokMask) << 29) | (u64)(v & kTokMask);
}
__device__ __forceinline__ uint32_t key_v(u64 key) { return (uint32_t)key & kTokMask; }
__device__ __forceinline__ uint32_t key_u(u64 key) { return (uint32_t)(key >> 29) & kTokMask; }
// Slot hash of a key: two 32-bit multiplies, high bits folded down.
__device__ __forceinline__ uint32_t dag_hash(u64 key) {
  uint32_t h = (uint32_t)key * 0x9E3779B1u ^ (uint32_t)(key >> 29) * 0x85EBCA6Bu;
  return h ^ (h >> 15);
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
// key / 2^32 as float, rounded once: the conversion of the integer rounds to nearest even, the
// scaling by a power of two is exact (the same value as through a double, in fewer and faster
// instructions).
__device__ __forceinline__ float key_to_score(u64 key) {
  return (float)key * (1.0f / 4294967296.0f);
}

// Probability -> multiple of 1/65536, round to nearest even, clamped, NaN -> 0.
__device__ __forceinline__ uint32_t quantize_prob(float p) {
  if (!(p == p)) return 0u;
  float x = rintf(p * 65536.0f);   // power-of-two scaling is exact; rintf is half-to-even
  x = fminf(fmaxf(x, 0.0f), 65536.0f);
  return (uint32_t)x;
}

// Lanes of the wave for which the condition holds.  Ballots of single compares combined with
// scalar ANDs are cheaper than one ballot of a compound condition, which the compiler turns
// into a select and a second compare.
__device__ __forceinline__ u64 wave_ballot(bool b) { return __builtin_amdgcn_ballot_w64(b); }

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
__device__ __forceinline__ Cand cand_from_lane(Cand c, int src) {
  Cand r;
  uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)c.key, src);
  uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(c.key >> 32), src);
  r.key = ((u64)hi << 32) | lo;
  r.v = __builtin_amdgcn_readlane(c.v, src);
  return r;
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

// Argmax over the 64 lanes of a wave; every lane gets the result.  Few lanes
// hold a candidate in practice: none or one is settled with a ballot and lane
// reads.  Otherwise four row_shr steps scan each row of 16 lanes, row_bcast:15
// and row_bcast:31 carry the row results up, and lane 63 ends with the total.
__device__ __forceinline__ Cand wave_argmax(Cand c) {
  u64 have = wave_ballot(c.v != INT_MAX);
  if (have == 0) return cand_none();
  if ((have & (have - 1)) == 0) return cand_from_lane(c, (int)__ffsll((long long)have) - 1);
  c = dpp_step<0x111, 0xF>(c);   // row_shr:1
  c = dpp_step<0x112, 0xF>(c);   // row_shr:2
  c = dpp_step<0x114, 0xF>(c);   // row_shr:4
  c = dpp_step<0x118, 0xF>(c);   // row_shr:8
  c = dpp_step<0x142, 0xA>(c);   // row_bcast:15 into rows 1 and 3
  c = dpp_step<0x143, 0xC>(c);   // row_bcast:31 into rows 2 and 3
  return cand_from_lane(c, 63);
}

// Requests all four 64-byte lines of a kernel's argument block at once and waits for them.
// Left to itself the compiler fetches the arguments where control flow first needs them, one
// line after the other, and every line is a miss in the scalar cache of a fresh launch: three
// memory round trips in a row before the first load of data can be issued.  After this call
// the compiler's own argument loads hit.  BYTES: size of the kernel's explicit arguments (only
// lines that hold some of them are touched; at most the first four).
template <size_t BYTES>
__device__ __forceinline__ void fetch_kernel_arguments() {
  static_assert(BYTES > 128, "meant for argument blocks of three lines or more");
  int32_t a, b, c, d;
  if (BYTES > 192)
    asm volatile(
        "s_load_dword %0, %4, 0x0\n\ts_load_dword %1, %4, 0x40\n\ts_load_dword %2, %4, 0x80\n\t"
        "s_load_dword %3, %4, 0xc0\n\ts_waitcnt lgkmcnt(0)"
        : "=&s"(a), "=&s"(b), "=&s"(c), "=&s"(d)
        : "s"(__builtin_amdgcn_kernarg_segment_ptr())
        : "memory");
  else
    asm volatile(
        "s_load_dword %0, %3, 0x0\n\ts_load_dword %1, %3, 0x40\n\ts_load_dword %2, %3, 0x80\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&s"(a), "=&s"(b), "=&s"(c)
        : "s"(__builtin_amdgcn_kernarg_segment_ptr())
        : "memory");
}

// x of lane (lane ^ R): within a quad of lanes one DPP move, else through the LDS crossbar.
template <int R>
__device__ __forceinline__ uint32_t from_xor_lane(int lane, uint32_t x) {
  static_assert(R >= 1 && R < kWave, "another lane of the wave");
  constexpr int kQuadPerm = R == 1 ? 0xB1 : R == 2 ? 0x4E : 0x1B;   // [1,0,3,2] [2,3,0,1] [3,2,1,0]
  if (R <= 3) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kQuadPerm, 0xF, 0xF, true);
  return (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ R) << 2, (int)x);
}
template <int R>
__device__ __forceinline__ u64 from_xor_lane64(int lane, u64 x) {
  return ((u64)from_xor_lane<R>(lane, (uint32_t)(x >> 32)) << 32) | from_xor_lane<R>(lane, (uint32_t)x);
}

// f(integral_constant<int, FIRST>) ... f(integral_constant<int, LAST - 1>)
template <int FIRST, int LAST, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (FIRST < LAST) {
    f(std::integral_constant<int, FIRST>{});
    static_for<FIRST + 1, LAST>(f);
  }
}

// x in the lanes of the mask, 0 in the others.  (The two idle cycles behind it: a DPP
// instruction may not read a register sooner after it was written, and the compiler does
// not look into an asm statement to see that this one writes it.)
__device__ __forceinline__ uint32_t lanes_of(u64 mask, uint32_t x) {
  uint32_t r;
  asm("v_cndmask_b32_e64 %0, 0, %1, %2\n\ts_nop 1" : "=v"(r) : "v"(x), "s"(mask));
  return r;
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_add(uint32_t x) {   // lanes the pattern does not reach add 0
  return x + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xF, false);
}

// Sum over the 64 lanes of a wave (the same lane moves as wave_argmax); every lane gets it.
__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
  x = dpp_add<0x111, 0xF>(x);    // row_shr:1
  x = dpp_add<0x112, 0xF>(x);    // row_shr:2
  x = dpp_add<0x114, 0xF>(x);    // row_shr:4
  x = dpp_add<0x118, 0xF>(x);    // row_shr:8
  x = dpp_add<0x142, 0xA>(x);    // row_bcast:15 into rows 1 and 3
  x = dpp_add<0x143, 0xC>(x);    // row_bcast:31 into rows 2 and 3
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_max(uint32_t x) {   // lanes the pattern does not reach see 0
  uint32_t y = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xF, false);
  return x > y ? x : y;
}
// Maximum over the 64 lanes of a wave (the lane moves of wave_sum); every lane gets it.
__device__ __forceinline__ uint32_t wave_max(uint32_t x) {
  x = dpp_max<0x111, 0xF>(x);
  x = dpp_max<0x112, 0xF>(x);
  x = dpp_max<0x114, 0xF>(x);
  x = dpp_max<0x118, 0xF>(x);
  x = dpp_max<0x142, 0xA>(x);
  x = dpp_max<0x143, 0xC>(x);
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

// arr[idx] for idx < N without indexing registers by a variable (0 when idx is out of range)
template <int N, int SIZE>
__device__ __forceinline__ int32_t pick_n(const int32_t (&arr)[SIZE], int32_t idx) {
  static_assert(N <= SIZE, "pick_n reads arr[0 .. N)");
  int32_t r = 0;
#pragma unroll
  for (int a = 0; a < N; ++a) r = (idx == a) ? arr[a] : r;
  return r;
}

// arr[idx] without indexing registers by a variable (0 when idx is out of range)
template <int SIZE>
__device__ __forceinline__ int32_t pick(const int32_t (&arr)[SIZE], int32_t idx) {
  int32_t r = 0;
#pragma unroll
  for (int a = 0; a < SIZE; ++a) r = (idx == a) ? arr[a] : r;
  return r;
}

// Forces a loaded value to be waited for here and not earlier: everything that
// uses it depends on this statement.  Lets independent loads issued before it
// share one memory round trip.
template <class T>
__device__ __forceinline__ void consume_here(T& v) {
  asm volatile("" : "+v"(v));
}

// BLOCK == kWave: code run by one wave on its own (a wave's LDS accesses execute in order),
// possibly beside other waves of the workgroup that do something else: no hardware barrier.
template <int BLOCK>
__device__ __forceinline__ void block_sync() {
  if (BLOCK == kWave) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  else __syncthreads();
}

// ---------------------------------------------------------------- device state

struct IndexView {              // device state inside the caller's workspace
  int32_t* tok;                 // [P][N][max_len] token histories
  uint32_t* pq;                 // [P][N][max_len] quantised generation probabilities
  const int32_t* meta_old;      // [P][N][meta_stride] before this launch: {length, last tail_len
                                //   tokens newest first}: one aligned load tells a path's end
  int32_t* meta_new;            // same rows after it (may alias meta_old when nothing else reads)
  uint32_t* status;             // sticky CSD_STATUS_* bits
  int32_t* gram;                // kmax-gram index [P][n_buckets][16], or null (scan mode)
  uint32_t bucket_mask;         // n_buckets - 1 (power of two)
  int32_t meta_stride;          // ints per meta row: 1 + tail_len rounded up to a multiple of 4
  int32_t tail_len;             // newest tokens kept in a meta row: kmax, or kmax + 1 when the
                                //   index serves one-edit matching (a match may look one further back)
  int32_t eshift;               // positions are packed as (path << eshift) | index
  int32_t P, N, max_len, vocab, kmax;
  int32_t eps;                  // edit tolerance (0 = exact match)
  int32_t options;              // bit 0: a path's own history is searched too; bit 1: a query
                                //   without matches is shortened by its oldest token until it has some
};

struct Match;

// A row's scan shared by several workgroups ("slices"), all on one XCD: every
// slice adds the matches it finds to the row's list in memory; the slice that
// finishes last (the row's state word tells it; nobody waits) goes on with the
// whole list.  n == 1: one workgroup per row, nothing of this is used.
struct ScanSlices {
  int32_t n;                    // slices per row (power of two)
  Match* matches;               // [rows][LdsScan::kMatch]
  u64* state;                   // [rows] low half: matches listed so far in this launch (the last
                                //   slice zeroes it again); high half: slices finished, over all launches
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
  int32_t n, N, max_len, meta_stride, eshift;

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
  __device__ __forceinline__ int32_t cell(int32_t j, int32_t t) const {   // j, t < 2^24
    return (int32_t)__umul24((uint32_t)j, (uint32_t)max_len) + t;
  }
  // Both readers select the address first and then issue ONE load outside any branch, so
  // that the loads of an unrolled loop all travel together instead of one per branch.
  __device__ __forceinline__ int32_t token(int32_t j, int32_t t, int32_t old_j) const {
    bool hist = t < old_j;
    const int32_t* base = hist ? tok : st;
    int64_t off = hist ? (int64_t)cell(j, t) : (int64_t)j * n + (t - old_j);
    return base[off];
  }
  // A probability as loaded, and what it takes to make the quantised value of it: the load
  // can be issued long before the value is needed (prob_value waits for it, prob_load does not).
  struct ProbWord {
    uint32_t word;
    bool hist, given;
  };
  __device__ __forceinline__ ProbWord prob_load(int32_t j, int32_t t, int32_t old_j) const {
    bool hist = t < old_j;
    bool given = !hist && sp != nullptr;
    const uint32_t* base = given ? reinterpret_cast<const uint32_t*>(sp) : pq;
    int64_t off = hist ? (int64_t)cell(j, t) : (given ? (int64_t)j * n + (t - old_j) : 0);
    return ProbWord{base[off], hist, given};
  }
  static __device__ __forceinline__ uint32_t prob_value(ProbWord w) {
    if (w.hist) return w.word;
    return w.given ? quantize_prob(__uint_as_float(w.word)) : 65536u;
  }
  __device__ __forceinline__ uint32_t prob(int32_t j, int32_t t, int32_t old_j) const {
    return prob_value(prob_load(j, t, old_j));
  }
  __device__ __forceinline__ int32_t pos(int32_t j, int32_t e) const { return (j << eshift) | e; }
  __device__ __forceinline__ int32_t pos_path(int32_t pos) const { return pos >> eshift; }
  __device__ __forceinline__ int32_t pos_index(int32_t pos) const {
    return pos & ((1 << eshift) - 1);
  }
};

struct Match {                  // one element of the candidate pool (Eq. 3)
  int32_t pos;                  // packed (j, e): e = index of the first continuation token
  int16_t rem_new;              // new_len_j - e: continuation tokens that exist, clipped to 63
  int16_t rel_old;              // old_len_j - e, clipped to [-32767, 63]; <= 0: e itself is new
};

struct Slot {
  u64 key;
  u64 val;
};

// On-chip state of one row.  TABLE = hash slots for DAG edges + nodes (power of
// two), MATCH = matches kept (beyond: streaming tier), WIN = words for cached
// continuations of matches, WAVES = waves of the workgroup, LENS = paths whose lengths
// are cached (more paths: their lengths are read from memory).
template <int TABLE, int MATCH, int WIN, int WAVES, int LENS = kLenCache>
struct LdsT {
  static constexpr int kTable = TABLE;
  static constexpr int kMatch = MATCH;
  static constexpr int kWin = WIN;
  static constexpr int kLens = LENS;
  Slot table[TABLE];
  uint16_t link[TABLE > MATCH ? TABLE : MATCH];   // edge slot -> slot of its target node (tier 1);
                                // the tree pool keeps one flag per listed match here
  Match match[MATCH];
  int32_t win[WIN];             // per cached match: L continuation tokens, then their L probabilities
  int32_t len_old[LENS];
  int32_t len_new[LENS];
  Cand red[2][WAVES];
  int32_t chosen[CSD_MAX_DRAFT_LEN];   // the draft so far (tree pool)
  int n_match;                  // total matches found (may exceed MATCH)
  int overflow;                 // a DAG table region ran out of room
};
// One wave per row (index mode): 38 KB, four rows share a CU's LDS.
typedef LdsT<1024, 1024, 2048, 1> LdsWave;
// The same for large batches, where the number of rows resident on a CU bounds
// the throughput: 9 KB, sixteen rows per CU (with the kernel built for eight waves
// per SIMD).  Rows with more than 256 matches or more than 32 distinct keys in a
// layer take the streaming tier.
typedef LdsT<256, 256, 512, 1, 64> LdsWaveSmall;
// One wave per row with one-edit matching through the index: such queries have
// many more matches, so the list is longer (66 KB, two rows per CU).
typedef LdsT<1024, 4096, 2048, 1> LdsWaveFuzzy;
// One wave per row, all rows of a problem (at most 16) in one workgroup that runs many
// steps per launch (the device-side loops): 10 KB per row, 160 KB per workgroup.  Rows with
// more than 64 matches (at a draft length of 8) take the bounded-memory tiers.
typedef LdsT<256, 128, 1024, 1, 16> LdsMulti;
// One 1024-thread workgroup per row (scan mode, where a fuzzy query can have
// thousands of matches): 128 KB, one row per CU (the windows are not used as such: the walk
// that tabulates node weights first keeps its keys and slots there).
typedef LdsT<4096, 4096, 6144, kScanBlock / kWave> LdsScan;

struct Ctx {                    // one (problem, query path)
  Paths y;
  const int32_t* gram;          // this problem's index tables, or null
  uint32_t bucket_mask;
  int32_t kmax;
  int32_t i;                    // query path
  int32_t skip;                 // the path that is not searched: i, or -1 (own history included)
  int32_t len_i;                // its length after the append
  int32_t eps;                  // edit tolerance of the match (Eq. 4): 0 or 1
  int32_t q;                    // effective query length min(k, len_i)
  int32_t Q[CSD_MAX_QUERY_LEN]; // Q[a] = a-th token from the end of path i
  int tid;
#ifdef CSD_STAMPS
  int32_t unit = 0;             // timing build: where this workgroup's stamps go
#endif
};

struct DraftArgs {
  int32_t k, L;
  uint32_t alpha_q;
  int32_t score_mode;
  int32_t pool_mode;            // CSD_POOL_*
  int32_t* draft_tokens;        // [P][N][L]
  int32_t* draft_len;           // [P][N]
  float* token_scores;          // [P][N][L] or null
  float* path_scores;           // [P][N] or null
  const int32_t* targets;       // [P][N][L] or null
  int32_t* accept_len;          // [P][N] or null
};

struct DraftOut {               // what one thread contributes to the outputs
  int32_t tok = -1;             // thread t keeps layer t+1
  u64 key = 0;
  u64 key_sum = 0;
  int32_t n = 0;
};

__device__ __forceinline__ Match make_match(const Paths& y, int32_t j, int32_t e, int32_t old_j,
                                            int32_t new_j) {
  int32_t rn = new_j - e, ro = old_j - e;
  Match m;
  m.pos = y.pos(j, e);
  m.rem_new = (int16_t)(rn > 63 ? 63 : rn);
  m.rel_old = (int16_t)(ro < -32767 ? -32767 : (ro > 63 ? 63 : ro));
  return m;
}

// The (u, v, p) instance that match m contributes to layer d, if it reaches it,
// read from memory.
// The predecessor of a layer-1 token is `root` (the last query token): the
// DAG hangs under the query, whatever token precedes a fuzzy match.
__device__ __forceinline__ bool layer_instance(const Paths& y, Match m, int32_t d, uint32_t root,
                                               uint32_t& u, uint32_t& v, u64& w) {
  if (d > (int32_t)m.rem_new) return false;        // the candidate has ended
  int32_t j = y.pos_path(m.pos);
  int32_t e = y.pos_index(m.pos);
  // rel_old is exact unless clipped at 63 (a step appends at most 32767 tokens), and
  // d <= 32 < 63: every index read below is then on the history side either way
  int32_t old_j = e + (int32_t)m.rel_old;
  uint32_t before = (uint32_t)y.token(j, e + (d >= 2 ? d - 2 : 0), old_j);   // no branch around the load
  u = d == 1 ? root : before;
  v = (uint32_t)y.token(j, e + d - 1, old_j);
  w = pack_cs(1u, y.prob(j, e + d - 1, old_j));
  return true;
}

// Workgroups are dealt round-robin to the 8 XCDs (workgroup b runs on XCD b mod 8), and
// each XCD has its own L2, cold at every launch.  Rows (problem, path) are therefore laid
// out so that (a) each XCD works on a contiguous range of rows: the paths of one problem
// share one L2; (b) no more XCDs are used than it takes to give every row a CU of its own
// (32 CUs per XCD): with few rows, one L2 fetches the kernel's code and the shared data
// once instead of eight times.  Workgroups dealt to the unused XCDs exit at once.
__host__ __device__ __forceinline__ int32_t xcds_used(int64_t rows) {
  int64_t x = (rows + 31) / 32;
  return (int32_t)(x < 1 ? 1 : (x > 8 ? 8 : x));
}
__device__ __forceinline__ int32_t xcd_row(int32_t rows) {
  int32_t xcd = (int32_t)(blockIdx.x & 7);
  if (xcd >= xcds_used(rows)) return -1;
  int32_t per_xcd = (int32_t)(gridDim.x >> 3);
  int32_t r = xcd * per_xcd + (int32_t)(blockIdx.x >> 3);
  return r < rows ? r : -1;
}
inline uint32_t xcd_grid(int64_t rows) {
  int64_t x = xcds_used(rows);
  return (uint32_t)((rows + x - 1) / x * 8);
}

__device__ __forceinline__ Ctx make_ctx(const IndexView& ix, const StepIn& in, int32_t row,
                                        int32_t& p_out) {
  Ctx c;
  int32_t p = row / ix.N;
  p_out = p;
  int64_t cells = (int64_t)p * ix.N * ix.max_len;
  c.i = row - p * ix.N;
  c.skip = (ix.options & 1) ? -1 : c.i;
  c.y.tok = ix.tok + cells;
  c.y.pq = ix.pq + cells;
  c.y.meta_old = ix.meta_old + (int64_t)p * ix.N * ix.meta_stride;
  c.y.meta_stride = ix.meta_stride;
  c.y.eshift = ix.eshift;
  c.y.n = in.n;
  c.y.st = in.n ? in.tok + (int64_t)p * ix.N * in.n : nullptr;
  c.y.sp = (in.n && in.prob) ? in.prob + (int64_t)p * ix.N * in.n : nullptr;
  c.y.sc = (in.n && in.counts) ? in.counts + (int64_t)p * ix.N : nullptr;
  c.y.N = ix.N;
  c.y.max_len = ix.max_len;
  c.gram = ix.gram ? ix.gram + (int64_t)p * ((int64_t)ix.bucket_mask + 1) * kBucketWords : nullptr;
  c.bucket_mask = ix.bucket_mask;
  c.kmax = ix.kmax;
  c.eps = ix.eps;
  c.len_i = 0;
  c.q = 0;
  c.tid = threadIdx.x;
  return c;
}

}  // namespace csd
