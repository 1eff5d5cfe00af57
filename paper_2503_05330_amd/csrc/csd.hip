// csd — consensus speculative drafting for N parallel sampling paths on gfx950.
//
// Device kernels and the C-ABI entry points declared in csd.h.  The method is
// the one of "Speculative Decoding for Multi-Sample Inference": suffix match
// across paths (Eq. 3), layered token DAG with aggregated edge weights (Eq. 5),
// greedy layer-wise extraction (rule after Eq. 5, Algorithm 1), and the greedy
// acceptance check ("Draft acceptance").
//
// Nothing here is a dense contraction, so there is no MFMA: the work is
// integer compares, LDS hash-histogram atomics and wavefront reductions.
//
// Exactness: every weight is an integer (probabilities are quantised to
// 1/65536 at append), so LDS atomics may accumulate in any order and the
// result is still unique.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "csd.h"

namespace {

typedef unsigned long long u64;

constexpr int kBlock = 256;                 // threads per (problem, path) workgroup
constexpr int kWaves = kBlock / 64;         // wave64
constexpr int kMatchCap = 1024;             // matches kept in LDS; beyond -> streaming tier
constexpr int kTableCap = 2048;             // LDS hash slots for DAG edges + nodes
constexpr uint32_t kTokMask = (1u << 29) - 1;
constexpr uint32_t kAnyTok = kTokMask;      // "any predecessor": marks node (in-weight) entries
constexpr u64 kEmpty = ~0ull;
constexpr int kMaxClassBits = 20;           // streaming tier: at most 2^20 token classes

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
__device__ __forceinline__ Cand wave_argmax(Cand c) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Cand x;
    x.key = __shfl_xor(c.key, o);
    x.v = __shfl_xor(c.v, o);
    c = cand_best(c, x);
  }
  return c;
}

// ---------------------------------------------------------------- per-workgroup state

struct Lds {
  u64 keys[kTableCap];
  u64 vals[kTableCap];
  int32_t match[kMatchCap];   // matches as offsets j*max_len + e into the problem's history
  Cand red[2][kWaves];
  int n_match;                // total matches found (may exceed kMatchCap)
  int n_keys;                 // distinct keys in the table
  int overflow;               // table ran out of room
};

struct Ctx {                  // one (problem, query path)
  const int32_t* tok;         // [N][max_len] of this problem
  const uint32_t* pq;         // same shape, quantised probabilities
  const int32_t* len;         // [N]
  int32_t N, max_len;
  int32_t i;                  // query path
  int32_t q;                  // effective query length min(k, len_i)
  int32_t Q[CSD_MAX_QUERY_LEN];   // Q[a] = a-th token from the end of path i
  int tid;
};

__device__ __forceinline__ void load_query(Ctx& c, int32_t k) {
  int32_t len_i = c.len[c.i];
  c.q = k < len_i ? k : len_i;
  const int32_t* row = c.tok + (int64_t)c.i * c.max_len;
#pragma unroll
  for (int a = 0; a < CSD_MAX_QUERY_LEN; ++a) c.Q[a] = (a < c.q) ? row[len_i - 1 - a] : 0;
}

// Does the q-gram that ends just before index e of `row` equal the query?
__device__ __forceinline__ bool gram_equals_query(const Ctx& c, const int32_t* row, int32_t e) {
  bool hit = row[e - 1] == c.Q[0];
#pragma unroll
  for (int a = 1; a < CSD_MAX_QUERY_LEN; ++a)
    if (a < c.q && hit) hit = row[e - 1 - a] == c.Q[a];
  return hit;
}

// ---------------------------------------------------------------- match sinks

// Compacts hits into the LDS match list with one LDS atomic per wave.
// push() must be reached by all 64 lanes of a wave together.
struct ListSink {
  Lds* s;
  __device__ __forceinline__ void push(bool hit, int32_t off) {
    u64 mask = __ballot(hit);
    if (mask == 0) return;
    int lane = __lane_id();
    int base = 0;
    if (lane == 0) base = atomicAdd(&s->n_match, (int)__popcll(mask));
    base = __shfl(base, 0);
    int slot = base + (int)__popcll(mask & ((1ull << lane) - 1ull));
    if (hit && slot < kMatchCap) s->match[slot] = off;
  }
};

// Marks hits in a bitmap over all positions of the problem (debug dump).
struct BitmapSink {
  uint32_t* bits;
  __device__ __forceinline__ void push(bool hit, int32_t off) {
    if (hit) atomicOr(&bits[off >> 5], 1u << (off & 31));
  }
};

// Eq. 3 by exhaustive comparison: every position e of every other path j with
// q <= e <= len_j - 1 is tested.  Loop bounds are uniform over the workgroup.
template <class Sink>
__device__ __forceinline__ void match_scan(const Ctx& c, Sink& sink) {
  for (int32_t j = 0; j < c.N; ++j) {
    if (j == c.i) continue;
    int32_t len_j = c.len[j];
    const int32_t* row = c.tok + (int64_t)j * c.max_len;
    for (int32_t e0 = c.q; e0 < len_j; e0 += kBlock) {
      int32_t e = e0 + c.tid;
      bool hit = (e < len_j) && gram_equals_query(c, row, e);
      sink.push(hit, j * c.max_len + e);
    }
  }
}

// ---------------------------------------------------------------- LDS hash table

__device__ __forceinline__ void table_clear(Lds& s, uint32_t mask, int tid) {
  for (uint32_t h = tid; h <= mask; h += kBlock) {
    s.keys[h] = kEmpty;
    s.vals[h] = 0ull;
  }
  if (tid == 0) {
    s.n_keys = 0;
    s.overflow = 0;
  }
}

// vals[key] += delta, inserting the key if new.  Sets s.overflow when the
// table is more than 3/4 full (the caller then falls back) — never spins.
__device__ __forceinline__ void table_add(Lds& s, uint32_t mask, u64 key, u64 delta) {
  uint32_t h = mix_u64(key) & mask;
  for (uint32_t probe = 0; probe <= mask; ++probe) {
    u64 cur = s.keys[h];
    if (cur == kEmpty) {
      cur = atomicCAS(&s.keys[h], kEmpty, key);
      if (cur == kEmpty) {
        int n = atomicAdd(&s.n_keys, 1) + 1;
        if ((uint32_t)n > (mask + 1) - ((mask + 1) >> 2)) s.overflow = 1;
        cur = key;
      }
    }
    if (cur == key) {
      atomicAdd(&s.vals[h], delta);
      return;
    }
    h = (h + 1) & mask;
  }
  s.overflow = 1;
}

__device__ __forceinline__ u64 table_get(const Lds& s, uint32_t mask, u64 key) {
  uint32_t h = mix_u64(key) & mask;
  for (uint32_t probe = 0; probe <= mask; ++probe) {
    u64 cur = s.keys[h];
    if (cur == key) return s.vals[h];
    if (cur == kEmpty) return 0ull;
    h = (h + 1) & mask;
  }
  return 0ull;
}

// Workgroup-wide argmax of the per-thread candidates; every thread gets the result.
__device__ __forceinline__ Cand block_argmax(Lds& s, Cand c, int tid, int parity) {
  c = wave_argmax(c);
  if ((tid & 63) == 0) s.red[parity][tid >> 6] = c;
  __syncthreads();
  Cand r = s.red[parity][0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) r = cand_best(r, s.red[parity][w]);
  return r;
}

// Successors of `cur` in layer d as held by the table, best one per thread.
__device__ __forceinline__ Cand scan_successors(const Lds& s, uint32_t mask, int d, int32_t cur,
                                                uint32_t alpha_q, int score_mode, int tid,
                                                Cand best) {
  u64 want = dag_key(d, (uint32_t)cur, 0) >> 29;
  for (uint32_t h = tid; h <= mask; h += kBlock) {
    u64 key = s.keys[h];
    if ((key >> 29) != want) continue;
    uint32_t v = (uint32_t)(key & kTokMask);
    u64 w = score_mode ? s.vals[h] : table_get(s, mask, dag_key(d, kAnyTok, v));
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

// ---------------------------------------------------------------- tier 1: everything in LDS

// Eq. 5: every (match, layer) instance adds (1, p) to its edge (d,u,v) and to
// its node (d,*,v).  Returns the table mask used.
__device__ __forceinline__ uint32_t build_dag(Lds& s, const Ctx& c, int32_t M, int32_t L) {
  uint32_t want = 4u * (uint32_t)M * (uint32_t)L;     // <= 50 % load without any merging
  uint32_t size = 64;
  while (size < want && size < (uint32_t)kTableCap) size <<= 1;
  uint32_t mask = size - 1;
  table_clear(s, mask, c.tid);
  __syncthreads();
  int32_t items = M * L;
  for (int32_t idx = c.tid; idx < items; idx += kBlock) {
    int32_t d = idx / M + 1;
    int32_t off = s.match[idx - (d - 1) * M];
    int32_t j = off / c.max_len;
    int32_t t = off - j * c.max_len + d - 1;         // index of the layer-d token in path j
    if (t < c.len[j] && !s.overflow) {
      uint32_t u = (uint32_t)c.tok[off + d - 2];
      uint32_t v = (uint32_t)c.tok[off + d - 1];
      u64 w = pack_cs(1u, c.pq[off + d - 1]);
      table_add(s, mask, dag_key(d, u, v), w);
      table_add(s, mask, dag_key(d, kAnyTok, v), w);
    }
  }
  __syncthreads();
  return mask;
}

// Greedy walk over the finished tables (rule after Eq. 5).
__device__ __forceinline__ void walk_dag(Lds& s, const Ctx& c, uint32_t mask, int32_t L,
                                         uint32_t alpha_q, int score_mode, DraftOut& o) {
  int32_t cur = c.Q[0];
  for (int32_t d = 1; d <= L; ++d) {
    Cand best = scan_successors(s, mask, d, cur, alpha_q, score_mode, c.tid, cand_none());
    best = block_argmax(s, best, c.tid, d & 1);
    if (best.v == INT_MAX) break;                     // leaf: no edge leaves cur
    if (c.tid == d - 1) { o.tok = best.v; o.key = best.key; }
    o.key_sum += best.key;
    o.n = d;
    cur = best.v;
  }
}

// ---------------------------------------------------------------- tier 2: streaming, layer by layer

// Calls f(off, j, e) for every match.  Uses the LDS list when it holds all of
// them, else compares every position again.
template <class F>
__device__ __forceinline__ void for_each_match(const Lds& s, const Ctx& c, int32_t M, F f) {
  if (M <= kMatchCap) {
    for (int32_t m = c.tid; m < M; m += kBlock) {
      int32_t off = s.match[m];
      int32_t j = off / c.max_len;
      f(off, j, off - j * c.max_len);
    }
  } else {
    for (int32_t j = 0; j < c.N; ++j) {
      if (j == c.i) continue;
      int32_t len_j = c.len[j];
      const int32_t* row = c.tok + (int64_t)j * c.max_len;
      for (int32_t e = c.q + c.tid; e < len_j; e += kBlock)
        if (gram_equals_query(c, row, e)) f(j * c.max_len + e, j, e);
    }
  }
}

// Same result as build_dag + walk_dag with bounded memory for any input: one
// layer at a time, and within a layer one class of tokens (by hash residue)
// at a time, doubling the number of classes whenever a class overflows LDS.
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
        __syncthreads();                               // previous readers are done
        table_clear(s, mask, c.tid);
        __syncthreads();
        for_each_match(s, c, M, [&](int32_t off, int32_t j, int32_t e) {
          int32_t t = e + d - 1;
          if (t >= c.len[j] || s.overflow) return;
          uint32_t v = (uint32_t)c.tok[off + d - 1];
          if ((mix_u64(v) & (n_class - 1)) != r) return;
          uint32_t u = (uint32_t)c.tok[off + d - 2];
          u64 w = pack_cs(1u, c.pq[off + d - 1]);
          table_add(s, mask, dag_key(d, kAnyTok, v), w);
          if (u == (uint32_t)cur) table_add(s, mask, dag_key(d, u, v), w);
        });
        __syncthreads();
        if (s.overflow) failed = true;                 // uniform: read after the barrier
        else best = scan_successors(s, mask, d, cur, alpha_q, score_mode, c.tid, best);
      }
      if (failed) ++class_bits;
    } while (failed && class_bits <= kMaxClassBits);
    if (failed) {                                      // cannot happen for vocab < 2^29 in practice
      if (c.tid == 0) atomicOr(status, CSD_STATUS_TABLE_FULL);
      break;
    }
    parity ^= 1;
    best = block_argmax(s, best, c.tid, parity);
    if (best.v == INT_MAX) break;
    if (c.tid == d - 1) { o.tok = best.v; o.key = best.key; }
    o.key_sum += best.key;
    o.n = d;
    cur = best.v;
  }
}

// ---------------------------------------------------------------- kernels

struct IndexView {              // device state inside the caller's workspace
  int32_t* tok;                 // [P][N][max_len]
  uint32_t* pq;                 // [P][N][max_len]
  int32_t* len;                 // [P][N]
  uint32_t* status;             // sticky CSD_STATUS_* bits
  int32_t P, N, max_len, vocab;
};

// Workgroups are dealt round-robin to the 8 XCDs; this maps them back so that
// each XCD works on a contiguous range of (problem, path) rows and the paths of
// one problem share one L2.  The grid is padded to a multiple of 8.
__device__ __forceinline__ int32_t xcd_row(int32_t rows) {
  int32_t per_xcd = (int32_t)(gridDim.x >> 3);
  int32_t r = (int32_t)(blockIdx.x & 7) * per_xcd + (int32_t)(blockIdx.x >> 3);
  return r < rows ? r : -1;
}
inline uint32_t xcd_grid(int64_t rows) { return (uint32_t)((rows + 7) / 8 * 8); }

__device__ __forceinline__ Ctx make_ctx(const IndexView& ix, int32_t row) {
  Ctx c;
  int32_t p = row / ix.N;
  c.i = row - p * ix.N;
  c.tok = ix.tok + (int64_t)p * ix.N * ix.max_len;
  c.pq = ix.pq + (int64_t)p * ix.N * ix.max_len;
  c.len = ix.len + (int64_t)p * ix.N;
  c.N = ix.N;
  c.max_len = ix.max_len;
  c.tid = threadIdx.x;
  return c;
}

__global__ __launch_bounds__(kBlock) void reset_kernel(IndexView ix) {
  int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (t < (int64_t)ix.P * ix.N) ix.len[t] = 0;
  if (t == 0) *ix.status = 0u;
}

// One thread per path: stores the step's tokens and quantised probabilities
// behind the path's current end.
__global__ __launch_bounds__(kBlock) void append_kernel(IndexView ix, const int32_t* tokens,
                                                        const float* probs, const int32_t* counts,
                                                        int32_t n) {
  int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (r >= (int64_t)ix.P * ix.N) return;
  int32_t cnt = counts ? counts[r] : n;
  cnt = cnt < 0 ? 0 : (cnt > n ? n : cnt);
  int32_t len = ix.len[r];
  uint32_t flags = 0;
  if (len + cnt > ix.max_len) {
    cnt = ix.max_len - len;
    flags |= CSD_STATUS_CAPACITY;
  }
  int32_t* trow = ix.tok + r * ix.max_len;
  uint32_t* prow = ix.pq + r * ix.max_len;
  for (int32_t t = 0; t < cnt; ++t) {
    int32_t v = tokens[r * n + t];
    if (v < 0 || v >= ix.vocab) flags |= CSD_STATUS_TOKEN_RANGE;
    trow[len + t] = v;
    prow[len + t] = probs ? quantize_prob(probs[r * n + t]) : 65536u;
  }
  ix.len[r] = len + cnt;
  if (flags) atomicOr(ix.status, flags);
}

// One workgroup per (problem, path): match (Eq. 3) -> DAG (Eq. 5) -> greedy walk.
__global__ __launch_bounds__(kBlock) void draft_kernel(IndexView ix, int32_t k, int32_t L,
                                                       uint32_t alpha_q, int32_t score_mode,
                                                       int32_t* draft_tokens, int32_t* draft_len,
                                                       float* token_scores, float* path_scores) {
  __shared__ Lds s;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  Ctx c = make_ctx(ix, row);
  load_query(c, k);
  if (c.tid == 0) s.n_match = 0;
  __syncthreads();

  DraftOut o;
  if (c.q > 0) {
    ListSink sink{&s};
    match_scan(c, sink);
    __syncthreads();
    int32_t M = s.n_match;
    if (M > 0) {
      bool streaming = M > kMatchCap;
      if (!streaming) {
        uint32_t mask = build_dag(s, c, M, L);
        streaming = s.overflow != 0;
        if (!streaming) walk_dag(s, c, mask, L, alpha_q, score_mode, o);
      }
      if (streaming) walk_streaming(s, c, M, L, alpha_q, score_mode, ix.status, o);
    }
  }
  if (c.tid < L) {
    bool live = c.tid < o.n;
    draft_tokens[(int64_t)row * L + c.tid] = live ? o.tok : -1;
    if (token_scores) token_scores[(int64_t)row * L + c.tid] = live ? key_to_score(o.key) : 0.0f;
  }
  if (c.tid == 0) {
    draft_len[row] = o.n;
    if (path_scores) path_scores[row] = key_to_score(o.key_sum);
  }
}

__global__ __launch_bounds__(kBlock) void accept_kernel(int64_t rows, int32_t L,
                                                        const int32_t* draft_tokens,
                                                        const int32_t* draft_len,
                                                        const int32_t* targets,
                                                        int32_t* accept_len) {
  int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (r >= rows) return;
  int32_t n = draft_len[r];
  n = n < 0 ? 0 : (n > L ? L : n);
  int32_t a = 0;
  while (a < n && draft_tokens[r * L + a] == targets[r * L + a]) ++a;
  accept_len[r] = a;
}

// ---- debug dumps ------------------------------------------------------------

__global__ __launch_bounds__(kBlock) void dump_match_bits_kernel(IndexView ix, int32_t k,
                                                                 uint32_t* bits, int32_t words) {
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  Ctx c = make_ctx(ix, row);
  load_query(c, k);
  if (c.q <= 0) return;
  BitmapSink sink{bits + (int64_t)row * words};
  match_scan(c, sink);
}

// counts[row] = number of set bits of the row (one workgroup per row)
__global__ __launch_bounds__(kBlock) void count_bits_kernel(const uint32_t* bits, int32_t words,
                                                            int32_t* counts) {
  __shared__ int total;
  if (threadIdx.x == 0) total = 0;
  __syncthreads();
  const uint32_t* b = bits + (int64_t)blockIdx.x * words;
  int n = 0;
  for (int32_t w = threadIdx.x; w < words; w += kBlock) n += __popc(b[w]);
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
__global__ __launch_bounds__(kBlock) void dump_edge_rows_kernel(IndexView ix, int32_t k, int32_t L,
                                                                u64* tmp_keys, u64* tmp_vals,
                                                                int32_t* counts) {
  __shared__ Lds s;
  __shared__ int n_edges;
  int32_t row = xcd_row(ix.P * ix.N);
  if (row < 0) return;
  Ctx c = make_ctx(ix, row);
  load_query(c, k);
  if (c.tid == 0) { s.n_match = 0; n_edges = 0; }
  __syncthreads();
  if (c.q <= 0) { if (c.tid == 0) counts[row] = 0; return; }
  ListSink sink{&s};
  match_scan(c, sink);
  __syncthreads();
  int32_t M = s.n_match;
  if (M == 0) { if (c.tid == 0) counts[row] = 0; return; }
  if (M > kMatchCap) { if (c.tid == 0) counts[row] = -1; return; }
  uint32_t mask = build_dag(s, c, M, L);
  if (s.overflow) { if (c.tid == 0) counts[row] = -1; return; }
  u64* ok = tmp_keys + (int64_t)row * kTableCap;
  u64* ov = tmp_vals + (int64_t)row * kTableCap;
  for (uint32_t h = c.tid; h <= mask; h += kBlock) {
    u64 key = s.keys[h];
    if (key == kEmpty || ((key >> 29) & kTokMask) == kAnyTok) continue;
    int rank = 0;                                     // keys are distinct: rank = sorted position
    for (uint32_t g = 0; g <= mask; ++g) {
      u64 other = s.keys[g];
      if (other != kEmpty && ((other >> 29) & kTokMask) != kAnyTok && other < key) ++rank;
    }
    ok[rank] = key;
    ov[rank] = s.vals[h];
    atomicAdd(&n_edges, 1);
  }
  __syncthreads();
  if (c.tid == 0) counts[row] = n_edges;
}

__global__ __launch_bounds__(kBlock) void scatter_edges_kernel(const u64* tmp_keys,
                                                               const u64* tmp_vals,
                                                               const int32_t* off, int32_t* out_duv,
                                                               uint64_t* out_cs, int64_t cap) {
  int32_t row = blockIdx.x;
  int64_t base = off[row];
  int32_t n = off[row + 1] - off[row];
  for (int32_t x = threadIdx.x; x < n; x += kBlock) {
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
  size_t tok, pq, len, status, total;
};

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
  l.len = at;    at += align_up(rows * sizeof(int32_t));
  l.status = at; at += align_up(4 * sizeof(uint32_t));
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
  IndexView view;
  uint32_t alpha_q;
  int64_t len_lo, len_hi;       // host-side bounds on every path's length
};

namespace {
hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
uint32_t blocks_for(int64_t n) { return (uint32_t)((n + kBlock - 1) / kBlock); }
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
  h->view.tok = reinterpret_cast<int32_t*>(base + l.tok);
  h->view.pq = reinterpret_cast<uint32_t*>(base + l.pq);
  h->view.len = reinterpret_cast<int32_t*>(base + l.len);
  h->view.status = reinterpret_cast<uint32_t*>(base + l.status);
  h->view.P = cfg->n_problems;
  h->view.N = cfg->n_paths;
  h->view.max_len = cfg->max_len;
  h->view.vocab = cfg->vocab;
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
  int64_t rows = (int64_t)h->view.P * h->view.N;
  reset_kernel<<<blocks_for(rows), kBlock, 0, as_stream(stream)>>>(h->view);
  CSD_HIP(hipGetLastError());
  h->len_lo = h->len_hi = 0;
  return CSD_OK;
}

int csd_append(csd_index* h, const int32_t* d_tokens, const float* d_probs,
               const int32_t* d_counts, int32_t n, void* stream) {
  if (!h || !d_tokens || n < 0) return CSD_ERR_INVALID_ARG;
  if (n == 0) return CSD_OK;
  if (!d_counts && h->len_lo + n > h->cfg.max_len) return CSD_ERR_CAPACITY;
  int64_t rows = (int64_t)h->view.P * h->view.N;
  append_kernel<<<blocks_for(rows), kBlock, 0, as_stream(stream)>>>(h->view, d_tokens, d_probs,
                                                                     d_counts, n);
  CSD_HIP(hipGetLastError());
  if (!d_counts) h->len_lo += n;
  h->len_hi += n;
  if (h->len_hi > h->cfg.max_len) h->len_hi = h->cfg.max_len;
  return CSD_OK;
}

int csd_draft(csd_index* h, int32_t query_len, int32_t draft_len, int32_t* d_draft_tokens,
              int32_t* d_draft_len, float* d_token_scores, float* d_path_scores, void* stream) {
  if (!h || !d_draft_tokens || !d_draft_len) return CSD_ERR_INVALID_ARG;
  if (query_len < 1 || query_len > h->cfg.max_query_len) return CSD_ERR_INVALID_ARG;
  if (draft_len < 1 || draft_len > h->cfg.max_draft_len) return CSD_ERR_INVALID_ARG;
  int64_t rows = (int64_t)h->view.P * h->view.N;
  draft_kernel<<<xcd_grid(rows), kBlock, 0, as_stream(stream)>>>(
      h->view, query_len, draft_len, h->alpha_q, h->cfg.score_mode, d_draft_tokens, d_draft_len,
      d_token_scores, d_path_scores);
  CSD_HIP(hipGetLastError());
  return CSD_OK;
}

int csd_accept(csd_index* h, const int32_t* d_draft_tokens, const int32_t* d_draft_len,
               const int32_t* d_targets, int32_t draft_len, int32_t* d_accept_len, void* stream) {
  if (!h || !d_draft_tokens || !d_draft_len || !d_targets || !d_accept_len)
    return CSD_ERR_INVALID_ARG;
  if (draft_len < 1 || draft_len > h->cfg.max_draft_len) return CSD_ERR_INVALID_ARG;
  int64_t rows = (int64_t)h->view.P * h->view.N;
  accept_kernel<<<blocks_for(rows), kBlock, 0, as_stream(stream)>>>(
      rows, draft_len, d_draft_tokens, d_draft_len, d_targets, d_accept_len);
  CSD_HIP(hipGetLastError());
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
  do {
    e = hipMemsetAsync(bits, 0, (size_t)rows * words * sizeof(uint32_t), st);
    if (e != hipSuccess) break;
    dump_match_bits_kernel<<<xcd_grid(rows), kBlock, 0, st>>>(h->view, query_len, bits, words);
    count_bits_kernel<<<rows, kBlock, 0, st>>>(bits, words, counts);
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
  if (query_len < 1 || query_len > h->cfg.max_query_len) return CSD_ERR_INVALID_ARG;
  if (draft_len < 1 || draft_len > h->cfg.max_draft_len) return CSD_ERR_INVALID_ARG;
  hipStream_t st = as_stream(stream);
  int32_t rows = h->view.P * h->view.N;
  u64* tmp = nullptr;
  int32_t* counts = nullptr;
  size_t tmp_elems = (size_t)rows * kTableCap;
  CSD_HIP(hipMalloc(&tmp, 2 * tmp_elems * sizeof(u64)));
  hipError_t e = hipMalloc(&counts, ((size_t)rows + 1) * sizeof(int32_t));
  if (e != hipSuccess) { (void)hipFree(tmp); return hip_fail(e, "hipMalloc"); }
  int32_t tail[2] = {0, 0};   // total rows, bad flag
  do {
    dump_edge_rows_kernel<<<xcd_grid(rows), kBlock, 0, st>>>(h->view, query_len, draft_len, tmp,
                                                             tmp + tmp_elems, counts);
    offsets_kernel<<<1, 1, 0, st>>>(counts, rows, d_edge_off, counts + rows);
    scatter_edges_kernel<<<rows, kBlock, 0, st>>>(tmp, tmp + tmp_elems, d_edge_off, d_edge_duv,
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
