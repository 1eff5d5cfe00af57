// csd — the layered token DAG (Eq. 5) and the greedy layer-wise walk over it
// (rule after Eq. 5, Algorithm 1).
//
// Forms with identical results (all sums are exact integers):
//   tier 0  one wave, no tables: the DAG lives in the lanes.  walk_instances:
//           a lane per (match, layer) instance, for up to 8 matches;
//           walk_matches: a lane per match (or per two), for up to 128;
//   tier 1  LDS hash histograms, all L layers at once: layer d owns one region of the LDS table that
//           holds its edges (d,u,v) -> (count, probability sum) and its nodes
//           (d,*,v) -> in-weight; every edge slot links to its target node, so
//           the walk can fetch all ranks before its serial part starts;
//   tier 1b a thread per match (up to a workgroup's worth), layer by layer: only the
//           successors of the current node are tabulated (walk_wide);
//   tier 2  bounded memory for any input: one layer at a time, and within a
//           layer one class of tokens (by hash residue) at a time.
#pragma once

#include "csd_common.cuh"

namespace csd {

struct Region {                 // slots [base, base + mask] of the LDS table
  uint32_t base, mask;
};

// Orders the workgroup's LDS traffic only: unlike __syncthreads() it does not
// wait for global loads in flight, so a prefetch can stay in the air across it.
template <int BLOCK>
__device__ __forceinline__ void lds_barrier() {
  if (BLOCK == kWave) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  else asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int BLOCK, class LDS>
__device__ __forceinline__ void table_clear(LDS& s, uint32_t n_slots, int tid) {
  for (uint32_t h = tid; h < n_slots; h += BLOCK) s.table[h] = Slot{kEmpty, 0ull};
  if (tid == 0) s.overflow = 0;
}

// table[key] += delta inside a region, inserting the key if new; returns the
// slot.  Sets s.overflow when the region has no free slot (the caller then
// falls back) — never spins.
template <class LDS>
__device__ __forceinline__ uint32_t table_add(LDS& s, Region r, u64 key, u64 delta) {
  uint32_t h = dag_hash(key) & r.mask;
  for (uint32_t probe = 0; probe <= r.mask; ++probe) {
    Slot* slot = &s.table[r.base + h];
    u64 cur = slot->key;
    if (cur == kEmpty) {
      cur = atomicCAS(&slot->key, kEmpty, key);
      if (cur == kEmpty) cur = key;
    }
    if (cur == key) {
      atomicAdd(&slot->val, delta);
      return r.base + h;
    }
    h = (h + 1) & r.mask;
  }
  s.overflow = 1;
  return r.base;
}

template <class LDS>
__device__ __forceinline__ u64 table_get(const LDS& s, Region r, u64 key) {
  uint32_t h = dag_hash(key) & r.mask;
  for (uint32_t probe = 0; probe <= r.mask; ++probe) {
    Slot x = s.table[r.base + h];
    if (x.key == key) return x.val;
    if (x.key == kEmpty) return 0ull;
    h = (h + 1) & r.mask;
  }
  return 0ull;
}

// Workgroup-wide argmax of the per-thread candidates; every thread gets the result.
template <int BLOCK, class LDS>
__device__ __forceinline__ Cand block_argmax(LDS& s, Cand c, int tid, int parity) {
  c = wave_argmax(c);
  if (BLOCK == kWave) return c;
  if ((tid & 63) == 0) s.red[parity][tid >> 6] = c;
  lds_barrier<BLOCK>();
  int lane = tid & 63;                                  // every wave reduces the waves' results
  return wave_argmax(lane < BLOCK / kWave ? s.red[parity][lane] : cand_none());
}

__device__ __forceinline__ void note_choice(DraftOut& o, Cand best, int32_t d, int tid) {
  if (tid == d - 1) {
    o.tok = best.v;
    o.key = best.key;
  }
  o.key_sum += best.key;
  o.n = d;
}

// ---------------------------------------------------------------- tier 1: everything in LDS

// Matches n_fresh .. win_cap - 1 of the list have their continuation cached in LDS (match x in
// window x).
struct WinInfo {
  int32_t n_fresh, win_cap;
  __device__ __forceinline__ bool cached(int32_t mi) const { return mi >= n_fresh && mi < win_cap; }
};

struct Tier1 {                  // geometry of the table for one query
  uint32_t region;              // slots per layer (power of two)
  __device__ __forceinline__ Region layer(int32_t d) const {
    return Region{(uint32_t)(d - 1) * region, region - 1};
  }
};

__device__ __forceinline__ Tier1 tier1_geometry(int32_t M, int32_t L, int table_cap) {
  uint32_t want = 4u * (uint32_t)M;                   // a layer holds <= 2M keys: <= 50 % load
  uint32_t cap = (uint32_t)table_cap / (uint32_t)L;   // what fits (rounded down to 2^x below)
  uint32_t size = 8;
  while (size < want && size * 2 <= cap) size <<= 1;
  return Tier1{size};
}

// Eq. 5: every (match, layer) instance adds (1, p) to its edge (d,u,v) and its
// weight to its node (d,*,v).  The weight is linear in (count, probability
// sum), so a node's value is directly the in-weight the walk ranks by:
// sum over instances of  alpha_q * p + (65536 - alpha_q) * 65536.  Every edge
// slot also records where its target node sits (s.link).
template <int BLOCK, class LDS>
__device__ __forceinline__ Tier1 build_dag(LDS& s, const Ctx& c, int32_t M, int32_t L, WinInfo wi,
                                           uint32_t alpha_q) {
  Tier1 t1 = tier1_geometry(M, L, LDS::kTable);
  table_clear<BLOCK>(s, t1.region * (uint32_t)L, c.tid);
  block_sync<BLOCK>();
  int32_t items = M * L;
  const float inv_m = 1.0f / (float)M;
  for (int32_t idx = c.tid; idx < items; idx += BLOCK) {
    int32_t d = (int32_t)((float)idx * inv_m);        // idx / M for idx < 2^15, fixed up below
    d += (d + 1) * M <= idx;
    d -= d * M > idx;
    d += 1;
    int32_t mi = idx - (d - 1) * M;
    Match m = s.match[mi];
    uint32_t u, v;
    u64 w;
    bool alive;
    const int32_t ws = mi;
    if (wi.cached(mi)) {                              // no memory access
      alive = d <= (int32_t)m.rem_new;
      const int32_t* win = s.win + ws * 2 * L;
      v = (uint32_t)win[d - 1];
      u = d == 1 ? (uint32_t)c.Q[0] : (uint32_t)win[d - 2];
      w = pack_cs(1u, (uint32_t)win[L + d - 1]);
    } else {
      alive = layer_instance(c.y, m, d, (uint32_t)c.Q[0], u, v, w);
    }
    if (alive && !s.overflow) {
      Region r = t1.layer(d);
      uint32_t edge = table_add(s, r, dag_key(d, u, v), w);
      uint32_t node = table_add(s, r, dag_key(d, kAnyTok, v), weight_key(w, alpha_q));
      s.link[edge] = (uint16_t)node;                  // all instances of an edge agree
    }
  }
  block_sync<BLOCK>();
  return t1;
}

// Smallest g with 2^g >= M (M >= 1).
__device__ __forceinline__ int lanes_log2(int32_t M) { return M <= 1 ? 0 : 32 - __clz(M - 1); }

// Tier 0, for one wave and few matches: no tables at all.  Every layer owns an
// aligned group of G = 2^g lanes (M <= G, G * L <= 64); lane (d-1) * G + m holds
// instance (layer d, match m): its predecessor u, its token v and its weight.
// All lanes work out, in exchanges with the lanes of their own and of the next
// group (lane ^ r), what the walk needs: the weight of the lanes of the group
// with the same token (the in-weight of the lane's node; score_mode 1: with the
// same u as well: the weight of its edge), whether the lane's edge is the one
// the greedy step takes out of u, and which lane the walk goes on to from it.
// The walk itself is then one lane read per layer.  Same sums as the tables of
// tier 1, in exact integers: the same draft.
// G is a template parameter so that the exchange loops unroll and their lane permutes travel
// together instead of one round trip through the LDS crossbar per iteration.
template <int G, class LDS>
__device__ __forceinline__ void walk_instances(LDS& s, const Ctx& c, int32_t M, int32_t L,
                                               WinInfo wi, uint32_t alpha_q, int score_mode,
                                               DraftOut& o) {
  constexpr uint32_t kDeadU = 0xFFFFFFFEu, kDeadV = 0xFFFFFFFFu;   // no token: ids are < 2^29
  static_assert(G >= 1 && G <= kWave && (G & (G - 1)) == 0, "a group is a power of two of lanes");
  constexpr int g = G == 1 ? 0 : G == 2 ? 1 : G == 4 ? 2 : G == 8 ? 3 : G == 16 ? 4 : G == 32 ? 5 : 6;
  const int lane = c.tid;
  const int32_t d_mine = (lane >> g) + 1, mi = lane & (G - 1);
  uint32_t u = kDeadU, v = kDeadV;
  u64 key = 0;
  if (mi < M && d_mine <= L) {
    Match m = s.match[mi];
    u64 w;
    bool alive;
    const int32_t ws = mi;
    if (wi.cached(mi)) {                              // no memory access
      alive = d_mine <= (int32_t)m.rem_new;
      const int32_t* win = s.win + ws * 2 * L;
      v = (uint32_t)win[d_mine - 1];
      u = d_mine == 1 ? (uint32_t)c.Q[0] : (uint32_t)win[d_mine - 2];
      w = pack_cs(1u, (uint32_t)win[L + d_mine - 1]);
    } else {
      alive = layer_instance(c.y, m, d_mine, (uint32_t)c.Q[0], u, v, w);
    }
    key = alive ? weight_key(w, alpha_q) : 0ull;
    u = alive ? u : kDeadU;
    v = alive ? v : kDeadV;
  }
  auto from = [](int addr, uint32_t x) { return (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)x); };
  auto from64 = [&](int addr, u64 x) {
    return ((u64)from(addr, (uint32_t)(x >> 32)) << 32) | from(addr, (uint32_t)x);
  };
  auto lane64 = [](u64 x, int src) {
    return ((u64)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), src) << 32) |
           (u64)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, src);
  };
  // rank: the weight the greedy step ranks this lane's edge by
  u64 rank = key;
  static_for<1, G>([&](auto r) {
    uint32_t pv = from_xor_lane<r()>(lane, v), pu = from_xor_lane<r()>(lane, u);
    u64 pk = from_xor_lane64<r()>(lane, key);
    bool add = pv == v && (score_mode == 0 || pu == u);
    rank += add ? pk : 0ull;
  });
  // winner: no lane of the group with the same predecessor has a larger rank, or the same
  // rank and a lower token id (lanes with the same u and v are all winners, or none is)
  bool winner = u != kDeadU;
  static_for<1, G>([&](auto r) {
    uint32_t pv = from_xor_lane<r()>(lane, v), pu = from_xor_lane<r()>(lane, u);
    u64 pr = from_xor_lane64<r()>(lane, rank);
    bool beats = pu == u && (pr > rank || (pr == rank && pv < v));
    winner = winner && !beats;
  });
  // succ: the lane the walk moves to from this one: the first winner of the next layer's group
  // whose predecessor is this lane's token
  const uint32_t wu = winner ? u : kDeadU;
  int32_t succ = kWave;
#pragma unroll
  for (int r = 0; r < G; ++r) {
    const int partner = (lane + G) ^ r;
    uint32_t pu = from(partner << 2, wu);
    succ = (pu == v && partner < succ) ? partner : succ;
  }
  succ = (winner && d_mine < L && succ < kWave) ? succ : -1;
  // the serial part: one lane read per layer
  const u64 first = wave_ballot(winner) & (G >= kWave ? ~0ull : (1ull << G) - 1);
  int32_t at = first ? (int32_t)__ffsll((long long)first) - 1 : -1;
  int32_t chosen = 0;                                 // lane d-1: the lane layer d's choice sits in
  for (int32_t d = 1; d <= L && at >= 0; ++d) {
    chosen = lane == d - 1 ? at : chosen;
    o.key_sum += lane64(rank, at);
    o.n = d;
    at = __builtin_amdgcn_readlane(succ, at);
  }
  const int addr = chosen << 2;
  const uint32_t tok = from(addr, v);
  const u64 k = from64(addr, rank);
  if (lane < o.n) {
    o.tok = (int32_t)tok;
    o.key = k;
  }
}

// Tier 0 for up to 64 R matches that all have (or get) an LDS window: lane m holds
// match m (and m + 64, ..) and reads its continuation one layer ahead of the walk.  A layer's
// successors are the lanes whose previous token is the current node; a
// successor's count is the population of a ballot, its probability sum one wave
// reduction, and from the two follows its weight (Eq. 5) exactly as the tables
// of tier 1 would hold it.  Matches without a window (found among the newest
// positions) write theirs first.
// `windows`: M windows of 2 L words (s.win, or any other LDS the caller has free); with
// `split` given, only the first `split` of them, the others lie at `windows_beyond`.
// TREE: the prefix-tree pool instead of the DAG: a layer's successors are the lanes whose
// whole continuation so far is the draft so far, and only they count for a successor's weight.
// R: matches per lane (lane l holds matches l, l + 64, ..): up to 64 R matches.
template <bool TREE = false, int R = 1, class LDS>
__device__ __forceinline__ void walk_matches(LDS& s, const Ctx& c, int32_t M, int32_t L, WinInfo wi,
                                             int32_t* windows, uint32_t alpha_q, int score_mode,
                                             DraftOut& o, int32_t* windows_beyond = nullptr,
                                             int32_t split = INT_MAX) {
  const int lane = c.tid;
  int32_t rem[R];                                     // layers this lane's matches reach
  const int32_t* win[R];
  uint32_t u[R], v[R], p[R];
  bool on_draft[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int32_t mi = lane + r * kWave;
    const int32_t wx = mi < M ? mi : 0;
    int32_t* mine = wx < split ? windows + wx * 2 * L : windows_beyond + (wx - split) * 2 * L;
    rem[r] = 0;
    if (mi < M) {
      Match m = s.match[mi];
      rem[r] = (int32_t)m.rem_new < L ? (int32_t)m.rem_new : L;
      if (!wi.cached(mi)) {
        for (int32_t d = 1; d <= rem[r]; ++d) {
          uint32_t uu, vv;
          u64 w;
          layer_instance(c.y, m, d, 0u, uu, vv, w);
          mine[d - 1] = (int32_t)vv;
          mine[L + d - 1] = (int32_t)cs_sum(w);
        }
      }
    }
    win[r] = mine;
    on_draft[r] = mi < M;
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    u[r] = (uint32_t)c.Q[0];
    v[r] = (uint32_t)win[r][0];
    p[r] = (uint32_t)win[r][L];
  }
  int32_t cur = c.Q[0];
  const uint32_t per_count = 65536u - alpha_q;        // Eq. 5 in fixed point, as weight_key()
  for (int32_t d = 1; d <= L; ++d) {
    const int32_t ahead = d < L ? d : L - 1;          // layer d + 1 travels while d is decided
    uint32_t v_next[R], p_next[R];
    u64 counted[R], todo[R], any = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      v_next[r] = (uint32_t)win[r][ahead];
      p_next[r] = (uint32_t)win[r][L + ahead];
      const u64 alive = wave_ballot(d <= rem[r]);
      const u64 cand = (TREE ? wave_ballot(on_draft[r]) : wave_ballot(u[r] == (uint32_t)cur)) & alive;
      counted[r] = (TREE || score_mode) ? cand : alive;   // whose weight a successor's rank sums
      todo[r] = cand;
      any |= cand;
    }
    if (!any) break;                                  // leaf: no edge leaves cur
    auto successor = [&]() {                          // the token of the first lane left, and its rank
      uint32_t vt = 0;
      bool found = false;
#pragma unroll
      for (int r = 0; r < R; ++r) {                   // (uniform: todo is a scalar)
        if (!found && todo[r] != 0) {
          vt = (uint32_t)__builtin_amdgcn_readlane((int)v[r], (int)__ffsll((long long)todo[r]) - 1);
          found = true;
        }
      }
      uint32_t count = 0, mine = 0;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const u64 same = wave_ballot(v[r] == vt) & counted[r];
        count += (uint32_t)__popcll(same);
        mine += lanes_of(same, p[r]);
        todo[r] &= ~same;
      }
      const uint32_t sum = wave_sum(mine);
      return Cand{(u64)alpha_q * sum + ((u64)(per_count * count) << 16), (int32_t)vt};
    };
    auto left = [&]() {
      u64 x = 0;
#pragma unroll
      for (int r = 0; r < R; ++r) x |= todo[r];
      return x;
    };
    Cand best = successor();
    while (left()) best = cand_best(best, successor());   // the matches disagree: one round per token
    note_choice(o, best, d, lane);
    cur = best.v;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (TREE) on_draft[r] = on_draft[r] && v[r] == (uint32_t)best.v;
      u[r] = v[r];
      v[r] = v_next[r];
      p[r] = p_next[r];
    }
  }
}

// Replaces the value of every edge slot by the weight the greedy step ranks it
// by: the in-weight of its target node (score_mode 0, the rule after Eq. 5) or
// its own weight (mode 1).  Node slots are only read.  The caller synchronises.
template <int BLOCK, class LDS>
__device__ __forceinline__ void score_edges(LDS& s, uint32_t n_slots, uint32_t alpha_q,
                                            int score_mode, int tid) {
#pragma unroll 4
  for (uint32_t h = tid; h < n_slots; h += BLOCK) {
    Slot x = s.table[h];
    uint32_t node = (uint32_t)s.link[h] & (uint32_t)(LDS::kTable - 1);   // stale links stay in range
    u64 in_weight = s.table[node].val;
    if (x.key != kEmpty && key_u(x.key) != kAnyTok)
      s.table[h].val = score_mode ? weight_key(x.val, alpha_q) : in_weight;
  }
}

// Greedy walk (rule after Eq. 5) over tables whose edges score_edges() has scored.
template <int BLOCK, class LDS>
__device__ __forceinline__ void walk_scored(LDS& s, const Ctx& c, Tier1 t1, int32_t L, DraftOut& o) {
  int32_t cur = c.Q[0];
  for (int32_t d = 1; d <= L; ++d) {
    Region r = t1.layer(d);
    u64 want = dag_key(d, (uint32_t)cur, 0) >> 29;
    Cand best = cand_none();
#pragma unroll 4
    for (uint32_t h = c.tid; h <= r.mask; h += BLOCK) {
      Slot x = s.table[r.base + h];
      if ((x.key >> 29) == want) best = cand_best(best, Cand{x.val, (int32_t)key_v(x.key)});
    }
    best = block_argmax<BLOCK>(s, best, c.tid, d & 1);
    if (best.v == INT_MAX) break;                     // leaf: no edge leaves cur
    note_choice(o, best, d, c.tid);
    cur = best.v;
  }
}

// Does the one-wave walk below keep all layers in registers?
template <int LCAP>
__device__ __forceinline__ bool walk_fits_registers(Tier1 t1, int32_t L) {
  return t1.region <= (uint32_t)kWave && L <= LCAP;
}

// Greedy walk over the finished tables (rule after Eq. 5).  When a layer's
// region fits the wave (one slot per lane) every lane fetches its slot of ALL
// layers, and the ranks behind them, before the walk starts: the serial part is
// then a compare, a ballot and a lane read per layer, with no memory latency.
// Larger tables are scored in place first and then searched layer by layer.
template <int BLOCK, int LCAP, class LDS>
__device__ __forceinline__ void walk_dag(LDS& s, const Ctx& c, Tier1 t1, int32_t L,
                                         uint32_t alpha_q, int score_mode, DraftOut& o) {
  int32_t cur = c.Q[0];
  if (BLOCK == kWave && walk_fits_registers<LCAP>(t1, L)) {
    // Three rounds of independent LDS reads (slot, link, linked node), none of them behind a
    // branch, so that the reads of all layers are in flight together.
    u64 key[LCAP], rank[LCAP];
    uint32_t at[LCAP], node[LCAP];
    const bool mine = (uint32_t)c.tid < t1.region;
#pragma unroll
    for (int d = 1; d <= LCAP; ++d)
      at[d - 1] = (d <= L && mine) ? (uint32_t)(d - 1) * t1.region + (uint32_t)c.tid : 0u;
#pragma unroll
    for (int d = 1; d <= LCAP; ++d) {
      Slot x = s.table[at[d - 1]];
      key[d - 1] = (d <= L && mine) ? x.key : kEmpty;
      rank[d - 1] = x.val;
      node[d - 1] = (uint32_t)s.link[at[d - 1]] & (uint32_t)(LDS::kTable - 1);   // stale links stay in range
    }
    if (score_mode == 0) {
#pragma unroll
      for (int d = 1; d <= LCAP; ++d) rank[d - 1] = s.table[node[d - 1]].val;
    } else {
#pragma unroll
      for (int d = 1; d <= LCAP; ++d) rank[d - 1] = weight_key(rank[d - 1], alpha_q);
    }
    bool going = true;                                // no `break`: the loop must unroll fully
#pragma unroll
    for (int d = 1; d <= LCAP; ++d) {
      if (d <= L && going) {
        u64 want = dag_key(d, (uint32_t)cur, 0) >> 29;
        Cand best = cand_none();
        if ((key[d - 1] >> 29) == want) best = Cand{rank[d - 1], (int32_t)key_v(key[d - 1])};
        best = wave_argmax(best);
        going = best.v != INT_MAX;                    // leaf: no edge leaves cur
        if (going) {
          note_choice(o, best, d, c.tid);
          cur = best.v;
        }
      }
    }
    return;
  }
  score_edges<BLOCK>(s, t1.region * (uint32_t)L, alpha_q, score_mode, c.tid);
  block_sync<BLOCK>();
  walk_scored<BLOCK>(s, c, t1, L, o);
}

// ---------------------------------------------------------------- layer by layer

// Successors of `cur` in layer d as held by a region with raw (C, S) values.
template <int BLOCK, class LDS>
__device__ __forceinline__ Cand scan_successors(const LDS& s, Region r, int d, int32_t cur,
                                                uint32_t alpha_q, int score_mode, int tid,
                                                Cand best) {
  u64 want = dag_key(d, (uint32_t)cur, 0) >> 29;
  for (uint32_t h = tid; h <= r.mask; h += BLOCK) {
    Slot x = s.table[r.base + h];
    if ((x.key >> 29) != want) continue;
    uint32_t v = key_v(x.key);
    u64 w = score_mode ? x.val : table_get(s, r, dag_key(d, kAnyTok, v));
    best = cand_best(best, Cand{weight_key(w, alpha_q), (int32_t)v});
  }
  return best;
}

// Tier 1b, for up to BLOCK matches where walk_tab (below) does not apply: edge scoring,
// token ids of 2^21 or more, more than its instances, or too many distinct continuations.
// One thread per match and no per-layer table of all instances: a layer only needs the weights of the successors of the current
// node, and those are few.  Per layer, (A) the candidates — matches whose previous token
// is the current node — enter their token in a hash set (a key carries the layer number,
// so the set is never cleared: entries of earlier layers count as free slots); (B) every
// match that reaches the layer looks its token up there and, if it is a successor, adds
// its (1, p) to the successor's cell (score_mode 1: only the candidates do); (C) the
// thread that entered a successor ranks it and puts it on a short list, which every wave
// then reads for the heaviest (ties: lowest token).  Same sums as the tables of tier 1, in
// exact integers: the same draft.  Set, cells and list lie over the (otherwise unused)
// table.  Waves without a match leave before the layers start (a workgroup barrier waits
// for the waves that are still running only), so a row with few matches pays for few waves.
// Nothing after this function may synchronise the workgroup.
// (Measured against two other forms with identical results: every instance of a layer added
// to a set of all the layer's keys, with two barriers per layer instead of three, was 4 %
// slower on the one-edit step; the ranks of all instances of all layers tabulated before the
// walk, which then needs one argmax and one barrier per layer, 20 % slower: unrolled over the
// layers its code is long, and code that runs once per launch is fetched cold.)
template <int BLOCK, class LDS>
__device__ __forceinline__ void walk_wide(LDS& s, const Ctx& c, int32_t M, int32_t L,
                                          uint32_t alpha_q, int score_mode, DraftOut& o) {
  constexpr uint32_t kSet = 2 * BLOCK;                 // at most BLOCK distinct successors: half load
  static_assert(2 * kSet * sizeof(u64) + 2 * BLOCK * sizeof(Cand) <= sizeof(s.table),
                "set, cells and the two successor lists fit the table");
  u64* keys = reinterpret_cast<u64*>(s.table);         // (layer << 32) | token, or kEmpty
  u64* cell = keys + kSet;                             // (count, probability sum) of the key's token
  Cand* list = reinterpret_cast<Cand*>(cell + kSet);   // [2][BLOCK] successors of a layer, ranked
  int32_t* listed = s.chosen;                          // [2] how many (the tree pool's array is free here)
  for (uint32_t h = c.tid; h < kSet; h += BLOCK) keys[h] = kEmpty;
  if (c.tid < 2) listed[c.tid] = 0;
  int32_t rem = 0, j = 0, e = 0, old_j = 1;
  if (c.tid < M) {
    Match m = s.match[c.tid];
    rem = (int32_t)m.rem_new < L ? (int32_t)m.rem_new : L;
    j = c.y.pos_path(m.pos);
    e = c.y.pos_index(m.pos);
    old_j = e + (int32_t)m.rel_old;                   // exact wherever it decides (see layer_instance)
  }
  int32_t cur = c.Q[0];
  uint32_t u = (uint32_t)c.Q[0];
  // a match's token and probability of layer x are requested two layers ahead of their use;
  // lanes whose candidate has ended by then read its first cell again: every lane loads,
  // nothing branches.  Nearly always everything a wave needs is history already: then it comes
  // from fixed addresses.  (Requesting the whole continuation up front, all loads together,
  // was slower: sixteen loads per thread before the first layer can start.)
  const int32_t* tok_at = c.y.tok + c.y.cell(j, e);
  const uint32_t* pq_at = c.y.pq + c.y.cell(j, e);
  const bool plain = wave_ballot(c.tid < M && old_j - e < rem) == 0;   // uniform over the wave
  auto request = [&](int32_t x, int32_t& tok, Paths::ProbWord& prob) {
    const bool has = x <= rem;
    if (plain) {
      tok = tok_at[has ? x - 1 : 0];
      prob = Paths::ProbWord{pq_at[has ? x - 1 : 0], true, false};
    } else {
      tok = c.y.token(has ? j : 0, has ? e + x - 1 : 0, has ? old_j : 1);
      prob = c.y.prob_load(has ? j : 0, has ? e + x - 1 : 0, has ? old_j : 1);
    }
  };
  int32_t tok_a, tok_b;
  Paths::ProbWord prob_a, prob_b;
  request(1, tok_a, prob_a);
  request(2, tok_b, prob_b);
  lds_barrier<BLOCK>();                               // the set is empty
  if (c.tid >= ((M + kWave - 1) & ~(kWave - 1))) return;   // waves without a match
  const int lane = c.tid & (kWave - 1);
  for (int32_t d = 1; d <= L; ++d) {
    consume_here(tok_a);
    consume_here(prob_a.word);
    const uint32_t v = (uint32_t)tok_a;
    const u64 w = pack_cs(1u, Paths::prob_value(prob_a));
    tok_a = tok_b;
    prob_a = prob_b;
    request(d + 2, tok_b, prob_b);
    const bool alive = d <= rem;
    const bool cand = alive && u == (uint32_t)cur;
    const u64 mine = ((u64)(uint32_t)d << 32) | v;
    const uint32_t h0 = (v * 0x9E3779B1u) >> 7 & (kSet - 1);
    const int par = d & 1;
    // (A) successors of the current node enter the set; the thread that enters one owns it
    uint32_t slot = h0;
    bool owner = false;
    if (cand) {
      u64 seen = keys[slot];
      for (uint32_t probe = 0; probe < 2 * kSet; ++probe) {
        if (seen == mine) break;
        if ((uint32_t)(seen >> 32) != (uint32_t)d) {   // free: empty, or an earlier layer's
          const u64 prev = atomicCAS(&keys[slot], seen, mine);
          if (prev == seen) {
            owner = true;
            cell[slot] = 0ull;
            break;
          }
          seen = prev;                                // somebody else took it: look again
          continue;
        }
        slot = (slot + 1) & (kSet - 1);
        seen = keys[slot];
      }
    }
    lds_barrier<BLOCK>();
    if (c.tid == 0) listed[par ^ 1] = 0;              // the next layer's list: its last readers are past the barrier
    // (B) Eq. 5: the instances of this layer whose token is a successor
    if (cand) {
      atomicAdd(&cell[slot], w);
    } else if (alive && score_mode == 0) {
      uint32_t h = h0;
      for (uint32_t probe = 0; probe < kSet; ++probe) {
        const u64 seen = keys[h];
        if (seen == mine) {
          atomicAdd(&cell[h], w);
          break;
        }
        if ((uint32_t)(seen >> 32) != (uint32_t)d) break;   // free slot: not a successor
        h = (h + 1) & (kSet - 1);
      }
    }
    lds_barrier<BLOCK>();
    // (C) every successor once, ranked by its owner; the heaviest wins, ties to the lowest token
    if (owner) list[par * BLOCK + atomicAdd(&listed[par], 1)] = Cand{weight_key(cell[slot], alpha_q), (int32_t)v};
    lds_barrier<BLOCK>();
    const int32_t n = listed[par];                     // <= BLOCK
    if (n == 0) break;                                 // leaf: no edge leaves cur
    Cand best = cand_none();
    if (n <= 4) {                                      // every lane reads the few entries
      for (int x = 0; x < n; ++x) best = cand_best(best, list[par * BLOCK + x]);
    } else {
      for (int x = lane; x < n; x += kWave) best = cand_best(best, list[par * BLOCK + x]);
      best = wave_argmax(best);
    }
    note_choice(o, best, d, c.tid);
    cur = best.v;
    u = v;
  }
}

// Tier 1c, the usual form for 65 .. BLOCK matches: Eq. 5's node weights do not depend on the
// walk (a node's in-weight counts EVERY match that carries its token in that layer), so they
// are tabulated first, for all layers at once and by all waves, and the greedy walk after
// that is short.
//   Fill: BLOCK / M threads share a match, each taking every (BLOCK / M)-th layer; an
//   instance (match, layer d, token v) finds or enters the 32-bit key (d, v) in a hash set (double hashing),
//   adds its (1, p) to the key's cell and notes the slot.  No barrier between layers.
//   Walk, one thread per match: per layer the candidates (matches whose previous token is
//   the current node; all of them in layer 1) rank their node, and the heaviest (ties: lowest
//   token) is found with a wave maximum and one 64-bit LDS atomic maximum per wave: weight
//   (+ 1, so that 0 means "no successor") above the inverted token.  One barrier per layer;
//   the next layer's slot, key, cell and rank are fetched and computed before it, behind the
//   atomic.
// Needs score_mode 0 (edge weights depend on the walk: walk_wide), tokens below 2^21 (the
// weight of at most 1024 instances takes 43 bits) and at most kTabInstances instances.  The
// set has two to four times as many slots as there are instances, but at most kTabSlots; an
// instance that finds no place within kTabProbes gives up, and the function then returns
// false with nothing decided (thousands of distinct continuations: the caller takes walk_wide).  Same sums as the other tiers, in exact
// integers: the same draft.  Cells lie over the table, the layers' maxima over the links,
// keys and slots behind the first BLOCK entries of the match list (which stay).
// After a return of true nothing may synchronise the workgroup.
constexpr int kTabSlots = 8192;
constexpr int kTabInstances = 8192;
constexpr int kTabProbes = 128;
constexpr int kTabTokenBits = 21;

template <int BLOCK>
__device__ __forceinline__ bool walk_tab_fits(int32_t M, int32_t L, int32_t vocab, int score_mode) {
  return score_mode == 0 && M <= BLOCK && M * L <= kTabInstances && vocab <= (1 << kTabTokenBits);
}

// Empties walk_tab's key set and zeroes its cells and the layers' maxima, all kTabSlots of
// them, with threads `first` .. BLOCK - 1 (the scan kernel has this done by the waves that
// idle while one of them hands the row's matches over; the first BLOCK entries of the match
// list are not touched).
template <int BLOCK, class LDS>
__device__ __forceinline__ void walk_tab_clear(LDS& s, int tid, int first) {
  uint2* cells2 = reinterpret_cast<uint2*>(s.table);
  uint2* keys2 = reinterpret_cast<uint2*>(&s.match[BLOCK]);
  u64* best = reinterpret_cast<u64*>(s.link);
  if (tid < first) return;
  for (uint32_t x = tid - first; x < kTabSlots; x += BLOCK - first) cells2[x] = uint2{0u, 0u};
  for (uint32_t x = tid - first; x < kTabSlots / 2; x += BLOCK - first) keys2[x] = uint2{~0u, ~0u};
  if (tid - first < CSD_MAX_DRAFT_LEN) best[tid - first] = 0ull;
  if (tid == first) s.overflow = 0;
}

// cleared: walk_tab_clear has been called (and a barrier passed) since the table was last used.
template <int BLOCK, class LDS>
__device__ __forceinline__ bool walk_tab(LDS& s, const Ctx& c, int32_t M, int32_t L, uint32_t alpha_q,
                                         DraftOut& o, bool cleared = false) {
  static_assert(LDS::kMatch >= BLOCK && sizeof(s.table) >= kTabSlots * sizeof(u64) &&
                sizeof(s.link) >= CSD_MAX_DRAFT_LEN * sizeof(u64),
                "cells over the table, the layers' maxima over the links");
  static_assert((LDS::kMatch - BLOCK) * sizeof(Match) + sizeof(s.win) >=
                kTabSlots * sizeof(uint32_t) + kTabInstances * sizeof(uint16_t),
                "keys and slots behind the listed matches");
  static_assert(offsetof(LDS, win) == offsetof(LDS, match) + sizeof(s.match), "no gap before the windows");
  constexpr uint32_t kNoKey = ~0u;
  constexpr uint32_t kTokBits = (1u << kTabTokenBits) - 1u;
  u64* cell = reinterpret_cast<u64*>(s.table);         // [n_slots] (count, probability sum)
  u64* best = reinterpret_cast<u64*>(s.link);          // [L] the layer's heaviest successor, packed
  uint32_t* keys = reinterpret_cast<uint32_t*>(&s.match[BLOCK]);   // [n_slots] (d - 1) << 24 | token
  uint16_t* slot_of = reinterpret_cast<uint16_t*>(keys + kTabSlots);   // [L][M]
  // two to four times as many slots as instances (a power of two, at most kTabSlots): what is
  // not used is not cleared
  int slot_bits = 32 - __clz(4 * M * L - 1);
  slot_bits = slot_bits < 10 ? 10 : (slot_bits > 13 ? 13 : slot_bits);
  if (cleared) slot_bits = 13;                         // (uniform) all of them are empty: use them
  const uint32_t n_slots = 1u << slot_bits;
  if (!cleared) {                                      // empty set, zero cells
    uint2* cells2 = reinterpret_cast<uint2*>(cell);
    uint2* keys2 = reinterpret_cast<uint2*>(keys);
    for (uint32_t x = c.tid; x < n_slots; x += BLOCK) cells2[x] = uint2{0u, 0u};
    for (uint32_t x = c.tid; x < n_slots / 2; x += BLOCK) keys2[x] = uint2{kNoKey, kNoKey};
    if (c.tid < CSD_MAX_DRAFT_LEN) best[c.tid] = 0ull;
    if (c.tid == 0) s.overflow = 0;
  }
  // the threads of a match: r-th of R, layers r + 1, r + 1 + R, ...
  const int32_t R = BLOCK / M;
  int32_t r = (int32_t)((float)c.tid * (1.0f / (float)M));   // tid / M, fixed up
  r += (r + 1) * M <= c.tid;
  r -= r * M > c.tid;
  const int32_t t = c.tid - r * M;
  const bool works = r < R;
  const Match m = s.match[works ? t : 0];
  const int32_t rem = (int32_t)m.rem_new < L ? (int32_t)m.rem_new : L;
  const int32_t j = c.y.pos_path(m.pos), e = c.y.pos_index(m.pos);
  const int32_t old_j = e + (int32_t)m.rel_old;       // exact wherever it decides (see layer_instance)
  const int32_t* tok_at = c.y.tok + c.y.cell(j, e);
  const uint32_t* pq_at = c.y.pq + c.y.cell(j, e);
  // One instance: the key (d, v) is found or entered, its cell takes the instance's (1, p).
  // Called by all lanes of a wave together; the probes are a loop of the wave (until no lane
  // is left looking), which costs fewer instructions than a loop of each lane.
  auto instance = [&](bool active, int32_t d, uint32_t v, uint32_t p) {
    const uint32_t mine = ((uint32_t)(d - 1) << 24) | v;
    uint32_t h = (mine * 0x9E3779B1u) >> (32 - slot_bits);   // the product's high bits: a slot
    const uint32_t stride = (mine * 0x85EBCA6Bu) >> 15 | 1u;  // odd: the probes reach every slot
    bool looking = active;
    for (int probe = 0; probe < kTabProbes && wave_ballot(looking) != 0; ++probe) {   // uniform
      uint32_t seen = keys[h];
      if (looking && seen == kNoKey) seen = atomicCAS(&keys[h], kNoKey, mine);
      const bool placed = seen == mine || seen == kNoKey;   // there already, or entered just now
      h = (looking && !placed) ? (h + stride) & (n_slots - 1) : h;
      looking = looking && !placed;
    }
    if (active && !looking) {
      atomicAdd(&cell[h], pack_cs(1u, p));
      slot_of[(d - 1) * M + t] = (uint16_t)h;
    } else if (active) {
      s.overflow = 1;
    }
  };
  // A thread's tokens and probabilities are requested two turns ahead, as in walk_wide.  When
  // everything the wave needs is history already (nearly always) they come from fixed addresses
  // and the probability is the quantised one.
  if (wave_ballot(works && old_j - e < rem) == 0) {    // uniform over the wave
    auto request = [&](int32_t x, uint32_t& tok, uint32_t& p) {
      const int32_t at = (works && x <= rem) ? x - 1 : 0;
      tok = (uint32_t)tok_at[at];
      p = pq_at[at];
    };
    uint32_t tok_a, tok_b, p_a, p_b;
    request(r + 1, tok_a, p_a);
    request(r + 1 + R, tok_b, p_b);
    lds_barrier<BLOCK>();
    CSD_STAMP(c.unit, 10, CSD_CLOCK());
    for (int32_t d = r + 1; d <= L; d += R) {
      consume_here(tok_a);
      consume_here(p_a);
      const uint32_t v = tok_a & 0xFFFFFFu, pv = p_a;
      tok_a = tok_b;
      p_a = p_b;
      request(d + 2 * R, tok_b, p_b);
      instance(works && d <= rem, d, v, pv);
    }
  } else {
    auto request = [&](int32_t x, int32_t& tok, Paths::ProbWord& prob) {
      const bool has = works && x <= rem;
      tok = c.y.token(has ? j : 0, has ? e + x - 1 : 0, has ? old_j : 1);
      prob = c.y.prob_load(has ? j : 0, has ? e + x - 1 : 0, has ? old_j : 1);
    };
    int32_t tok_a, tok_b;
    Paths::ProbWord prob_a, prob_b;
    request(r + 1, tok_a, prob_a);
    request(r + 1 + R, tok_b, prob_b);
    lds_barrier<BLOCK>();
    CSD_STAMP(c.unit, 10, CSD_CLOCK());
    for (int32_t d = r + 1; d <= L; d += R) {
      consume_here(tok_a);
      consume_here(prob_a.word);
      const uint32_t v = (uint32_t)tok_a & 0xFFFFFFu, pv = Paths::prob_value(prob_a);
      tok_a = tok_b;
      prob_a = prob_b;
      request(d + 2 * R, tok_b, prob_b);
      instance(works && d <= rem, d, v, pv);
    }
  }
  lds_barrier<BLOCK>();                                // Eq. 5's sums are complete
  CSD_STAMP(c.unit, 11, CSD_CLOCK());
  if (s.overflow) return false;                        // uniform over the workgroup
  if (c.tid >= ((M + kWave - 1) & ~(kWave - 1))) return true;   // waves without a match of their own
  const int lane = c.tid & (kWave - 1);
  const bool mine_too = c.tid < M;                     // here r = 0, t = tid
  // A layer's node of this thread's match is no part of the choice: its slot is read two
  // layers ahead, key and cell one layer ahead, its rank (as the maximum takes it) is computed
  // behind the atomic of the layer before.
  auto slot_at = [&](int32_t d) { return (mine_too && d <= rem) ? (uint32_t)slot_of[(d - 1) * M + c.tid] : 0u; };
  auto rank = [&](uint32_t key, u64 sums, uint32_t& v, uint32_t& hi, uint32_t& lo) {
    v = key & 0xFFFFFFu;
    const u64 packed = ((weight_key(sums, alpha_q) + 1ull) << kTabTokenBits) | (u64)(kTokBits - (v & kTokBits));
    hi = (uint32_t)(packed >> 32);
    lo = (uint32_t)packed;
  };
  int32_t cur = c.Q[0];
  uint32_t u = (uint32_t)c.Q[0], v, hi, lo;
  const uint32_t slot_1 = slot_at(1), slot_2 = slot_at(2);
  uint32_t slot_n = slot_at(3);
  rank(keys[slot_1], cell[slot_1], v, hi, lo);
  uint32_t key_n = keys[slot_2];
  u64 sums_n = cell[slot_2];
  for (int32_t d = 1; d <= L; ++d) {
    const bool cand = mine_too && d <= rem && u == (uint32_t)cur;
    const uint32_t top_hi = wave_max(cand ? hi : 0u);
    const uint32_t top_lo = wave_max((cand && hi == top_hi) ? lo : 0u);
    if (lane == 0 && (top_hi | top_lo) != 0u) atomicMax(&best[d - 1], ((u64)top_hi << 32) | top_lo);
    uint32_t v_next, hi_next, lo_next;
    rank(key_n, sums_n, v_next, hi_next, lo_next);     // layer d + 1
    consume_here(hi_next);                             // (computed here, behind the atomic: not after the barrier)
    consume_here(lo_next);
    lds_barrier<BLOCK>();
    const u64 top = best[d - 1];
    key_n = keys[slot_n];                              // layer d + 2
    sums_n = cell[slot_n];
    slot_n = slot_at(d + 3);
    if (top == 0ull) break;                            // leaf: no edge leaves cur
    const Cand chosen{(top >> kTabTokenBits) - 1ull, (int32_t)(kTokBits - ((uint32_t)top & kTokBits))};
    note_choice(o, chosen, d, c.tid);
    cur = chosen.v;
    u = v;
    v = v_next;
    hi = hi_next;
    lo = lo_next;
  }
  return true;
}

// The same idea for ONE wave (the one-wave kernels), in place of the per-layer tables of all
// instances when a row has more matches than the lane-per-match walks take: with one-edit
// matching such a row's continuations mostly differ, and the walks that settle one distinct
// token per round, like the tables with an edge and a node entry per instance, cost it 100 us
// and more.  The layers are done in runs that keep the key set at most three quarters full
// (a run's first layer is entered once more by the next run, whose first walked layer reads
// its matches' previous tokens there).  Fill: a run's instances are dealt to the lanes layer
// by layer; an instance's token and probability come from its match's LDS window or, for
// matches without one, from memory (both requested for the next instance before this one is
// entered; every lane issues both loads, from a harmless address where it has no use for one).
// Walk: a lane looks at its matches (lane, lane + 64, ..) layer by layer; the previous
// layer's token of a match is read back through its slot.  Set and cells lie over table and
// links, the slots in the upper half of the match list.  Returns false, with nothing
// decided, when an instance of the first run finds no place (later runs cannot fail: see below).
template <class LDS>
constexpr uint32_t tab_wave_slots() {
  uint32_t n = 1;
  while (2 * n * 12 <= sizeof(Slot) * LDS::kTable + sizeof(uint16_t) * (LDS::kTable > LDS::kMatch ? LDS::kTable : LDS::kMatch))
    n *= 2;
  return n;
}
template <class LDS>
__device__ __forceinline__ bool walk_tab_wave_fits(int32_t M, int32_t vocab, int score_mode) {
  if (tab_wave_slots<LDS>() < 1024) return false;      // (the small layouts: not worth its code there)
  return score_mode == 0 && vocab <= (1 << kTabTokenBits) && M <= LDS::kMatch / 2 &&
         (uint32_t)(2 * M) <= tab_wave_slots<LDS>() / 4 * 3;     // runs of at least one new layer
}

template <class LDS>
__device__ __forceinline__ bool walk_tab_wave(LDS& s, const Ctx& c, WinInfo wi, int32_t M, int32_t L,
                                              uint32_t alpha_q, DraftOut& o) {
  constexpr uint32_t kSlots = tab_wave_slots<LDS>();
  static_assert(offsetof(LDS, link) == offsetof(LDS, table) + sizeof(s.table), "the links follow the table");
  static_assert(LDS::kWin >= 2 * CSD_MAX_DRAFT_LEN, "window 0 exists for any draft length");
  static_assert((LDS::kMatch / 2) * sizeof(Match) >= kSlots * sizeof(uint16_t), "a slot per instance of a run");
  constexpr uint32_t kNoKey = ~0u;
  constexpr uint32_t kTokBits = (1u << kTabTokenBits) - 1u;
  u64* cell = reinterpret_cast<u64*>(s.table);                        // [kSlots]
  uint32_t* keys = reinterpret_cast<uint32_t*>(cell + kSlots);         // [kSlots] (d - 1) << 24 | token
  uint16_t* slot_of = reinterpret_cast<uint16_t*>(&s.match[LDS::kMatch / 2]);   // [layers of the run][M]
  const int lane = c.tid;
  struct Instance {
    int32_t mi, d;
    bool alive, cached;
    int32_t tok_window, tok_memory;
    uint32_t p_window;
    Paths::ProbWord p_memory;
  };
  auto request = [&](int32_t mi, int32_t d, int32_t d_last) {
    Instance x;
    x.mi = mi;
    x.d = d;
    const bool there = d <= d_last;
    const Match m = s.match[there ? mi : 0];
    x.alive = there && d <= (int32_t)m.rem_new;
    x.cached = wi.cached(mi);
    const bool from_memory = x.alive && !x.cached;
    const int32_t j = c.y.pos_path(m.pos), e = c.y.pos_index(m.pos);
    const int32_t old_j = e + (int32_t)m.rel_old;     // exact wherever it decides (see layer_instance)
    x.tok_memory = c.y.token(from_memory ? j : 0, from_memory ? e + d - 1 : 0, from_memory ? old_j : 1);
    x.p_memory = c.y.prob_load(from_memory ? j : 0, from_memory ? e + d - 1 : 0, from_memory ? old_j : 1);
    const int32_t* win = s.win + ((x.alive && x.cached) ? mi : 0) * 2 * L;
    x.tok_window = win[x.alive ? d - 1 : 0];
    x.p_window = (uint32_t)win[L + (x.alive ? d - 1 : 0)];
    return x;
  };
  const int32_t per_run = (int32_t)(kSlots / 4 * 3) / M - 1;   // new layers per run, >= 1
  int32_t cur = c.Q[0];
  for (int32_t d0 = 1; d0 <= L; d0 += per_run) {
    const int32_t d_first = d0 > 1 ? d0 - 1 : 1;      // entered: d_first .. d_last; walked: d0 .. d_last
    const int32_t d_last = d0 + per_run - 1 < L ? d0 + per_run - 1 : L;
    for (uint32_t x = lane; x < kSlots; x += kWave) {
      cell[x] = 0ull;
      keys[x] = kNoKey;
    }
    lds_barrier<kWave>();
    // ---- fill: the run's instances (layer, match), lane by lane
    int32_t mi = lane, d = d_first;
    while (mi >= M && d <= d_last) {
      mi -= M;
      ++d;
    }
    bool failed = false;
    auto advance = [&]() {                               // the lane's next instance
      mi += kWave;
      while (mi >= M && d <= d_last) {
        mi -= M;
        ++d;
      }
    };
    // requested one instance ahead (three ahead was no faster: the wave is bound by the
    // instructions it issues, not by these loads)
    constexpr int kAhead = 1;
    Instance queue[kAhead];
#pragma unroll
    for (int x = 0; x < kAhead; ++x) {
      queue[x] = request(mi, d, d_last);
      advance();
    }
    while (wave_ballot(queue[0].d <= d_last) != 0) {     // uniform over the wave
      const Instance now = queue[0];
#pragma unroll
      for (int x = 0; x + 1 < kAhead; ++x) queue[x] = queue[x + 1];
      queue[kAhead - 1] = request(mi, d, d_last);
      advance();
      const uint32_t v = (uint32_t)(now.cached ? now.tok_window : now.tok_memory) & 0xFFFFFFu;
      const uint32_t p = now.cached ? now.p_window : Paths::prob_value(now.p_memory);
      const uint32_t mine = ((uint32_t)(now.d - 1) << 24) | v;
      uint32_t h = (mine * 0x9E3779B1u) >> (32 - __builtin_ctz(kSlots));   // the product's high bits: a slot
      const uint32_t stride = (mine * 0x85EBCA6Bu) >> 15 | 1u;   // odd: the probes reach every slot
      bool looking = now.alive;
      // (at most three quarters of the slots are taken: with an odd stride a free one is
      // reached within kSlots probes; the bound below is only ever met by a first run that
      // the caller may still hand to the tables)
      const int most = d0 == 1 ? kTabProbes : (int)kSlots;
      for (int probe = 0; probe < most && wave_ballot(looking) != 0; ++probe) {   // uniform
        uint32_t seen = keys[h];
        if (looking && seen == kNoKey) seen = atomicCAS(&keys[h], kNoKey, mine);
        const bool placed = seen == mine || seen == kNoKey;   // there already, or entered just now
        h = (looking && !placed) ? (h + stride) & (kSlots - 1) : h;
        looking = looking && !placed;
      }
      if (now.alive && !looking) {
        atomicAdd(&cell[h], pack_cs(1u, p));
        slot_of[(now.d - d_first) * M + now.mi] = (uint16_t)h;
      }
      failed = failed || looking;
    }
    lds_barrier<kWave>();
    if (wave_ballot(failed) != 0) return false;         // uniform over the wave; first run only
    // ---- walk
    bool ended = false;
    for (int32_t dd = d0; dd <= d_last; ++dd) {
      uint32_t best_hi = 0, best_lo = 0;
      for (int32_t m0 = lane; m0 < M; m0 += kWave) {
        const Match m = s.match[m0];
        if (dd > (int32_t)m.rem_new) continue;
        if (dd > 1 && (keys[slot_of[(dd - 1 - d_first) * M + m0]] & 0xFFFFFFu) != (uint32_t)cur) continue;
        const uint32_t slot = slot_of[(dd - d_first) * M + m0];
        const uint32_t v = keys[slot] & 0xFFFFFFu;
        const u64 packed = ((weight_key(cell[slot], alpha_q) + 1ull) << kTabTokenBits) | (u64)(kTokBits - (v & kTokBits));
        const uint32_t hi = (uint32_t)(packed >> 32), lo = (uint32_t)packed;
        const bool more = hi > best_hi || (hi == best_hi && lo > best_lo);
        best_hi = more ? hi : best_hi;
        best_lo = more ? lo : best_lo;
      }
      const uint32_t top_hi = wave_max(best_hi);
      const uint32_t top_lo = wave_max(best_hi == top_hi ? best_lo : 0u);
      ended = (top_hi | top_lo) == 0u;
      if (ended) break;                                 // leaf: no edge leaves cur
      const u64 top = ((u64)top_hi << 32) | top_lo;
      const Cand chosen{(top >> kTabTokenBits) - 1ull, (int32_t)(kTokBits - ((uint32_t)top & kTokBits))};
      note_choice(o, chosen, dd, lane);
      cur = chosen.v;
    }
    if (ended) break;
    lds_barrier<kWave>();                               // the walk's reads are done before the next clearing
  }
  return true;
}

// ---------------------------------------------------------------- tier 2: streaming

// Token and quantised probability of the d-th continuation token (d >= 1) of a
// match that reaches it: from the match's LDS window if it has one, else from memory.
template <class LDS>
__device__ __forceinline__ void continuation_at(const LDS& s, const Ctx& c, WinInfo wi, int32_t L,
                                                int32_t mi, Match m, int32_t d, uint32_t& v,
                                                uint32_t& p) {
  const int32_t ws = mi;
  if (wi.cached(mi)) {
    const int32_t* win = s.win + ws * 2 * L;
    v = (uint32_t)win[d - 1];
    p = (uint32_t)win[L + d - 1];
  } else {
    int32_t j = c.y.pos_path(m.pos), e = c.y.pos_index(m.pos);
    int32_t old_j = e + (int32_t)m.rel_old;           // exact wherever it decides (see layer_instance)
    v = (uint32_t)c.y.token(j, e + d - 1, old_j);
    p = c.y.prob(j, e + d - 1, old_j);
  }
}

// Same result as tier 1 with bounded memory for any input.  `each_match(f)`
// calls f(Match, index in the LDS match list or -1) for every match (from the
// list, or by matching again); listed matches with a window are read from LDS.
// M (the number of matches) only sizes the table region.
template <int BLOCK, class LDS, class EachMatch>
__device__ __forceinline__ void walk_streaming(LDS& s, const Ctx& c, WinInfo wi, int32_t M, int32_t L,
                                               uint32_t alpha_q, int score_mode, uint32_t* status,
                                               DraftOut& o, EachMatch each_match) {
  uint32_t size = 64;
  while (size < 4u * (uint32_t)M && size < (uint32_t)LDS::kTable) size <<= 1;
  const Region all{0u, size - 1u};
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
        table_clear<BLOCK>(s, size, c.tid);
        block_sync<BLOCK>();
        each_match([&](Match m, int32_t mi) {
          if (s.overflow || d > (int32_t)m.rem_new) return;
          uint32_t u = (uint32_t)c.Q[0], v, p, unused;
          continuation_at(s, c, wi, L, mi, m, d, v, p);
          if (d >= 2) continuation_at(s, c, wi, L, mi, m, d - 1, u, unused);
          if (((v * 0x9E3779B1u) >> 12 & (n_class - 1)) != r) return;
          u64 w = pack_cs(1u, p);
          table_add(s, all, dag_key(d, kAnyTok, v), w);
          if (u == (uint32_t)cur) table_add(s, all, dag_key(d, u, v), w);
        });
        block_sync<BLOCK>();
        if (s.overflow) failed = true;                 // uniform: read after the barrier
        else best = scan_successors<BLOCK>(s, all, d, cur, alpha_q, score_mode, c.tid, best);
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
    note_choice(o, best, d, c.tid);
    cur = best.v;
  }
}

// ---------------------------------------------------------------- tree and list pools
//
// The variants the paper's ablation compares the DAG with.  Both read the same
// candidate pool.  `each_match(f)` calls f(Match, index in the LDS match list
// or -1) for every match.

// Prefix tree: candidates share a node only while ALL their tokens so far are
// equal.  Greedy descent: at depth d the candidates that carry the draft so
// far vote for their next token with Eq. 5's weight; the heaviest child wins
// (ties: lowest token id).  Matches in the LDS list keep an "on the draft so
// far" flag (in s.link, which only the DAG tiers use otherwise); matches that
// are re-found instead of stored compare their whole prefix.  A layer that
// does not fit the table is split into token classes, as in the streaming tier.
template <int BLOCK, class LDS, class EachMatch>
__device__ __forceinline__ void walk_tree(LDS& s, const Ctx& c, WinInfo wi, int32_t M, int32_t L,
                                          uint32_t alpha_q, uint32_t* status, DraftOut& o,
                                          EachMatch each_match) {
  uint32_t size = 64;
  while (size < 4u * (uint32_t)M && size < (uint32_t)LDS::kTable) size <<= 1;
  const Region all{0u, size - 1u};
  for (int32_t m = c.tid; m < M && m < LDS::kMatch; m += BLOCK) s.link[m] = 1;
  int32_t cur = c.Q[0];                               // only labels the table keys of a depth
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
        block_sync<BLOCK>();                           // previous readers are done; flags and chosen[] visible
        table_clear<BLOCK>(s, size, c.tid);
        block_sync<BLOCK>();
        each_match([&](Match m, int32_t mi) {
          if (s.overflow || d > (int32_t)m.rem_new) return;
          uint32_t v, p, before = 0, unused;
          continuation_at(s, c, wi, L, mi, m, d, v, p);
          if (d >= 2) continuation_at(s, c, wi, L, mi, m, d - 1, before, unused);
          bool on = d == 1 || before == (uint32_t)s.chosen[d - 2];
          if (mi >= 0) {
            on = on && s.link[mi] != 0;                // the flag covers depths 1 .. d-2
            s.link[mi] = on ? 1 : 0;                   // now 1 .. d-1 (idempotent over classes)
          } else {
            for (int32_t x = 1; x + 1 < d && on; ++x) {
              continuation_at(s, c, wi, L, mi, m, x, before, unused);
              on = before == (uint32_t)s.chosen[x - 1];
            }
          }
          if (!on || ((v * 0x9E3779B1u) >> 12 & (n_class - 1)) != r) return;
          table_add(s, all, dag_key(d, (uint32_t)cur, v), pack_cs(1u, p));
        });
        block_sync<BLOCK>();
        if (s.overflow) failed = true;                 // uniform: read after the barrier
        else best = scan_successors<BLOCK>(s, all, d, cur, alpha_q, 1, c.tid, best);
      }
      if (failed) ++class_bits;
    } while (failed && class_bits <= kMaxClassBits);
    if (failed) {
      if (c.tid == 0) atomicOr(status, CSD_STATUS_TABLE_FULL);
      break;
    }
    parity ^= 1;
    best = block_argmax<BLOCK>(s, best, c.tid, parity);
    if (best.v == INT_MAX) break;                     // leaf: no candidate goes on
    note_choice(o, best, d, c.tid);
    if (c.tid == 0) s.chosen[d - 1] = best.v;
    cur = best.v;
  }
}

// List: no merging.  The draft is the continuation of the single candidate
// whose tokens' weights (Eq. 5 with one instance each) add up to the most;
// ties go to the first candidate in (path, position) order.
template <int BLOCK, class LDS, class EachMatch>
__device__ __forceinline__ void walk_list(LDS& s, const Ctx& c, WinInfo wi, int32_t L,
                                          uint32_t alpha_q, DraftOut& o, EachMatch each_match) {
  Cand best = cand_none();
  each_match([&](Match m, int32_t mi) {
    int32_t rem = (int32_t)m.rem_new < L ? (int32_t)m.rem_new : L;
    u64 total = 0;
#pragma unroll 4
    for (int32_t d = 1; d <= rem; ++d) {
      uint32_t v, p;
      continuation_at(s, c, wi, L, mi, m, d, v, p);
      total += weight_key(pack_cs(1u, p), alpha_q);
    }
    best = cand_best(best, Cand{total, m.pos});       // packed (path, index): ascending = (j, e) order
  });
  best = block_argmax<BLOCK>(s, best, c.tid, 0);
  if (best.v == INT_MAX) return;
  int32_t j = c.y.pos_path(best.v), e = c.y.pos_index(best.v), old_j, new_j;
  lens_of(s, c.y, j, old_j, new_j);
  int32_t rem = new_j - e < L ? new_j - e : L;
  if (c.tid < rem) {
    o.tok = c.y.token(j, e + c.tid, old_j);
    o.key = weight_key(pack_cs(1u, c.y.prob(j, e + c.tid, old_j)), alpha_q);
  }
  o.key_sum = best.key;
  o.n = rem;
}

// Writes the edge entries of a finished, unscored tier-1 table, sorted by key,
// to ok / ov (debug dump).  Returns through *n_edges (an LDS counter).
template <int BLOCK, class LDS>
__device__ __forceinline__ void emit_sorted_edges(LDS& s, uint32_t n_slots, int tid, int* n_edges,
                                                  u64* ok, u64* ov) {
  for (uint32_t h = tid; h < n_slots; h += BLOCK) {
    u64 key = s.table[h].key;
    if (key == kEmpty || key_u(key) == kAnyTok) continue;
    int rank = 0;                                     // keys are distinct: rank = sorted position
    for (uint32_t g = 0; g < n_slots; ++g) {
      u64 other = s.table[g].key;
      if (other != kEmpty && key_u(other) != kAnyTok && other < key) ++rank;
    }
    ok[rank] = key;
    ov[rank] = s.table[h].val;
    atomicAdd(n_edges, 1);
  }
}

}  // namespace csd
