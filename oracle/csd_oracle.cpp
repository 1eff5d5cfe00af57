/*
 * CPU oracle for consensus draft construction across N parallel sampling
 * paths ("Speculative Decoding for Multi-Sample Inference", Method section,
 * Eq. 3, Eq. 5, the greedy extraction rule, the "Draft acceptance" paragraph
 * and Algorithm 1 of Appendix A).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * statement of what the method computes, written to be checked against the
 * paper by eye.  It shares no code, header, table or helper with the GPU
 * library, and the GPU library never calls it.  Only the tests, the smoke
 * check and the benchmark's CPU-baseline leg may load it.
 *
 * The method is a heuristic defined by its algorithm, so the oracle is the
 * algorithm itself, step by step, in the order of Algorithm 1:
 *   1. take the k-token suffix of path i;
 *   2. scan every other path j for places where that suffix occurs and
 *      collect the tokens that follow (the candidate pool C_t, Eq. 3);
 *   3. build the layered DAG: layer d holds the d-th token after each match,
 *      equal tokens of a layer are one node, and every (u -> v) transition
 *      between consecutive layers accumulates a weight (Eq. 5);
 *   4. walk the layers greedily (the extraction rule after Eq. 5);
 *   5. count how many leading draft tokens equal the verification targets
 *      ("Draft acceptance").
 * Every history is scanned naively for every query; tables are std::map.
 *
 * Readings of the paper taken here (each is also listed in the design notes):
 *  R1  A match must be followed by at least one token, and the continuation
 *      starts at the token AFTER the matched suffix (Introduction: "tokens
 *      immediately following these matches").  0-based: position e of path j
 *      is a match when y_j[e-q .. e-1] equals the query and e < len_j.
 *  R2  Any position of path j's current history qualifies, also beyond
 *      path i's own length (Eq. 3's t' <= t only says "already generated").
 *  R3  q = min(k, len_i); q = 0 gives an empty draft.  Path i itself is
 *      never searched (j != i, Eq. 3) — unless R17 is switched on.
 *  R4  Candidates are a multiset: every (j, e) is one instance of Eq. 5's
 *      sum, even when two continuations hold the same tokens.
 *  R5  p_theta(v_i | u_i) is the probability the model assigned to token v
 *      when it sampled it in path j (supplied by the caller with the token).
 *      It is quantised once to a 16-bit fraction: round-to-nearest-even of
 *      p * 65536, clamped to [0, 65536]; NaN counts as 0.  With no
 *      probabilities supplied every p is 1.
 *  R6  Freq(u -> v) is the raw count of instances with u in layer d-1 and v
 *      in layer d.
 *  R7  All weights are exact integers: with alpha_q = round(alpha * 65536),
 *      a count C and a probability sum S (in 1/65536 units) give
 *      key = alpha_q * S + (65536 - alpha_q) * (C << 16) = weight * 2^32.
 *  R8  The greedy step picks, among the successors v of the current node
 *      (edges (cur, v) of layer d), the one whose weight is largest; the
 *      weight is the node in-weight  sum over u of w(u, v)  (score_mode 0,
 *      the paper's formula) or the single edge weight w(cur, v)
 *      (score_mode 1).  Ties go to the lowest token id.  The walk stops at L
 *      tokens or when the current node has no successor (leaf / empty DAG).
 *  R9  The predecessor of a layer-1 token is the last query token.
 *  R10 token_score[d] = key / 2^32 as float, path_score = (sum of keys)/2^32.
 *  R11 Accept length = number of leading draft tokens equal to the targets,
 *      in [0, draft_len]; no bonus token (Table 1's values never exceed L).
 *  R12 Fuzzy suffix matching (Eq. 4), tolerance eps >= 0: position e of path j
 *      (0 <= e < len_j) is a match when SOME substring of path j that ends just
 *      before e, of any length l with l <= e, is within Levenshtein distance
 *      eps of the query (unit costs for substitution, insertion, deletion).
 *      Only lengths q-eps .. q+eps can qualify.  Each e counts once, however
 *      many substrings qualify.  eps = 0 is the exact match of Eq. 3.
 *  R13 With eps > 0 the token before a match need not be the last query token,
 *      so the DAG's root is the query itself: the predecessor of EVERY
 *      layer-1 token is the last query token (for eps = 0 this is R9).
 *  R14 Tree pool (pool_mode 1; the ablation's "tree", which the paper names
 *      but does not define): the candidates' continuations form a prefix
 *      tree — candidates share a node as long as ALL their tokens so far are
 *      equal, not just the last one as in the DAG.  A child's weight is
 *      Eq. 5's weight over the candidates that pass through it.  The draft
 *      descends from the root to the heaviest child (ties: lowest token id)
 *      until L tokens or a leaf.  score_mode does not apply.
 *  R15 List pool (pool_mode 2; the ablation's "list"): the candidates are
 *      not merged at all.  The draft is the continuation (at most L tokens)
 *      of ONE candidate: the one whose tokens' weights — Eq. 5 with a single
 *      instance each, alpha*p + (1-alpha)*1 — add up to the most; ties go to
 *      the first candidate in (path, position) order.  token_score is each
 *      token's own weight.  score_mode does not apply.
 *  R17 Self-history (not in the paper; retrieval / prompt-lookup style
 *      drafting; `extras` bit 0): path i's own history is searched like any
 *      other path's.  The occurrence of the query at the very end of path i
 *      has no successor and is therefore no match (R1).
 *  R18 Query back-off (not in the paper; `extras` bit 1): if the q-token query
 *      has no match, the query is shortened by its OLDEST token, down to one
 *      token, until its match set is non-empty; the draft is built from the
 *      first non-empty set.  No length with a match: empty draft.
 *
 * Threads.  oracle_draft_many runs the drafts of many independent
 * (history state, problem, path) rows on several host threads; each row is
 * one call of oracle_draft, whose arithmetic is untouched (the rows share
 * nothing but read-only inputs, so the result does not depend on the number
 * of threads: a CPU test compares it with the serial loop bit for bit).
 *
 * Build: g++ -O2 -pthread -shared -fPIC -o libcsd_oracle.so csd_oracle.cpp
 */
#include <atomic>
#include <cmath>
#include <cstdint>
#include <map>
#include <thread>
#include <utility>
#include <vector>

namespace {

struct Weight {            /* one DAG edge or node: Eq. 5's two sums */
  uint64_t C = 0;          /* Freq: number of instances              */
  uint64_t S = 0;          /* sum of quantised probabilities         */
};

struct Candidate {         /* one element of the pool C_t (Eq. 3)    */
  int32_t j;               /* path it was found in                   */
  int32_t e;               /* index of its first continuation token  */
};

/* R5: probability -> integer in [0, 65536]. */
uint32_t quantize_prob(float p) {
  if (std::isnan(p)) return 0;
  double x = std::nearbyint(static_cast<double>(p) * 65536.0); /* half-even */
  if (x < 0.0) x = 0.0;
  if (x > 65536.0) x = 65536.0;
  return static_cast<uint32_t>(x);
}

/* One problem's histories: tok[j*max_len + t], prob likewise (may be null). */
struct Paths {
  const int32_t* tok;
  const float* prob;
  const int32_t* len;
  int32_t N;
  int32_t max_len;
  int32_t token(int32_t j, int32_t t) const { return tok[(int64_t)j * max_len + t]; }
  uint32_t pq(int32_t j, int32_t t) const {
    return prob ? quantize_prob(prob[(int64_t)j * max_len + t]) : 65536u;
  }
};

/* Levenshtein distance between a[0..na) and b[0..nb): the textbook dynamic
 * programme over the (na+1) x (nb+1) table, unit costs. */
int32_t edit_distance(const int32_t* a, int32_t na, const int32_t* b, int32_t nb) {
  std::vector<std::vector<int32_t> > D(na + 1, std::vector<int32_t>(nb + 1, 0));
  for (int32_t x = 0; x <= na; ++x) D[x][0] = x;
  for (int32_t y = 0; y <= nb; ++y) D[0][y] = y;
  for (int32_t x = 1; x <= na; ++x)
    for (int32_t y = 1; y <= nb; ++y) {
      int32_t best = D[x - 1][y - 1] + (a[x - 1] != b[y - 1] ? 1 : 0);   /* substitute / keep */
      if (D[x - 1][y] + 1 < best) best = D[x - 1][y] + 1;                /* delete from a     */
      if (D[x][y - 1] + 1 < best) best = D[x][y - 1] + 1;                /* insert into a     */
      D[x][y] = best;
    }
  return D[na][nb];
}

/* Algorithm 1, the search loop (Eq. 3, with Eq. 4's tolerance): the candidate
 * pool of path i. */
std::vector<Candidate> candidate_pool(const Paths& Y, int32_t i, int32_t k, int32_t eps,
                                      bool include_self, int32_t* q_out) {
  std::vector<Candidate> pool;
  int32_t len_i = Y.len[i];
  int32_t q = k < len_i ? k : len_i;                       /* R3 */
  *q_out = q;
  if (q <= 0) return pool;
  const int32_t* query = Y.tok + (int64_t)i * Y.max_len + (len_i - q);
  for (int32_t j = 0; j < Y.N; ++j) {
    if (j == i && !include_self) continue;                 /* R3; R17 */
    const int32_t* yj = Y.tok + (int64_t)j * Y.max_len;
    for (int32_t e = 0; e <= Y.len[j] - 1; ++e) {          /* R1, R2 */
      bool match = false;
      if (eps == 0) {
        /* Eq. 3 as it stands: the q tokens before e are the query (distance 0 is equality) */
        match = e >= q;
        for (int32_t a = 0; a < q && match; ++a) match = yj[e - q + a] == query[a];
      } else {
        /* R12: substrings ending before e; |l - q| <= distance, so only these lengths can do */
        for (int32_t l = (q > eps ? q - eps : 0); l <= q + eps && l <= e && !match; ++l)
          if (edit_distance(query, q, yj + (e - l), l) <= eps) match = true;
      }
      if (match) pool.push_back(Candidate{j, e});
    }
  }
  return pool;                                             /* ascending (j, e) */
}

/* The pool a draft is built from: that of the k-token query, or with back-off
 * (R18) that of the longest shorter query that has one. */
std::vector<Candidate> pool_for_draft(const Paths& Y, int32_t i, int32_t k, int32_t eps,
                                      int32_t extras) {
  const bool include_self = (extras & 1) != 0, back_off = (extras & 2) != 0;
  int32_t q;
  std::vector<Candidate> pool = candidate_pool(Y, i, k, eps, include_self, &q);
  if (back_off)
    for (int32_t shorter = q - 1; pool.empty() && shorter >= 1; --shorter)
      pool = candidate_pool(Y, i, shorter, eps, include_self, &q);
  return pool;
}

typedef std::map<std::pair<int32_t, int32_t>, Weight> EdgeTable;   /* (u, v) -> weight */

/* Algorithm 1, DAG construction (Eq. 5): edges[d-1] is the table of layer d. */
std::vector<EdgeTable> build_dag(const Paths& Y, const std::vector<Candidate>& pool, int32_t L,
                                 int32_t root) {
  std::vector<EdgeTable> edges(L > 0 ? L : 0);
  for (int32_t d = 1; d <= L; ++d) {
    for (const Candidate& c : pool) {
      int32_t t = c.e + d - 1;                 /* d-th token after the match */
      if (t >= Y.len[c.j]) continue;           /* this candidate has ended   */
      int32_t u = d == 1 ? root : Y.token(c.j, t - 1);   /* R9, R13 */
      int32_t v = Y.token(c.j, t);
      Weight& w = edges[d - 1][std::make_pair(u, v)];
      w.C += 1;                                /* R4, R6 */
      w.S += Y.pq(c.j, t);                     /* R5     */
    }
  }
  return edges;
}

uint64_t weight_key(const Weight& w, uint32_t alpha_q) {   /* R7 */
  return (uint64_t)alpha_q * w.S + (uint64_t)(65536u - alpha_q) * (w.C << 16);
}

}  // namespace

extern "C" {

uint32_t oracle_quantize_prob(float p) { return quantize_prob(p); }

/* Levenshtein distance of two token strings (R12), exposed so that it can be pinned. */
int32_t oracle_edit_distance(const int32_t* a, int32_t na, const int32_t* b, int32_t nb) {
  return edit_distance(a, na, b, nb);
}

/* alpha in [0,1] -> alpha_q in [0, 65536] (R7). */
uint32_t oracle_alpha_q(double alpha) {
  double x = std::nearbyint(alpha * 65536.0);
  if (x < 0.0) x = 0.0;
  if (x > 65536.0) x = 65536.0;
  return (uint32_t)x;
}

/* Match set of path i (Eq. 3) as (j, e) rows in ascending order.  Returns the
 * number of matches; writes at most cap rows. */
int64_t oracle_matches(const int32_t* tok, const int32_t* len, int32_t N, int32_t max_len,
                       int32_t i, int32_t k, int32_t eps, int32_t extras, int32_t* out_je,
                       int64_t cap) {
  Paths Y{tok, nullptr, len, N, max_len};
  int32_t q;
  std::vector<Candidate> pool = candidate_pool(Y, i, k, eps, (extras & 1) != 0, &q);
  for (int64_t m = 0; m < (int64_t)pool.size() && m < cap; ++m) {
    out_je[2 * m] = pool[m].j;
    out_je[2 * m + 1] = pool[m].e;
  }
  return (int64_t)pool.size();
}

/* Edge tables of path i's DAG (Eq. 5) as rows (d, u, v) / (C, S) sorted by
 * (d, u, v).  Returns the number of rows; writes at most cap rows. */
int64_t oracle_edges(const int32_t* tok, const float* prob, const int32_t* len, int32_t N,
                     int32_t max_len, int32_t i, int32_t k, int32_t eps, int32_t extras, int32_t L,
                     int32_t* out_duv, uint64_t* out_cs, int64_t cap) {
  Paths Y{tok, prob, len, N, max_len};
  int32_t q;
  std::vector<Candidate> pool = candidate_pool(Y, i, k, eps, (extras & 1) != 0, &q);
  /* R9: the root is the last query token; an empty path has no query, no pool and no edges */
  int32_t root = Y.len[i] > 0 ? Y.token(i, Y.len[i] - 1) : 0;
  std::vector<EdgeTable> edges = build_dag(Y, pool, L, root);
  int64_t n = 0;
  for (int32_t d = 1; d <= L; ++d) {
    for (const auto& kv : edges[d - 1]) {
      if (n < cap) {
        out_duv[3 * n] = d;
        out_duv[3 * n + 1] = kv.first.first;
        out_duv[3 * n + 2] = kv.first.second;
        out_cs[2 * n] = kv.second.C;
        out_cs[2 * n + 1] = kv.second.S;
      }
      ++n;
    }
  }
  return n;
}

typedef std::vector<std::pair<int32_t, uint64_t> > Draft;   /* (token, key) per layer */

/* The greedy extraction rule after Eq. 5 on the layered DAG (R8, R9, R13). */
Draft draft_from_dag(const Paths& Y, const std::vector<Candidate>& pool, int32_t L, int32_t root,
                     uint32_t alpha_q, int32_t score_mode) {
  std::vector<EdgeTable> edges = build_dag(Y, pool, L, root);
  Draft out;
  int32_t cur = root;
  for (int32_t d = 1; d <= L; ++d) {
    const EdgeTable& E = edges[d - 1];
    /* node in-weights of this layer: sum over all predecessors u (R8) */
    std::map<int32_t, Weight> node;
    for (const auto& kv : E) {
      Weight& w = node[kv.first.second];
      w.C += kv.second.C;
      w.S += kv.second.S;
    }
    bool found = false;
    int32_t best_v = 0;
    uint64_t best_key = 0;
    for (const auto& kv : E) {                   /* ascending (u, v) */
      if (kv.first.first != cur) continue;       /* successors of cur only */
      int32_t v = kv.first.second;
      uint64_t key = weight_key(score_mode == 0 ? node[v] : kv.second, alpha_q);
      if (!found || key > best_key) {            /* strict > keeps the lowest id on ties */
        found = true;
        best_v = v;
        best_key = key;
      }
    }
    if (!found) break;                           /* leaf, or the layer is empty */
    out.push_back(std::make_pair(best_v, best_key));
    cur = best_v;
  }
  return out;
}

/* R14: greedy descent of the candidates' prefix tree.  `here` holds the
 * candidates that pass through the current tree node. */
Draft draft_from_tree(const Paths& Y, const std::vector<Candidate>& pool, int32_t L,
                      uint32_t alpha_q) {
  Draft out;
  std::vector<Candidate> here = pool;            /* the root: every candidate */
  for (int32_t d = 1; d <= L; ++d) {
    std::map<int32_t, Weight> child;             /* token -> weight of that child */
    for (const Candidate& c : here) {
      int32_t t = c.e + d - 1;
      if (t >= Y.len[c.j]) continue;             /* this candidate has ended */
      Weight& w = child[Y.token(c.j, t)];
      w.C += 1;
      w.S += Y.pq(c.j, t);
    }
    bool found = false;
    int32_t best_v = 0;
    uint64_t best_key = 0;
    for (const auto& kv : child) {               /* ascending token id */
      uint64_t key = weight_key(kv.second, alpha_q);
      if (!found || key > best_key) {
        found = true;
        best_v = kv.first;
        best_key = key;
      }
    }
    if (!found) break;                           /* leaf */
    out.push_back(std::make_pair(best_v, best_key));
    std::vector<Candidate> below;
    for (const Candidate& c : here)
      if (c.e + d - 1 < Y.len[c.j] && Y.token(c.j, c.e + d - 1) == best_v) below.push_back(c);
    here = below;
  }
  return out;
}

/* R15: the single heaviest candidate of the unmerged list. */
Draft draft_from_list(const Paths& Y, const std::vector<Candidate>& pool, int32_t L,
                      uint32_t alpha_q) {
  bool found = false;
  uint64_t best_total = 0;
  Draft best;
  for (const Candidate& c : pool) {              /* ascending (j, e) */
    Draft mine;
    uint64_t total = 0;
    for (int32_t d = 1; d <= L && c.e + d - 1 < Y.len[c.j]; ++d) {
      Weight w;
      w.C = 1;
      w.S = Y.pq(c.j, c.e + d - 1);
      mine.push_back(std::make_pair(Y.token(c.j, c.e + d - 1), weight_key(w, alpha_q)));
      total += weight_key(w, alpha_q);
    }
    if (!found || total > best_total) {          /* strict >: the first candidate wins ties */
      found = true;
      best_total = total;
      best = mine;
    }
  }
  return best;
}

/* Draft of path i (Algorithm 1 as a whole) from the pool organised as a DAG
 * (pool_mode 0, the method), a prefix tree (1) or a list (2).  draft[L] is
 * padded with -1, token_scores[L] with 0.  Returns the draft length. */
int32_t oracle_draft(const int32_t* tok, const float* prob, const int32_t* len, int32_t N,
                     int32_t max_len, int32_t i, int32_t k, int32_t eps, int32_t L, uint32_t alpha_q,
                     int32_t score_mode, int32_t pool_mode, int32_t extras, int32_t* draft,
                     float* token_scores, float* path_score) {
  for (int32_t d = 0; d < L; ++d) { draft[d] = -1; token_scores[d] = 0.0f; }
  *path_score = 0.0f;
  Paths Y{tok, prob, len, N, max_len};
  std::vector<Candidate> pool = pool_for_draft(Y, i, k, eps, extras);
  if (pool.empty()) return 0;
  int32_t root = Y.token(i, Y.len[i] - 1);       /* R9: root = last query token */
  Draft chosen = pool_mode == 1 ? draft_from_tree(Y, pool, L, alpha_q)
               : pool_mode == 2 ? draft_from_list(Y, pool, L, alpha_q)
                                : draft_from_dag(Y, pool, L, root, alpha_q, score_mode);
  uint64_t key_sum = 0;
  int32_t n = 0;
  for (const auto& tk : chosen) {
    draft[n] = tk.first;
    token_scores[n] = (float)((double)tk.second / 4294967296.0);   /* R10 */
    key_sum += tk.second;
    ++n;
  }
  *path_score = (float)((double)key_sum / 4294967296.0);
  return n;
}

/* "Draft acceptance": length of the longest draft prefix equal to the targets (R11). */
int32_t oracle_accept(const int32_t* draft, int32_t draft_len, const int32_t* target) {
  int32_t a = 0;
  while (a < draft_len && draft[a] == target[a]) ++a;
  return a;
}

/* Convenience loop used for replays and for timing: every path of every
 * problem.  Arrays are [P][N][...]; target / accept_len may be null. */
void oracle_draft_all(const int32_t* tok, const float* prob, const int32_t* len, int32_t P,
                      int32_t N, int32_t max_len, int32_t k, int32_t eps, int32_t L,
                      uint32_t alpha_q, int32_t score_mode, int32_t pool_mode, int32_t extras,
                      int32_t* draft, int32_t* draft_len, float* token_scores, float* path_scores,
                      const int32_t* target, int32_t* accept_len) {
  for (int32_t p = 0; p < P; ++p) {
    const int32_t* tk = tok + (int64_t)p * N * max_len;
    const float* pr = prob ? prob + (int64_t)p * N * max_len : nullptr;
    const int32_t* ln = len + (int64_t)p * N;
    for (int32_t i = 0; i < N; ++i) {
      int64_t r = (int64_t)p * N + i;
      draft_len[r] = oracle_draft(tk, pr, ln, N, max_len, i, k, eps, L, alpha_q, score_mode,
                                  pool_mode, extras, draft + r * L, token_scores + r * L,
                                  path_scores + r);
      if (target && accept_len)
        accept_len[r] = oracle_accept(draft + r * L, draft_len[r], target + r * L);
    }
  }
}

/* The same over S independent history states of one path set (the states of a
 * replay: len [S][P][N] says how much of each path exists in state s), on
 * n_threads host threads.  Rows (s, p, i) are handed out one at a time; each
 * is one oracle_draft (+ oracle_accept) call, exactly as in oracle_draft_all.
 * Outputs are [S][P][N][...]; target [S][P][N][L] and accept_len may be null.
 * n_threads <= 1: a plain serial loop on the calling thread. */
void oracle_draft_many(const int32_t* tok, const float* prob, const int32_t* len, int32_t S, int32_t P,
                       int32_t N, int32_t max_len, int32_t k, int32_t eps, int32_t L, uint32_t alpha_q,
                       int32_t score_mode, int32_t pool_mode, int32_t extras, int32_t n_threads,
                       int32_t* draft, int32_t* draft_len, float* token_scores, float* path_scores,
                       const int32_t* target, int32_t* accept_len) {
  const int64_t rows = (int64_t)P * N, items = (int64_t)S * rows;
  auto one_row = [&](int64_t x) {
    const int64_t s = x / rows, r = x % rows;
    const int32_t p = (int32_t)(r / N), i = (int32_t)(r % N);
    const int32_t* tk = tok + (int64_t)p * N * max_len;
    const float* pr = prob ? prob + (int64_t)p * N * max_len : nullptr;
    const int32_t* ln = len + s * rows + (int64_t)p * N;
    draft_len[x] = oracle_draft(tk, pr, ln, N, max_len, i, k, eps, L, alpha_q, score_mode, pool_mode,
                                extras, draft + x * L, token_scores + x * L, path_scores + x);
    if (target && accept_len) accept_len[x] = oracle_accept(draft + x * L, draft_len[x], target + x * L);
  };
  if (n_threads <= 1) {
    for (int64_t x = 0; x < items; ++x) one_row(x);
    return;
  }
  std::atomic<int64_t> next(0);
  auto worker = [&]() {
    for (int64_t x = next.fetch_add(1); x < items; x = next.fetch_add(1)) one_row(x);
  };
  std::vector<std::thread> pool;
  for (int32_t t = 1; t < n_threads; ++t) pool.emplace_back(worker);
  worker();
  for (std::thread& t : pool) t.join();
}

/* The propose / verify / accept loop of speculative decoding (Background
 * section; "Draft acceptance") around the draft construction, with a stand-in
 * for the model: what the model samples for path i is that path's own future,
 * future_tok[p][i][...].  Every step, every path first appends the tokens the
 * previous step settled — the accepted draft tokens plus the one token the
 * model emits itself (1 token at the first step), clipped at max_len — then
 * drafts from the pool of all paths, and its draft is checked against its
 * next L future tokens (-1 beyond the end never matches).  len [P][N] holds the
 * lengths on entry and on exit; outputs are [n_steps][P][N][...]. */
void oracle_accept_loop(const int32_t* future_tok, const float* future_prob, int32_t* len, int32_t P,
                        int32_t N, int32_t max_len, int32_t k, int32_t eps, int32_t L,
                        uint32_t alpha_q, int32_t score_mode, int32_t pool_mode, int32_t extras,
                        int32_t n_steps, int32_t* draft, int32_t* draft_len, int32_t* accept_len,
                        int32_t* path_len) {
  int64_t rows = (int64_t)P * N;
  std::vector<int32_t> settled(rows, 0);          /* accept length of the previous step */
  std::vector<int32_t> target(L > 0 ? L : 0);
  for (int32_t s = 0; s < n_steps; ++s) {
    for (int64_t r = 0; r < rows; ++r) {          /* append phase: all paths */
      int32_t grow = settled[r] + 1;
      if (grow > max_len - len[r]) grow = max_len - len[r];
      len[r] += grow;
      path_len[s * rows + r] = len[r];
    }
    for (int32_t p = 0; p < P; ++p) {             /* draft + acceptance phase */
      const int32_t* tk = future_tok + (int64_t)p * N * max_len;
      const float* pr = future_prob ? future_prob + (int64_t)p * N * max_len : nullptr;
      const int32_t* ln = len + (int64_t)p * N;
      for (int32_t i = 0; i < N; ++i) {
        int64_t r = (int64_t)p * N + i;
        int64_t o = s * rows + r;
        float unused_scores[64], unused_total;
        draft_len[o] = oracle_draft(tk, pr, ln, N, max_len, i, k, eps, L, alpha_q, score_mode,
                                    pool_mode, extras, draft + o * L, unused_scores, &unused_total);
        for (int32_t d = 0; d < L; ++d)
          target[d] = ln[i] + d < max_len ? tk[(int64_t)i * max_len + ln[i] + d] : -1;
        accept_len[o] = oracle_accept(draft + o * L, draft_len[o], target.data());
        settled[r] = accept_len[o];
      }
    }
  }
}

}  /* extern "C" */
