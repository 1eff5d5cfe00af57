/*
 * csd — consensus speculative drafting across N parallel sampling paths.
 *
 * C-ABI boundary of the MI355X (gfx950) library.  The operations follow the
 * problem statement of "Speculative Decoding for Multi-Sample Inference"
 * (Method section and Algorithm 1 of Appendix A): keep the token histories of
 * N parallel sampling paths (the "dynamic draft pool"), and at every decoding
 * step produce, for every path, a draft of up to L tokens by
 *   (1) matching the path's last k tokens against every OTHER path's history
 *       (Eq. 3),
 *   (2) merging the tokens that follow the matches into a layered token DAG
 *       whose edges carry  w(u,v) = alpha * sum_i p(v_i|u_i)
 *                                   + (1 - alpha) * Freq(u -> v)      (Eq. 5),
 *   (3) walking the layers greedily by largest weight (rule after Eq. 5),
 * and then measuring how many leading draft tokens equal the tokens the
 * target model sampled ("Draft acceptance" paragraph).
 *
 * Conventions
 *  - P problems are independent; each has N paths of at most max_len tokens.
 *  - Every pointer named d_* is DEVICE memory owned by the caller.  Arrays are
 *    dense row-major with the shape given in brackets.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Every call except csd_status / csd_dump_* only enqueues work on `stream`
 *    and returns; nothing is allocated, freed or synchronised by them.
 *  - The library owns only the small host-side handle.  All device state lives
 *    in the caller's workspace, which must stay allocated, and untouched by
 *    the caller, until csd_destroy.
 *  - All functions return CSD_OK (0) or a negative csd_error.  On an error
 *    of a single-step call (csd_append, csd_draft, csd_accept, csd_step)
 *    nothing has been enqueued and the handle is as it was.  The multi-step
 *    calls (csd_replay, csd_accept_loop) check all arguments before the first
 *    launch; a CSD_ERR_HIP from a later launch leaves the earlier steps
 *    enqueued.  A handle is not thread-safe.
 *  - Token ids must lie in [0, vocab).  Ids outside are a caller error: the
 *    append kernel raises CSD_STATUS_TOKEN_RANGE (see csd_status); drafts that
 *    involve such ids are memory-safe but unspecified.
 *
 * Exactness.  Probabilities are quantised once at append to multiples of
 * 1/65536 (round to nearest even, clamped to [0,1], NaN -> 0); alpha likewise.
 * All sums are exact 64-bit integers, so every output is independent of the
 * order in which the GPU accumulates: draft tokens, lengths and accept lengths
 * are exact, and scores are the exact rational weight rounded once to float.
 */
#ifndef CSD_H_
#define CSD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct csd_index csd_index; /* opaque, host-side, library-owned */

typedef enum {
  CSD_OK = 0,
  CSD_ERR_INVALID_ARG = -1,   /* NULL pointer, dimension or argument out of range     */
  CSD_ERR_CAPACITY = -2,      /* append would exceed max_len / dump buffer too small  */
  CSD_ERR_WORKSPACE = -3,     /* workspace too small or misaligned (needs 256 B)      */
  CSD_ERR_HIP = -4,           /* a HIP runtime call failed                            */
  CSD_ERR_UNIMPLEMENTED = -5, /* unknown flag bits, or a configuration this build
                                 does not implement (max_edits > 1, ...)              */
  CSD_ERR_SCRATCH_LIMIT = -6  /* csd_accept_loop_noalloc: the input needs more scratch
                                 memory than the library's fixed array holds          */
} csd_error;

/* Limits of this build (csd_create rejects configurations beyond them). */
#define CSD_MAX_QUERY_LEN 8
#define CSD_MAX_DRAFT_LEN 32
#define CSD_MAX_EDITS 3             /* largest edit tolerance of the suffix match (Eq. 4) */
#define CSD_MAX_VOCAB ((1 << 29) - 1)
#define CSD_MAX_POSITIONS (1 << 24) /* n_paths * max_len per problem */
#define CSD_MAX_STEP_TOKENS 32767   /* csd_step: tokens per path per call */

/* csd_config.flags: how matches are found (Eq. 3).  Both give identical results. */
#define CSD_MATCH_AUTO 0   /* library picks                                         */
#define CSD_POOL_DAG 0
#define CSD_POOL_TREE 1
#define CSD_POOL_LIST 2

#define CSD_MATCH_SCAN 1   /* compare the query against every history position      */
#define CSD_MATCH_INDEX 2  /* look the query up in the incremental n-gram hash index, which
                              holds grams of max_query_len tokens: set max_query_len to the
                              query_len the decode loop uses; shorter queries are scanned */

/* csd_config.flags, options that may be OR-ed to a CSD_MATCH_* value.  Neither is in the
 * paper; they are what retrieval-style drafting from a single sequence does. */
#define CSD_INCLUDE_SELF 4   /* path i's own history is searched like any other path's
                                (the query's own occurrence at the end of path i has no
                                successor and never counts)                             */
#define CSD_QUERY_BACKOFF 8  /* a query without matches is shortened by its oldest token,
                                down to one token, until it has some; the draft is built
                                from the first non-empty match set.  Shortened queries are
                                always scanned: CSD_MATCH_AUTO picks the scan with this.  */

/* Sticky device-side status bits, read with csd_status. */
#define CSD_STATUS_CAPACITY 1u     /* an append was clipped at max_len               */
#define CSD_STATUS_TOKEN_RANGE 2u  /* a token id outside [0, vocab) was appended     */
#define CSD_STATUS_TABLE_FULL 4u   /* a draft was cut short: DAG tables exhausted.
                                      Cannot happen with vocab <= 2^24, whatever the
                                      input.  The bounded-memory tier splits a layer's
                                      tokens into up to 2^20 classes by bits 12..31 of
                                      id * 0x9E3779B1 mod 2^32; at most 65 ids below 2^24
                                      (2045 below 2^29) share a class, and the smallest
                                      on-chip table holds 256 keys (two per id).  Beyond
                                      2^24 it takes a layer whose continuation tokens
                                      include more than 128 distinct ids of ONE class
                                      (512 with fewer than 2048 rows per launch): only a
                                      constructed input does that.  The draft then ends
                                      before that layer; everything else stays exact.   */

typedef struct {
  int32_t n_problems;     /* P > 0                                                    */
  int32_t n_paths;        /* N > 0                                                    */
  int32_t max_len;        /* tokens per path, > 0; N * max_len <= CSD_MAX_POSITIONS   */
  int32_t vocab;          /* V in [1, CSD_MAX_VOCAB]                                  */
  int32_t max_query_len;  /* upper bound of csd_draft's query_len, 1..CSD_MAX_QUERY_LEN */
  int32_t max_draft_len;  /* upper bound of csd_draft's draft_len, 1..CSD_MAX_DRAFT_LEN */
  float alpha;            /* Eq. 5's alpha in [0,1]; the paper's experiments use 1    */
  int32_t score_mode;     /* 0: greedy step ranks successors by node in-weight
                             sum_u w(u,v) (the rule after Eq. 5); 1: by w(cur,v)      */
  int32_t flags;          /* one CSD_MATCH_* value, optionally | CSD_INCLUDE_SELF and/or
                             | CSD_QUERY_BACKOFF; all other bits must be 0            */
  int32_t max_edits;      /* Eq. 4's edit-distance tolerance eps of the suffix match, in
                             [0, CSD_MAX_EDITS]: 0 = exact (Eq. 3), 1 = one substitution,
                             insertion or deletion (the paper's experiments use 1), 2 and
                             3 likewise (Levenshtein distance; always matched by scan:
                             CSD_ERR_UNIMPLEMENTED with CSD_MATCH_INDEX).  A position e of
                             another path matches when some substring ending just before
                             e is within eps edits of the query, each e counting once (a
                             query of at most eps tokens matches everywhere).  One-edit
                             matches are found by scan, or through the index, which then
                             files every position under the max_query_len + 1 variants
                             of its gram (the gram itself and the gram without one of its
                             tokens): CSD_MATCH_AUTO takes the index from max_query_len 4
                             on if there are more than 128 rows (problem, path) or a
                             problem has 2^14 positions (n_paths * max_len) or more, else
                             the scan; CSD_MATCH_INDEX takes it from max_query_len 2 on
                             (1: CSD_ERR_UNIMPLEMENTED).                                 */
  int32_t pool_mode;      /* how the candidate pool is organised before the greedy
                             extraction: CSD_POOL_DAG (the method: equal tokens of a layer
                             are one node, Eq. 5), CSD_POOL_TREE (prefix tree: candidates
                             share a node only while all their tokens so far are equal; a
                             child's weight is Eq. 5's over the candidates through it) or
                             CSD_POOL_LIST (no merging: the continuation of the single
                             candidate whose tokens' weights alpha*p + (1-alpha) add up to
                             the most, ties to the first in (path, position) order).
                             TREE and LIST are the variants the paper's ablation compares
                             the DAG with; score_mode does not apply to them.          */
} csd_config;

/* Size in bytes of the device workspace csd_create needs for this config. */
int csd_workspace_bytes(const csd_config* cfg, size_t* out_bytes);

/* Creates an index (the draft pool of the Method section, "Dynamic Draft Pool
 * Construction") over P x N empty paths inside d_workspace (256-byte aligned,
 * at least csd_workspace_bytes) and enqueues its initialisation on `stream`. */
int csd_create(const csd_config* cfg, void* d_workspace, size_t workspace_bytes, void* stream,
               csd_index** out_index);

/* Frees the host handle.  Does not touch the workspace. */
int csd_destroy(csd_index* index);

/* Empties every path (same state as after csd_create). */
int csd_reset(csd_index* index, void* stream);

/* Appends up to n tokens to every path: the pool "iteratively" grows with the
 * generation (Method, "Dynamic Draft Pool Construction").
 *   d_tokens [P][N][n] int32  tokens sampled this step, oldest first.
 *   d_probs  [P][N][n] float  probability the model gave each of them when it
 *                             sampled it (Eq. 5's p_theta); NULL = all 1.
 *   d_counts [P][N]    int32  how many of the n tokens path (p,i) really takes
 *                             (clamped to [0,n]); NULL = n for every path.
 * CSD_ERR_CAPACITY if the host can tell that a path would exceed max_len
 * (always the case with d_counts == NULL); with d_counts the kernel clips the
 * append at max_len and raises CSD_STATUS_CAPACITY. */
int csd_append(csd_index* index, const int32_t* d_tokens, const float* d_probs,
               const int32_t* d_counts, int32_t n, void* stream);

/* Builds the draft of every path (Algorithm 1): suffix match of the last
 * q = min(query_len, len_i) tokens against all other paths (Eq. 3), DAG edge
 * weights (Eq. 5), greedy walk of at most draft_len layers.
 *   d_draft_tokens [P][N][draft_len] int32  draft, padded with -1.
 *   d_draft_len    [P][N]            int32  number of draft tokens (0 = no match).
 *   d_token_scores [P][N][draft_len] float  weight of each chosen token, padded
 *                                           with 0; may be NULL.
 *   d_path_scores  [P][N]            float  sum of those weights; may be NULL.
 * query_len in [1, max_query_len], draft_len in [1, max_draft_len]. */
int csd_draft(csd_index* index, int32_t query_len, int32_t draft_len, int32_t* d_draft_tokens,
              int32_t* d_draft_len, float* d_token_scores, float* d_path_scores, void* stream);

/* Greedy accept length ("Draft acceptance"): for every path the number of
 * leading draft tokens equal to the target tokens, in [0, draft_len[p][i]].
 *   d_targets    [P][N][draft_len] int32  tokens the target model sampled.
 *   d_accept_len [P][N]            int32  output. */
int csd_accept(csd_index* index, const int32_t* d_draft_tokens, const int32_t* d_draft_len,
               const int32_t* d_targets, int32_t draft_len, int32_t* d_accept_len, void* stream);

/* One decoding step in ONE launch (two with the index matcher when n > 64, or n > 1
 * with one-edit matching):
 * csd_append(d_tokens, d_probs, d_counts, n),
 * then csd_draft(query_len, draft_len, ...) on the grown paths, then, if
 * d_targets is given, csd_accept of the fresh drafts (Algorithm 1 run at step t
 * of the generation, followed by the check of "Draft acceptance").  Results are
 * identical to the three separate calls.  Arguments as in those calls;
 * d_targets and d_accept_len are both NULL or both non-NULL; n in
 * [1, CSD_MAX_STEP_TOKENS].  Consecutive calls on one index must be enqueued
 * on the same stream (or be ordered by the caller). */
int csd_step(csd_index* index, const int32_t* d_tokens, const float* d_probs,
             const int32_t* d_counts, int32_t n, int32_t query_len, int32_t draft_len,
             int32_t* d_draft_tokens, int32_t* d_draft_len, float* d_token_scores,
             float* d_path_scores, const int32_t* d_targets, int32_t* d_accept_len, void* stream);

/* n_steps consecutive decoding steps with one token per path and step, issued
 * from a host loop inside the library (no device-side loop): step t appends
 * d_tokens[t] (with d_probs[t], may be NULL), drafts into slice t of the
 * outputs and, if d_targets is given, checks slice t of it.
 *   d_tokens [n_steps][P][N], d_probs same; d_draft_tokens [n_steps][P][N][draft_len],
 *   d_draft_len [n_steps][P][N], d_token_scores / d_path_scores likewise or NULL,
 *   d_targets [n_steps][P][N][draft_len] and d_accept_len [n_steps][P][N] or both NULL.
 * fused != 0: one csd_step launch per step; fused == 0: csd_append, csd_draft
 * and csd_accept launches per step.  Both give identical results. */
int csd_replay(csd_index* index, int32_t n_steps, const int32_t* d_tokens, const float* d_probs,
               int32_t query_len, int32_t draft_len, int32_t* d_draft_tokens,
               int32_t* d_draft_len, float* d_token_scores, float* d_path_scores,
               const int32_t* d_targets, int32_t* d_accept_len, int32_t fused, void* stream);

/* The propose / verify / accept loop of speculative decoding (Background
 * section: the draft is verified and the longest correct prefix kept; "Draft
 * acceptance") around the draft construction, with a stand-in for the model:
 * what the model samples for a path is that path's own future,
 * d_future_tokens [P][N][max_len] (d_future_probs likewise, may be NULL).
 * Starting from the index's current state, every step (i) appends to every
 * path the tokens the previous step settled — its accept length plus the one
 * token the model emits itself; 1 token at the first step — clipped at max_len,
 * (ii) drafts for every path from the pool of all paths, (iii) checks each draft
 * against the path's next draft_len future tokens.  Path lengths diverge as
 * paths accept different numbers of tokens.  A host loop inside the library:
 * per step one small kernel that gathers the step's input and csd_step with
 * draft_len + 1 tokens per path and counts (with the index matcher, exact
 * matching and twice the minimum of scratch memory: one launch per step, whose
 * tail gathers the next step's input).
 *   d_scratch: device memory, 4-byte aligned, scratch_bytes >=
 *     P*N*(3*draft_len + 3)*4 (step tokens, probabilities, targets, counts);
 *     with twice as much, steps alternate between the two halves;
 *   d_draft_tokens [n_steps][P][N][draft_len], d_draft_len, d_accept_len and
 *   d_path_len (lengths after the step's append) [n_steps][P][N].
 * Errors: CSD_ERR_INVALID_ARG, CSD_ERR_WORKSPACE (scratch too small or
 * misaligned).  Only enqueues. */
int csd_accept_loop(csd_index* index, int32_t n_steps, const int32_t* d_future_tokens,
                    const float* d_future_probs, int32_t query_len, int32_t draft_len,
                    void* d_scratch, size_t scratch_bytes, int32_t* d_draft_tokens,
                    int32_t* d_draft_len, int32_t* d_accept_len, int32_t* d_path_len, void* stream);

/* How many steps one launch of csd_replay (fused != 0) and csd_accept_loop runs.
 * 1 (the default): a launch per step.  More: a device-side loop — one workgroup per
 * problem, one wave per path, a workgroup barrier between steps — runs up to `steps`
 * steps per launch where the configuration allows it: exact matching through the index,
 * max_query_len <= 4, n_paths <= 16 (csd_accept_loop also needs twice the minimum of
 * scratch memory); otherwise the calls work as with 1.  Results are identical.  Nothing
 * happens on the host between two steps of these calls, so nothing is lost, and the
 * per-step cost of a launch (dispatch, cold caches, argument fetch) is paid once per
 * `steps` steps.  csd_step and the other per-step calls are not affected.
 * CSD_ERR_INVALID_ARG if steps < 1. */
int csd_set_steps_per_launch(csd_index* index, int32_t steps);

/* csd_accept_loop for callers that cannot allocate device memory or hand over a scratch
 * buffer: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments (without d_scratch / scratch_bytes), same results, same
 * launches as csd_accept_loop with twice the minimum of scratch memory; the step
 * buffers live in a fixed array of CSD_NOALLOC_SCRATCH_BYTES inside the library's device
 * image (one copy per GPU, held until the process ends).  Calls no hipMalloc / hipFree
 * nor anything else that allocates.
 *   Limit: 2 * P*N*(3*draft_len + 3)*4 bytes <= CSD_NOALLOC_SCRATCH_BYTES, else
 *   CSD_ERR_SCRATCH_LIMIT (nothing enqueued).
 *   The device current at the call must be the one the index's workspace is on.
 *   All calls on one GPU share the array: calls that overlap in time on one GPU (two
 *   streams, two indexes) race; serialise them.  Nothing in the array has to start at
 *   zero: every word is written by the launch before the one that reads it. */
#define CSD_NOALLOC_SCRATCH_BYTES (1u << 20)
int csd_accept_loop_noalloc(csd_index* index, int32_t n_steps, const int32_t* d_future_tokens,
                            const float* d_future_probs, int32_t query_len, int32_t draft_len,
                            int32_t* d_draft_tokens, int32_t* d_draft_len, int32_t* d_accept_len,
                            int32_t* d_path_len, void* stream);

/* Waits for `stream` and copies the sticky CSD_STATUS_* bits to *host_flags. */
int csd_status(csd_index* index, uint32_t* host_flags, void* stream);

/* ---- debug / parity only: canonical dumps of intermediate results ---------
 * These allocate temporary device memory, synchronise `stream`, and are not
 * meant for the decoding loop.  They run the same matching and aggregation
 * device code as csd_draft. */

/* Match sets of Eq. 3.  Row r = p*N + i owns d_match_je[d_match_off[r] ..
 * d_match_off[r+1]) as (j, e) pairs in ascending order: path j, index e of the
 * first token after the match.  d_match_je [cap][2], d_match_off [P*N+1].
 * CSD_ERR_CAPACITY if there are more than cap matches (offsets still valid). */
int csd_dump_matches(csd_index* index, int32_t query_len, int32_t* d_match_je,
                     int32_t* d_match_off, int64_t cap, void* stream);

/* Edge tables of Eq. 5.  Row r owns rows d_edge_off[r] .. d_edge_off[r+1] of
 * d_edge_duv [cap][3] = (layer d in 1..draft_len, u, v) sorted ascending and
 * d_edge_cs [cap][2] = (count C, probability sum S in 1/65536 units).
 * CSD_ERR_CAPACITY if cap is too small or a path's tables exceed the
 * on-chip tier (such a path is still drafted correctly by csd_draft). */
int csd_dump_edges(csd_index* index, int32_t query_len, int32_t draft_len, int32_t* d_edge_duv,
                   uint64_t* d_edge_cs, int32_t* d_edge_off, int64_t cap, void* stream);

/* Measurement aid, not part of the method: copies `bytes` (a multiple of 16,
 * both pointers 16-byte aligned) from d_src to d_dst with a plain copy kernel.
 * Hardware traffic counters (bytes fetched / written per dispatch) are
 * calibrated against this kernel of known size. */
int csd_debug_copy(void* d_dst, const void* d_src, size_t bytes, void* stream);

/* Text for a csd_error (and, for CSD_ERR_HIP, the last HIP error string). */
const char* csd_strerror(int err);

#ifdef __cplusplus
}
#endif
#endif /* CSD_H_ */
