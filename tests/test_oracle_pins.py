"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle is checked against things other than itself: a hand-derived worked
example (tests/golden), closed forms, invariants, reductions to library
routines (collections.Counter, numpy.nonzero) and an exact-rational brute
force on thousands of tiny inputs.
"""
import json
import os
from collections import Counter
from fractions import Fraction

import numpy as np
import pytest

import bruteforce as bf
from paper_2503_05330_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_dag.json")


def pack(paths, probs=None, max_len=None):
    """Ragged python lists -> (tok [N][max_len], prob or None, len [N])."""
    N = len(paths)
    max_len = max_len or max(1, max(len(p) for p in paths))
    tok = np.full((N, max_len), -7, dtype=np.int32)      # junk past the end must be ignored
    pr = None if probs is None else np.full((N, max_len), 0.123, dtype=np.float32)
    for j, p in enumerate(paths):
        tok[j, :len(p)] = p
        if probs is not None:
            pr[j, :len(p)] = probs[j]
    return tok, pr, np.array([len(p) for p in paths], dtype=np.int32)


# ---------------------------------------------------------------- worked example
def test_hand_worked_example(oracle):
    g = json.load(open(GOLDEN))
    tok, _, ln = pack(g["paths"])
    i, k, L = g["query_path"], g["k"], g["L"]
    assert oracle.matches(tok, ln, i, k).tolist() == g["matches"]
    duv, cs = oracle.edges(tok, None, ln, i, k, L)
    assert [list(r) + [int(c[0])] for r, c in zip(duv.tolist(), cs)] == g["edges_counts"]
    assert (cs[:, 1] == cs[:, 0] * 65536).all()          # p = 1 for every instance
    for mode in (0, 1):
        want = g["no_probs"]["mode%d" % mode]
        for alpha in (0.0, 0.3, 1.0):                    # no probs: alpha cannot matter
            d, n, ts, ps = oracle.draft(tok, None, ln, i, k, L, alpha, mode)
            assert d[:n].tolist() == want["draft"] and n == len(want["draft"])
            assert ts[:n].tolist() == want["token_scores"] and float(ps) == want["path_score"]
    tokp, pr, ln = pack(g["paths"], g["probs"])
    for key, alpha in (("alpha1_mode0", 1.0), ("alpha0.5_mode0", 0.5)):
        want = g["with_probs"][key]
        d, n, ts, ps = oracle.draft(tokp, pr, ln, i, k, L, alpha, 0)
        assert d[:n].tolist() == want["draft"]
        assert ts[:n].tolist() == want["token_scores"] and float(ps) == want["path_score"]
    for a in g["accept"]:
        d, n, _, _ = oracle.draft(tok, None, ln, i, k, L, 1.0, a["mode"])
        assert oracle.accept(d, n, np.array(a["target"], dtype=np.int32)) == a["accept_len"]


def test_strict_length_reading_would_lose_a_match(oracle):
    """Reading R2: path 1's second occurrence lies beyond path 0's own length
    (e = 7 > len_0 = 4) and still counts."""
    g = json.load(open(GOLDEN))
    tok, _, ln = pack(g["paths"])
    assert [1, 7] in oracle.matches(tok, ln, 0, 2).tolist()


# ---------------------------------------------------------------- quantisation
def test_quantize_prob_values(oracle):
    q = oracle.quantize_prob
    assert q(0.0) == 0 and q(1.0) == 65536 and q(0.5) == 32768 and q(0.25) == 16384
    assert q(-0.5) == 0 and q(7.0) == 65536 and q(float("nan")) == 0
    assert q(1.0 / 65536) == 1
    # exact halves go to the even neighbour
    assert q(2.5 / 65536) == 2 and q(3.5 / 65536) == 4 and q(0.5 / 65536) == 0
    assert q(np.float32(0.7)) == round(float(np.float32(0.7)) * 65536)
    assert oracle.alpha_q(1.0) == 65536 and oracle.alpha_q(0.0) == 0 and oracle.alpha_q(0.5) == 32768


# ---------------------------------------------------------------- closed forms
def test_closed_form_identical_paths_draft_own_continuation(oracle):
    """N identical paths over a sequence without repeated q-grams; path 0 is
    truncated to t tokens: its draft is seq[t:t+L], each score N-1."""
    N, T, k, L = 5, 40, 3, 6
    seq = list(range(100, 100 + T))                      # all tokens distinct
    for t in (3, 10, T - 2):
        paths = [seq[:t]] + [seq for _ in range(N - 1)]
        tok, _, ln = pack(paths)
        d, n, ts, ps = oracle.draft(tok, None, ln, 0, k, L)
        want = seq[t:t + L]
        assert d[:n].tolist() == want and n == len(want)
        assert ts[:n].tolist() == [float(N - 1)] * n and float(ps) == n * (N - 1)
        assert (d[n:] == -1).all() and (ts[n:] == 0).all()
    # a full-length path's suffix sits at the very end of the others: no successor, no draft
    tok, _, ln = pack([seq] * N)
    assert oracle.draft(tok, None, ln, 0, k, L)[1] == 0


def test_closed_form_constant_paths(oracle):
    """All tokens equal: M = (N-1)(T-q); alive at layer d = (N-1)(T-q-d+1)."""
    N, T, k, L, c = 4, 20, 3, 6, 9
    tok, _, ln = pack([[c] * T] * N)
    assert len(oracle.matches(tok, ln, 1, k)) == (N - 1) * (T - k)
    d, n, ts, ps = oracle.draft(tok, None, ln, 1, k, L)
    assert n == min(L, T - k) and d[:n].tolist() == [c] * n
    assert ts[:n].tolist() == [float((N - 1) * (T - k - dd + 1)) for dd in range(1, n + 1)]
    # short paths: the walk ends when no candidate is alive any more
    T2 = 6
    tok, _, ln = pack([[c] * T2] * N)
    d, n, ts, _ = oracle.draft(tok, None, ln, 0, k, L)
    assert n == T2 - k and ts[:n].tolist() == [float((N - 1) * (T2 - k - dd + 1)) for dd in range(1, n + 1)]


def test_closed_form_disjoint_vocab_is_empty(oracle):
    paths = [list(range(100 * j, 100 * j + 30)) for j in range(4)]
    tok, _, ln = pack(paths)
    for i in range(4):
        d, n, ts, ps = oracle.draft(tok, None, ln, i, 2, 5)
        assert n == 0 and (d == -1).all() and (ts == 0).all() and float(ps) == 0.0
        assert len(oracle.matches(tok, ln, i, 2)) == 0
        assert len(oracle.edges(tok, None, ln, i, 2, 5)[0]) == 0


def test_short_and_empty_paths(oracle):
    paths = [[], [4, 4, 4, 4], [4]]
    tok, _, ln = pack(paths)
    assert oracle.draft(tok, None, ln, 0, 3, 4)[1] == 0          # q = 0
    # path 2 has one token: q clips to 1 and matches path 1 at e = 1, 2, 3
    assert oracle.matches(tok, ln, 2, 3).tolist() == [[1, 1], [1, 2], [1, 3]]
    d, n, ts, _ = oracle.draft(tok, None, ln, 2, 3, 4)
    assert d[:n].tolist() == [4, 4, 4] and ts[:n].tolist() == [3.0, 2.0, 1.0]


def test_ties_break_to_lowest_id(oracle):
    # two continuations of equal weight after the query (7): tokens 30 and 12
    paths = [[1, 7], [7, 30, 5], [7, 12, 5], [0, 7]]
    tok, _, ln = pack(paths)
    for mode in (0, 1):
        d, n, ts, _ = oracle.draft(tok, None, ln, 0, 1, 2, 1.0, mode)
        assert d[:n].tolist() == [12, 5] and ts[:n].tolist() == [1.0, 2.0 if mode == 0 else 1.0]


# ---------------------------------------------------------------- library reductions
def test_match_positions_reduce_to_numpy_nonzero(oracle):
    rng = np.random.default_rng(7)
    other = rng.integers(0, 6, size=200).astype(np.int32)
    for tokq in range(6):
        tok, _, ln = pack([[3, tokq], other.tolist()])
        got = oracle.matches(tok, ln, 0, 1)
        want = np.nonzero(other[:-1] == tokq)[0] + 1          # successor index; last token has none
        assert (got[:, 0] == 1).all() and got[:, 1].tolist() == want.tolist()


def test_layer1_counts_reduce_to_ngram_counter(oracle):
    """L = 1, alpha = 0: the edge table is the successor-count table of the
    q-gram over the other paths — a plain n-gram Counter."""
    w = synth.scaled(synth.WORKLOADS["C1"], vocab=12, pool=6, max_len=96)
    tokens, probs = synth.make_paths(w)
    tok = tokens[0]
    ln = np.array([96, 80, 96, 50], dtype=np.int32)
    for q in (1, 2, 3):
        for i in range(4):
            gram = tuple(tok[i, ln[i] - q:ln[i]])
            cnt = Counter()
            for j in range(4):
                if j == i:
                    continue
                seq = tok[j, :ln[j]].tolist()
                cnt.update(seq[e] for e in range(q, len(seq)) if tuple(seq[e - q:e]) == gram)
            duv, cs = oracle.edges(tok, probs[0], ln, i, q, 1)
            assert {int(r[2]): int(c[0]) for r, c in zip(duv, cs)} == dict(cnt)
            assert (duv[:, 0] == 1).all() and (duv[:, 1] == gram[-1]).all()
            d, n, ts, _ = oracle.draft(tok, probs[0], ln, i, q, 1, alpha=0.0)
            if cnt:
                top = max(cnt.values())
                assert n == 1 and d[0] == min(v for v, c in cnt.items() if c == top) and ts[0] == top
            else:
                assert n == 0


# ---------------------------------------------------------------- brute force
def _random_case(rng):
    N = int(rng.integers(2, 5))
    V = int(rng.integers(2, 7))
    paths = [rng.integers(0, V, size=int(rng.integers(0, 25))).tolist() for _ in range(N)]
    # probabilities on a coarse dyadic grid so that ties between sums are common
    probs = [(rng.integers(0, 9, size=len(p)) / 8.0).astype(np.float32).tolist() for p in paths]
    return paths, probs


def test_brute_force_tiny_inputs(oracle):
    rng = np.random.default_rng(12345)
    n_nonempty = 0
    for case in range(1500):
        paths, probs = _random_case(rng)
        use_probs = case % 3 != 0
        k = int(rng.integers(1, 5))
        L = int(rng.integers(1, 7))
        alpha = Fraction(int(rng.integers(0, 5)), 4)
        mode = int(rng.integers(0, 2))
        tok, pr, ln = pack(paths, probs if use_probs else None, max_len=26)
        for i in range(len(paths)):
            q, M = bf.match_set(paths, i, k)
            assert oracle.matches(tok, ln, i, k).tolist() == [list(m) for m in sorted(M)]
            E = bf.edge_tables(paths, probs if use_probs else None, i, k, L)
            duv, cs = oracle.edges(tok, pr, ln, i, k, L)
            assert [tuple(r) for r in duv.tolist()] == sorted(E)
            for r, c in zip(duv.tolist(), cs):
                assert int(c[0]) == E[tuple(r)][0] and Fraction(int(c[1]), 65536) == E[tuple(r)][1]
            toks, scores = bf.draft(paths, probs if use_probs else None, i, k, L, alpha, mode)
            d, n, ts, ps = oracle.draft(tok, pr, ln, i, k, L, float(alpha), mode)
            assert d[:n].tolist() == toks and n == len(toks)
            assert (d[n:] == -1).all() and (ts[n:] == 0).all()
            assert ts[:n].tolist() == [float(np.float32(float(s))) for s in scores]
            assert float(ps) == float(np.float32(float(sum(scores, Fraction(0)))))
            n_nonempty += n > 0
            tgt = rng.integers(0, 3, size=L).astype(np.int32)
            if n and rng.random() < 0.5:
                tgt[:n] = d[:n]
                tgt[int(rng.integers(0, L)):] = -5
            assert oracle.accept(d, n, tgt) == bf.accept(toks, tgt.tolist())
    assert n_nonempty > 1000


def test_real_valued_probabilities_against_fractions(oracle):
    """Arbitrary float32 probabilities and alpha = k/65536: the integer key
    equals Eq. 5 evaluated exactly on the quantised probabilities."""
    rng = np.random.default_rng(99)
    for case in range(200):
        N = 3
        paths = [rng.integers(0, 4, size=int(rng.integers(4, 30))).tolist() for _ in range(N)]
        probs = [rng.random(len(p)).astype(np.float32).tolist() for p in paths]
        alpha_q = int(rng.integers(0, 65537))
        tok, pr, ln = pack(paths, probs)
        for mode in (0, 1):
            toks, scores = bf.draft(paths, probs, 0, 2, 5, Fraction(alpha_q, 65536), mode)
            d, n, ts, ps = oracle.draft(tok, pr, ln, 0, 2, 5, alpha_q / 65536.0, mode)
            assert d[:n].tolist() == toks
            assert ts[:n].tolist() == [float(np.float32(float(s))) for s in scores]


# ---------------------------------------------------------------- invariants on the synthetic workloads
@pytest.mark.parametrize("name", ["C1", "C2"])
def test_invariants_on_synthetic_paths(oracle, name):
    w = synth.WORKLOADS[name]
    if name == "C2":
        w = synth.scaled(w, max_len=256, n_paths=8)
    tokens, probs = synth.make_paths(w)
    tok, pr = tokens[0], probs[0]
    k, L = w.query_len, w.draft_len
    seen = 0
    for t in range(8, w.max_len, 23):
        ln = np.full(w.n_paths, t, dtype=np.int32)
        for i in range(w.n_paths):
            M = oracle.matches(tok, ln, i, k)
            duv, cs = oracle.edges(tok, pr, ln, i, k, L)
            E = {tuple(r): (int(c[0]), int(c[1])) for r, c in zip(duv.tolist(), cs)}
            for mode in (0, 1):
                d, n, ts, ps = oracle.draft(tok, pr, ln, i, k, L, 1.0, mode)
                if len(M) == 0:
                    assert n == 0
                    continue
                assert n >= 1            # every match has a successor, so layer 1 is never empty
                cur = int(tok[i, t - 1])
                for dd in range(n):
                    c, s = E[(dd + 1, cur, int(d[dd]))]      # KeyError = transition is not an edge
                    assert c > 0
                    assert float(ts[dd]) * 65536 >= s * (1 - 1e-6)   # in-weight >= edge weight
                    cur = int(d[dd])
                seen += 1
            # alpha = 0 ignores probabilities; without probabilities alpha is irrelevant
            a = oracle.draft(tok, pr, ln, i, k, L, 0.0, 0)
            b = oracle.draft(tok, None, ln, i, k, L, 0.0, 0)
            c_ = oracle.draft(tok, None, ln, i, k, L, 0.37, 0)
            assert a[0].tolist() == b[0].tolist() == c_[0].tolist()
            assert a[2].tolist() == b[2].tolist() == c_[2].tolist()
    assert seen > 20


def test_draft_all_matches_single_calls(oracle):
    w = synth.scaled(synth.WORKLOADS["C4"], n_problems=3, n_paths=5, max_len=120)
    tokens, probs = synth.make_paths(w)
    ln = np.random.default_rng(3).integers(0, 121, size=(3, 5)).astype(np.int32)
    tg = synth.make_targets(tokens, 60, w.draft_len)
    out = oracle.draft_all(tokens, probs, ln, 3, w.draft_len, 1.0, 0, tg)
    for p in range(3):
        for i in range(5):
            d, n, ts, ps = oracle.draft(tokens[p], probs[p], ln[p], i, 3, w.draft_len)
            assert out["draft"][p, i].tolist() == d.tolist() and out["draft_len"][p, i] == n
            assert out["token_scores"][p, i].tolist() == ts.tolist() and out["path_scores"][p, i] == ps
            assert out["accept_len"][p, i] == oracle.accept(d, n, tg[p, i])


def test_threaded_batch_equals_the_serial_loop_bit_for_bit(oracle):
    """oracle.draft_many (rows handed to several host threads) against draft_all called state by
    state on one thread: same bits for every output, whatever the number of threads, under
    exact and one-edit matching and every pool."""
    w = synth.scaled(synth.WORKLOADS["C4"], n_problems=3, n_paths=6, max_len=150)
    tokens, probs = synth.make_paths(w)
    rng = np.random.default_rng(11)
    S, L = 9, w.draft_len
    lens = rng.integers(0, 151, size=(S, 3, 6)).astype(np.int32)
    lens[0] = 150
    targets = np.stack([synth.make_noisy_targets(w, tokens, 40 + s, L) for s in range(S)])
    for eps, pool, extras in ((0, 0, {}), (1, 0, {}), (0, 1, {}), (1, 2, {}),
                              (0, 0, dict(include_self=True, backoff=True))):
        serial = [oracle.draft_all(tokens, probs, lens[s], 3, L, 0.75, 1, targets[s], eps=eps,
                                   pool_mode=pool, **extras) for s in range(S)]
        for threads in (1, 2, 8, 37):
            many = oracle.draft_many(tokens, probs, lens, 3, L, 0.75, 1, targets, eps=eps, pool_mode=pool,
                                     threads=threads, **extras)
            for key in ("draft", "draft_len", "token_scores", "path_scores", "accept_len"):
                want = np.stack([x[key] for x in serial])
                assert many[key].tobytes() == want.tobytes(), (key, eps, pool, threads)
    assert int(np.stack([x["draft_len"] for x in serial]).max()) > 0
    none = oracle.draft_many(tokens, None, lens[:2], 3, L, threads=4)
    assert none["accept_len"] is None and none["draft"].shape == (2, 3, 6, L)
    assert 1 <= oracle.host_threads() <= 16


def test_generator_is_seeded_and_shaped():
    for name, w in synth.WORKLOADS.items():
        if name in ("C4", "C5"):
            w = synth.scaled(w, n_problems=min(w.n_problems, 2), max_len=512)
        a, pa = synth.make_paths(w)
        b, pb = synth.make_paths(w)
        assert (a == b).all() and (pa == pb).all()
        assert a.shape == (w.n_problems, w.n_paths, w.max_len) and a.dtype == np.int32
        assert a.min() >= 0 and a.max() < w.vocab and pa.min() > 0 and pa.max() <= 1


# ---------------------------------------------------------------- fuzzy suffix matching (Eq. 4)
def test_edit_distance_textbook_values(oracle):
    word = lambda w: [ord(c) for c in w]
    assert oracle.edit_distance(word("kitten"), word("sitting")) == 3
    assert oracle.edit_distance(word("flaw"), word("lawn")) == 2
    assert oracle.edit_distance(word("intention"), word("execution")) == 5
    assert oracle.edit_distance([], word("abc")) == 3 and oracle.edit_distance(word("abc"), []) == 3
    assert oracle.edit_distance(word("abc"), word("abc")) == 0
    rng = np.random.default_rng(4)
    for _ in range(300):
        a = tuple(rng.integers(0, 3, size=int(rng.integers(0, 7))).tolist())
        b = tuple(rng.integers(0, 3, size=int(rng.integers(0, 7))).tolist())
        assert oracle.edit_distance(a, b) == bf.lev(a, b) == bf.lev(b, a)
        assert (oracle.edit_distance(a, b) <= 1) == bf.within_one_edit(a, b)


def test_fuzzy_hand_cases(oracle):
    # query (1,2,3); the other path holds it with one substitution, one deletion, one insertion
    paths = [[9, 1, 2, 3],
             [1, 7, 3, 50, 0, 1, 3, 51, 0, 1, 2, 8, 3, 52, 0, 4, 4, 4, 53]]
    tok, _, ln = pack(paths)
    exact = oracle.matches(tok, ln, 0, 3, 0)
    assert len(exact) == 0
    fuzzy = oracle.matches(tok, ln, 0, 3, 1)
    # after (1,7,3): e=3; after (1,3): e=7; after (1,2): e=11; after (1,2,8): e=12; after (1,2,8,3): e=13
    assert fuzzy.tolist() == [[1, 3], [1, 7], [1, 11], [1, 12], [1, 13]]
    d, n, ts, _ = oracle.draft(tok, None, ln, 0, 3, 1, 1.0, 0, eps=1)
    # layer 1 hangs under the query whatever token precedes the match: 50, 51, 8, 3, 52
    assert n == 1 and d[0] == 3 and ts[0] == 1.0
    duv, cs = oracle.edges(tok, None, ln, 0, 3, 1, eps=1)
    assert duv.tolist() == [[1, 3, 3], [1, 3, 8], [1, 3, 50], [1, 3, 51], [1, 3, 52]]
    assert (cs[:, 0] == 1).all()


def test_fuzzy_tolerance_zero_is_exact_and_sets_grow(oracle):
    w = synth.scaled(synth.WORKLOADS["C1"], vocab=40, pool=8, max_len=80)
    tokens, probs = synth.make_paths(w)
    ln = np.array([80, 61, 80, 33], dtype=np.int32)
    for i in range(4):
        for k in (1, 2, 3):
            m0 = {tuple(r) for r in oracle.matches(tokens[0], ln, i, k, 0).tolist()}
            m1 = {tuple(r) for r in oracle.matches(tokens[0], ln, i, k, 1).tolist()}
            m2 = {tuple(r) for r in oracle.matches(tokens[0], ln, i, k, 2).tolist()}
            assert m0 <= m1 <= m2
            if k >= 2:       # one edit always admits the exact matches of the (k-1)-suffix
                short = {tuple(r) for r in oracle.matches(tokens[0], ln, i, k - 1, 0).tolist()}
                assert short <= m1


def test_fuzzy_brute_force_tiny_inputs(oracle):
    rng = np.random.default_rng(777)
    n_more = 0
    for case in range(500):
        paths, probs = _random_case(rng)
        use_probs = case % 2 == 0
        k = int(rng.integers(1, 5))
        L = int(rng.integers(1, 6))
        eps = (2, 1, 1, 3, 1)[case % 5]
        alpha = Fraction(int(rng.integers(0, 5)), 4)
        mode = int(rng.integers(0, 2))
        tok, pr, ln = pack(paths, probs if use_probs else None, max_len=26)
        for i in range(len(paths)):
            q, M = bf.match_set(paths, i, k, eps)
            assert oracle.matches(tok, ln, i, k, eps).tolist() == [list(m) for m in sorted(M)]
            n_more += len(M) > len(bf.match_set(paths, i, k, 0)[1])
            E = bf.edge_tables(paths, probs if use_probs else None, i, k, L, eps)
            duv, cs = oracle.edges(tok, pr, ln, i, k, L, eps)
            assert [tuple(r) for r in duv.tolist()] == sorted(E)
            for r, c in zip(duv.tolist(), cs):
                assert int(c[0]) == E[tuple(r)][0] and Fraction(int(c[1]), 65536) == E[tuple(r)][1]
            toks, scores = bf.draft(paths, probs if use_probs else None, i, k, L, alpha, mode, eps)
            d, n, ts, ps = oracle.draft(tok, pr, ln, i, k, L, float(alpha), mode, eps)
            assert d[:n].tolist() == toks and n == len(toks)
            assert ts[:n].tolist() == [float(np.float32(float(s))) for s in scores]
    assert n_more > 200


# ---------------------------------------------------------------- tree and list pools (the ablation's variants)
def test_pool_modes_hand_case(oracle):
    # query (1, 2); continuations in the other paths: [5,6,7] twice, [5,8,9] once, [4,6,7] once.
    paths = [[1, 2],
             [1, 2, 5, 6, 7, 0, 1, 2, 5, 6, 7],
             [1, 2, 5, 8, 9, 3, 3, 1, 2, 4, 6, 7]]
    tok, _, ln = pack(paths)
    dag = oracle.draft(tok, None, ln, 0, 2, 3, 1.0, 0, pool_mode=0)
    tree = oracle.draft(tok, None, ln, 0, 2, 3, 1.0, 0, pool_mode=1)
    lst = oracle.draft(tok, None, ln, 0, 2, 3, 1.0, 0, pool_mode=2)
    # DAG: layer 1 {5: 3, 4: 1}; layer 2 after 5: 6 (in-weight 3, merging the 6 after 4); layer 3: 7 (3)
    assert dag[0][:dag[1]].tolist() == [5, 6, 7] and dag[2][:3].tolist() == [3.0, 3.0, 3.0]
    # tree: 5 (3 candidates) -> 6 (2 of them; the 6 after 4 is another branch) -> 7 (2)
    assert tree[0][:tree[1]].tolist() == [5, 6, 7] and tree[2][:3].tolist() == [3.0, 2.0, 2.0]
    # list: every candidate weighs 3 (three tokens of weight 1): the first one, path 1 at e = 2
    assert lst[0][:lst[1]].tolist() == [5, 6, 7] and lst[2][:3].tolist() == [1.0, 1.0, 1.0]
    assert float(lst[3]) == 3.0 and float(tree[3]) == 7.0 and float(dag[3]) == 9.0


def test_pool_modes_differ_where_they_should(oracle):
    # after query (1): candidates [2,3] x2 (paths 1, 2) and [4,3] x3 ... the DAG merges the 3s of layer 2
    paths = [[1], [1, 2, 3], [1, 2, 3], [1, 4, 9], [1, 4, 9, 9], [1, 4, 8]]
    tok, _, ln = pack(paths)
    tree = oracle.draft(tok, None, ln, 0, 1, 2, 1.0, 0, pool_mode=1)
    assert tree[0][:tree[1]].tolist() == [4, 9] and tree[2][:2].tolist() == [3.0, 2.0]
    lst = oracle.draft(tok, None, ln, 0, 1, 3, 1.0, 0, pool_mode=2)
    # the longest continuation wins under alpha = 1 without probabilities: path 4, [4, 9, 9]
    assert lst[0][:lst[1]].tolist() == [4, 9, 9]
    # with probabilities the list follows the most probable single candidate
    probs = [[1.0], [1.0, 0.875, 0.875], [1.0, 0.5, 0.5], [1.0, 0.25, 0.25], [1.0, 0.25, 0.25, 0.25], [1.0, 0.5, 0.5]]
    tok, pr, ln = pack(paths, probs)
    lst = oracle.draft(tok, pr, ln, 0, 1, 3, 1.0, 0, pool_mode=2)
    assert lst[0][:lst[1]].tolist() == [2, 3] and float(lst[3]) == 1.75


def test_pool_modes_brute_force_tiny_inputs(oracle):
    rng = np.random.default_rng(4242)
    n_tree_differs = n_list_differs = 0
    for case in range(600):
        paths, probs = _random_case(rng)
        use_probs = case % 2 == 0
        k = int(rng.integers(1, 4))
        L = int(rng.integers(1, 6))
        eps = 1 if case % 4 == 0 else 0
        alpha = Fraction(int(rng.integers(0, 5)), 4)
        tok, pr, ln = pack(paths, probs if use_probs else None, max_len=26)
        for i in range(len(paths)):
            pp = probs if use_probs else None
            dag = oracle.draft(tok, pr, ln, i, k, L, float(alpha), 1, eps, 0)
            for mode, brute in ((1, bf.tree_draft), (2, bf.list_draft)):
                toks, scores = brute(paths, pp, i, k, L, alpha, eps)
                d, n, ts, ps = oracle.draft(tok, pr, ln, i, k, L, float(alpha), 0, eps, mode)
                assert d[:n].tolist() == toks and (d[n:] == -1).all()
                assert ts[:n].tolist() == [float(np.float32(float(s))) for s in scores]
                assert float(ps) == float(np.float32(float(sum(scores, Fraction(0)))))
                if mode == 1:
                    n_tree_differs += d[:n].tolist() != dag[0][:dag[1]].tolist()
                else:
                    n_list_differs += d[:n].tolist() != dag[0][:dag[1]].tolist()
            # a tree or list draft is the start of a real continuation; the first token of the
            # tree is the DAG's first token (layer 1 is the same tally under edge scoring)
            _, M = bf.match_set(paths, i, k, eps)
            tree = oracle.draft(tok, pr, ln, i, k, L, float(alpha), 0, eps, 1)
            lst = oracle.draft(tok, pr, ln, i, k, L, float(alpha), 0, eps, 2)
            for d, n, _, _ in (tree, lst):
                assert n == 0 or any(list(paths[j][e:e + n]) == d[:n].tolist() for (j, e) in M)
            assert (tree[1] > 0) == (dag[1] > 0) == (lst[1] > 0) == (len(M) > 0)
            if dag[1] > 0:
                assert tree[0][0] == dag[0][0] and tree[2][0] == dag[2][0]
    assert n_tree_differs > 20 and n_list_differs > 20


# ---------------------------------------------------------------- the propose / verify / accept loop
def test_accept_loop_closed_forms(oracle):
    T, N, k, L = 60, 4, 3, 5
    seq = np.arange(100, 100 + T, dtype=np.int32)           # no repeated q-gram
    tok = np.tile(seq, (1, N, 1))
    # (a) identical paths in lockstep: the suffix sits at the END of every other path, so it
    # has no successor there: no match, nothing accepted, one token per step
    r = oracle.accept_loop(tok, None, np.zeros((1, N), np.int32), k, L, 20)
    assert (r["draft_len"] == 0).all() and (r["accept_len"] == 0).all()
    assert (r["path_len"][:, 0, :] == (np.arange(20) + 1)[:, None]).all()
    # (b) the other paths are complete: path 0 drafts its own future and all of it is accepted
    lens = np.array([[k, T, T, T]], np.int32)
    r = oracle.accept_loop(tok, None, lens, k, L, 12)
    want_len, settled = k, 0
    for s in range(12):
        want_len = min(T, want_len + settled + 1)
        assert r["path_len"][s, 0, 0] == want_len and (r["path_len"][s, 0, 1:] == T).all()
        settled = min(L, T - want_len)
        assert r["accept_len"][s, 0, 0] == settled == r["draft_len"][s, 0, 0]
        assert r["draft"][s, 0, 0, :settled].tolist() == seq[want_len:want_len + settled].tolist()
    assert r["final_len"][0, 0] == T


def test_accept_loop_is_the_composition_of_its_steps(oracle):
    w = synth.WORKLOADS["C1"]
    tokens, probs = synth.make_paths(w)
    k, L, S = w.query_len, w.draft_len, 90
    for eps, pool_mode in ((0, 0), (1, 0), (0, 1), (0, 2)):
        r = oracle.accept_loop(tokens, probs, np.zeros(tokens.shape[:2], np.int32), k, L, S, eps=eps,
                               pool_mode=pool_mode)
        prev_len = np.zeros(tokens.shape[:2], np.int64)
        prev_acc = np.zeros(tokens.shape[:2], np.int64)
        for s in range(S):
            lens = np.minimum(prev_len + prev_acc + 1, w.max_len)
            assert np.array_equal(r["path_len"][s], lens)
            step = oracle.draft_all(tokens, probs, lens.astype(np.int32), k, L, eps=eps, pool_mode=pool_mode)
            assert np.array_equal(step["draft"], r["draft"][s]) and np.array_equal(step["draft_len"], r["draft_len"][s])
            for i in range(w.n_paths):
                future = tokens[0, i, lens[0, i]:lens[0, i] + L].tolist()
                n = int(step["draft_len"][0, i])
                assert r["accept_len"][s, 0, i] == bf.accept(step["draft"][0, i, :n].tolist(), future)
            prev_len, prev_acc = lens, r["accept_len"][s].astype(np.int64)
        assert r["accept_len"].sum() > 0 and r["path_len"][-1].max() > r["path_len"][-1].min() > S - 1


def test_accept_length_grows_with_the_number_of_paths(oracle):
    """The paper's qualitative finding (sample-size analysis): more parallel paths give longer
    accepted drafts.  On the synthetic pool of C2 the mean accept length per step rises
    monotonically from N = 2 to 16."""
    w = synth.WORKLOADS["C2"]
    tokens, probs = synth.make_paths(w)
    mean = {}
    for N in (2, 4, 8, 16):
        r = oracle.accept_loop(tokens[:, :N], probs[:, :N], np.zeros((1, N), np.int32), w.query_len,
                               w.draft_len, 400)
        mean[N] = r["accept_len"].mean()
    assert mean[2] < mean[4] < mean[8] < mean[16] and mean[16] > 3 * mean[2]


# ---------------------------------------------------------------- self-history and query back-off
def test_self_history_and_back_off_hand_cases(oracle):
    # one periodic path: without its own history there is nothing to search; with it the two
    # earlier occurrences of (2, 3) both continue 1 2 3, so every layer counts 2 (then 1)
    tok, _, ln = pack([[1, 2, 3, 1, 2, 3, 1, 2, 3]])
    assert oracle.draft(tok, None, ln, 0, 2, 4)[1] == 0
    assert oracle.matches(tok, ln, 0, 2, include_self=True).tolist() == [[0, 3], [0, 6]]
    d, n, ts, _ = oracle.draft(tok, None, ln, 0, 2, 4, include_self=True)
    assert d[:n].tolist() == [1, 2, 3, 1] and ts[:n].tolist() == [2.0, 2.0, 2.0, 1.0]
    # the query's own occurrence at the end of the path has no successor: never a match
    tok, _, ln = pack([[4, 5, 6]])
    assert oracle.matches(tok, ln, 0, 2, include_self=True).tolist() == []
    # back-off: (2, 3, 9) occurs nowhere else, (3, 9) does, and is followed by 7 8
    tok, _, ln = pack([[1, 2, 3, 9], [5, 3, 9, 7, 8], [9, 6, 6]])
    assert oracle.draft(tok, None, ln, 0, 3, 3)[1] == 0
    d, n, _, _ = oracle.draft(tok, None, ln, 0, 3, 3, backoff=True)
    assert d[:n].tolist() == [7, 8]
    assert d.tolist() == oracle.draft(tok, None, ln, 0, 2, 3)[0].tolist()
    # ... and stops at the first non-empty set: the one-token query (9) would also see path 2
    assert oracle.draft(tok, None, ln, 0, 1, 3)[0][:1].tolist() == [6]
    # nothing at any length: empty
    tok, _, ln = pack([[1, 2, 3], [4, 5, 6]])
    assert oracle.draft(tok, None, ln, 0, 3, 3, backoff=True)[1] == 0


def test_self_history_and_back_off_brute_force_tiny_inputs(oracle):
    rng = np.random.default_rng(1718)
    n_self_differs = n_backed_off = 0
    for case in range(700):
        paths, probs = _random_case(rng)
        use_probs = case % 2 == 0
        k = int(rng.integers(1, 5))
        L = int(rng.integers(1, 6))
        eps = 1 if case % 5 == 0 else 0
        alpha = Fraction(int(rng.integers(0, 5)), 4)
        mode = int(rng.integers(0, 2))
        inc, back = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        tok, pr, ln = pack(paths, probs if use_probs else None, max_len=26)
        pp = probs if use_probs else None
        for i in range(len(paths)):
            _, M = bf.match_set(paths, i, k, eps, inc)
            assert oracle.matches(tok, ln, i, k, eps, include_self=inc).tolist() == [list(m) for m in sorted(M)]
            E = bf.edge_tables(paths, pp, i, k, L, eps, inc)
            duv, _ = oracle.edges(tok, pr, ln, i, k, L, eps, include_self=inc)
            assert [tuple(r) for r in duv.tolist()] == sorted(E)
            for pool_mode, brute in ((0, None), (1, bf.tree_draft), (2, bf.list_draft)):
                if brute is None:
                    toks, scores = bf.draft(paths, pp, i, k, L, alpha, mode, eps, inc, back)
                else:
                    toks, scores = brute(paths, pp, i, k, L, alpha, eps, inc, back)
                d, n, ts, ps = oracle.draft(tok, pr, ln, i, k, L, float(alpha), mode, eps, pool_mode,
                                            include_self=inc, backoff=back)
                assert d[:n].tolist() == toks and (d[n:] == -1).all()
                assert ts[:n].tolist() == [float(np.float32(float(s))) for s in scores]
                assert float(ps) == float(np.float32(float(sum(scores, Fraction(0)))))
            plain = oracle.draft(tok, pr, ln, i, k, L, float(alpha), mode, eps, 0)
            both = oracle.draft(tok, pr, ln, i, k, L, float(alpha), mode, eps, 0, include_self=inc, backoff=back)
            # neither option can empty a draft, and back-off changes nothing where k has matches
            assert both[1] > 0 or plain[1] == 0
            if plain[1] > 0 and not inc:
                assert both[0].tolist() == plain[0].tolist()
            n_self_differs += inc and not back and both[0].tolist() != plain[0].tolist()
            n_backed_off += back and bf.backed_off_k(paths, i, k, eps, inc) < min(k, len(paths[i]))
    assert n_self_differs > 20 and n_backed_off > 20


def test_options_reach_the_batched_entry_points(oracle):
    w = synth.scaled(synth.WORKLOADS["C1"], max_len=48)
    tokens, probs = synth.make_paths(w)
    lens = np.full(tokens.shape[:2], 40, dtype=np.int32)
    for inc, back in ((True, False), (False, True), (True, True)):
        allp = oracle.draft_all(tokens, probs, lens, 3, 5, 1.0, 0, include_self=inc, backoff=back)
        for i in range(w.n_paths):
            d, n, ts, ps = oracle.draft(tokens[0], probs[0], lens[0], i, 3, 5, 1.0, 0, include_self=inc, backoff=back)
            assert allp["draft"][0, i].tolist() == d.tolist() and allp["draft_len"][0, i] == n
    # the accept loop with both options: every step is the draft of the lengths it reports
    start = np.full(tokens.shape[:2], 8, dtype=np.int32)
    run = oracle.accept_loop(tokens, probs, start, 3, 5, 6, include_self=True, backoff=True)
    for s in range(6):
        step = oracle.draft_all(tokens, probs, run["path_len"][s], 3, 5, 1.0, 0, include_self=True, backoff=True)
        assert step["draft"].tolist() == run["draft"][s].tolist()


def test_pins_pass_with_the_oracle_built_under_sanitizers():
    """The whole pin suite once more in a child process whose oracle is compiled with
    -fsanitize=address,undefined (host code only): an out-of-bounds read, a use after free or
    signed overflow anywhere in the oracle aborts the child."""
    import subprocess
    import sys
    if os.environ.get("CSD_ORACLE_SANITIZE") == "1":
        pytest.skip("already inside the sanitized run")
    libasan = subprocess.check_output(["g++", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(libasan) or not os.path.exists(libasan):
        pytest.skip("no libasan in this toolchain")
    env = dict(os.environ, CSD_ORACLE_SANITIZE="1", ASAN_OPTIONS="detect_leaks=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    env["LD_PRELOAD"] = ":".join(x for x in (libasan, os.environ.get("LD_PRELOAD", "")) if x)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.abspath(__file__), "-x", "-q", "-p",
                          "no:cacheprovider"], cwd=root, env=env, capture_output=True, text=True, timeout=1500)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert " passed" in run.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail
