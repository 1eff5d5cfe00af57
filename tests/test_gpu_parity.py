"""GPU parity: the HIP library, called through its C-ABI, against the CPU
oracle on the same seeded inputs.  Bit-exact on match positions, edge tables,
draft tokens, draft lengths and accept lengths; scores within 1e-6 relative
(they are in fact the same exact integers rounded once to float)."""
import numpy as np
import pytest
import torch

from paper_2503_05330_amd import binding, synth
from replay import assert_step_equal, gpu_replay

pytestmark = pytest.mark.gpu


def oracle_step(oracle, tokens, probs, lens_t, k, L, alpha, mode, target=None):
    return oracle.draft_all(tokens, probs, lens_t, k, L, alpha, mode, target)


def check_dumps(oracle, ix, tokens, probs, lens_t, k, L, eps=0, rows=None):
    """Match sets and edge tables of every row (or of `rows`) at the index's current state.
    The edge tables come from the LDS-table builder (build_dag), whatever form of the walk the
    step kernel would choose for the row."""
    P, N, _ = tokens.shape
    je, moff = ix.dump_matches(k)
    duv, cs, eoff = ix.dump_edges(k, L)
    for r in (range(P * N) if rows is None else rows):
        p, i = divmod(r, N)
        want = oracle.matches(tokens[p], lens_t[p], i, k, eps=eps)
        assert np.array_equal(je[moff[r]:moff[r + 1]], want), "matches row %d" % r
        wduv, wcs = oracle.edges(tokens[p], None if probs is None else probs[p], lens_t[p], i, k, L, eps=eps)
        assert np.array_equal(duv[eoff[r]:eoff[r + 1]], wduv), "edge keys row %d" % r
        assert np.array_equal(cs[eoff[r]:eoff[r + 1]], wcs), "edge weights row %d" % r


SCAN, INDEX = binding.MATCH_SCAN, binding.MATCH_INDEX
ALL_VARIANTS = ((INDEX, "replay"), (INDEX, "calls"), (SCAN, "step"), (SCAN, "replay_unfused"))


def oracle_steps(oracle, tokens, probs, steps, k, L, alpha, mode, targets=None, **kw):
    """The oracle's outputs after steps[x] + 1 tokens per path, for all x, in one threaded call:
    {step: dict as draft_all returns it}."""
    P, N, _ = tokens.shape
    lens = np.empty((len(steps), P, N), dtype=np.int32)
    lens[:] = (np.asarray(steps, dtype=np.int32) + 1)[:, None, None]
    tg = None if targets is None else np.ascontiguousarray(targets[list(steps)])
    many = oracle.draft_many(tokens, probs, lens, k, L, alpha, mode, tg, **kw)
    return {t: {key: (None if val is None else val[x]) for key, val in many.items()}
            for x, t in enumerate(steps)}


def run_config(oracle, w, use_probs, alpha, mode, check_every=1, dump_at=(), accept=False,
               variants=ALL_VARIANTS, max_edits=0):
    """Replays the workload once per (matcher, call pattern) variant and compares every
    checked step of every variant with the oracle (computed once, all steps in one threaded
    call)."""
    tokens, probs = synth.make_paths(w)
    if not use_probs:
        probs = None
    T = w.max_len
    targets = None
    if accept:
        targets = np.stack([synth.make_noisy_targets(w, tokens, t + 1, w.draft_len) for t in range(T)])
    steps = sorted(set(list(range(0, T, check_every)) + [T - 1]))
    print("oracle", w.name, len(steps), "steps", flush=True)
    want = oracle_steps(oracle, tokens, probs, steps, w.query_len, w.draft_len, alpha, mode, targets,
                        eps=max_edits)
    assert sum(int((x["draft_len"] > 0).sum()) for x in want.values()) > 0
    got = None
    for flags, how in variants:
        print("replay", w.name, "P,N,T", tokens.shape, "probs", use_probs, "alpha", alpha, "mode", mode,
              "flags", flags, "how", how, "max_edits", max_edits, flush=True)
        got = gpu_replay(tokens, probs, w.query_len, w.draft_len, alpha, mode, flags, targets=targets,
                         how=how, max_edits=max_edits)
        assert got["status"] == 0
        for t in steps:
            assert_step_equal(got, want[t], t, "%s flags=%d %s" % (w.name, flags, how))
    # intermediate results at chosen history lengths (fresh index, appended in one call)
    for flags in sorted(set(f for f, _ in variants)):
        for t in dump_at:
            print("dumps", w.name, "flags", flags, "history", t, flush=True)
            dev = torch.device("cuda:0")
            ix = binding.Index(w.n_problems, w.n_paths, T, w.vocab, w.query_len, w.draft_len, alpha,
                               mode, flags, device=dev, max_edits=max_edits)
            ix.append(torch.from_numpy(np.ascontiguousarray(tokens[:, :, :t])).to(dev),
                      None if probs is None else torch.from_numpy(np.ascontiguousarray(probs[:, :, :t])).to(dev),
                      None, t)
            lens_t = np.full(tokens.shape[:2], t, dtype=np.int32)
            check_dumps(oracle, ix, tokens, probs, lens_t, w.query_len, w.draft_len, eps=max_edits)
            for q in range(1, w.query_len):      # shorter queries at full history: many more matches
                if max_edits:
                    break
                je, moff = ix.dump_matches(q)
                for p in range(min(w.n_problems, 2)):
                    for i in range(w.n_paths):
                        r = p * w.n_paths + i
                        assert np.array_equal(je[moff[r]:moff[r + 1]],
                                              oracle.matches(tokens[p], lens_t[p], i, q))
            assert ix.status() == 0
    return got


def test_c1_every_step_all_modes(oracle):
    w = synth.WORKLOADS["C1"]
    run_config(oracle, w, True, 1.0, 0, dump_at=(5, 100, 256))
    run_config(oracle, w, True, 0.5, 1)
    run_config(oracle, w, False, 1.0, 0, dump_at=(256,))
    run_config(oracle, w, True, 0.0, 0)


def test_c2_every_step(oracle):
    w = synth.WORKLOADS["C2"]
    run_config(oracle, w, True, 1.0, 0, dump_at=(511, 1024))
    run_config(oracle, w, False, 1.0, 1, variants=((INDEX, "step"), (SCAN, "calls")))


def test_c2_match_sets_and_edge_tables_along_the_replay(oracle):
    """Match sets (Eq. 3) and edge tables (Eq. 5) of every row after every 64th step of the C2
    replay, from the index as the replay itself leaves it (not from a freshly filled one), under
    both matchers."""
    w = synth.WORKLOADS["C2"]
    tokens, probs = synth.make_paths(w)
    T, k, L = w.max_len, w.query_len, w.draft_len
    dev = torch.device("cuda:0")
    d_tok = torch.from_numpy(np.ascontiguousarray(tokens.transpose(2, 0, 1))).to(dev)
    d_pr = torch.from_numpy(np.ascontiguousarray(probs.transpose(2, 0, 1))).to(dev)
    for flags in (INDEX, SCAN):
        ix = binding.Index(1, w.n_paths, T, w.vocab, k, L, 1.0, 0, flags, device=dev)
        for t0 in range(0, T, 64):
            ix.replay(64, d_tok[t0:t0 + 64], d_pr[t0:t0 + 64], k, L)
            print("dumps along the replay: flags", flags, "history", t0 + 64, flush=True)
            lens_t = np.full((1, w.n_paths), t0 + 64, dtype=np.int32)
            check_dumps(oracle, ix, tokens, probs, lens_t, k, L)
        assert ix.status() == 0


def test_c3_every_step(oracle):
    w = synth.WORKLOADS["C3"]
    run_config(oracle, w, True, 1.0, 0, check_every=1, dump_at=(2048,),
               variants=((INDEX, "replay"), (SCAN, "replay")))


def test_c4_batched_problems(oracle):
    w = synth.WORKLOADS["C4"]
    run_config(oracle, w, True, 1.0, 0, check_every=1, dump_at=(1024,),
               variants=((INDEX, "replay"), (SCAN, "replay"), (INDEX, "replay_unfused")))


def test_c5_sparse_matches_with_accept(oracle):
    w = synth.WORKLOADS["C5"]
    got = run_config(oracle, w, True, 1.0, 0, check_every=1, dump_at=(4096,), accept=True,
                     variants=((INDEX, "replay"), (SCAN, "replay"), (INDEX, "calls")))
    assert got["accept_len"].max() > 0


def test_ragged_appends(oracle):
    for name in ("C1", "C2"):
        w = synth.WORKLOADS[name]
        tokens, probs = synth.make_paths(w)
        steps = w.max_len // 2
        counts = synth.make_ragged_counts(w, 4, steps)
        want = None
        for flags, how in ((INDEX, "step"), (INDEX, "calls"), (SCAN, "step"), (SCAN, "calls")):
            got = gpu_replay(tokens, probs, w.query_len, w.draft_len, flags=flags, steps=steps,
                             counts=counts, n_per_step=4, how=how)
            assert got["status"] in (0, binding.STATUS_CAPACITY)
            assert got["lens"].max() > got["lens"].min()
            if want is None:
                want = [oracle_step(oracle, tokens, probs, got["lens"][t], w.query_len, w.draft_len, 1.0, 0)
                        for t in range(steps)]
            for t in range(steps):
                assert_step_equal(got, want[t], t, "ragged %s flags=%d %s" % (name, flags, how))


def test_long_ragged_steps_around_the_fused_limit(oracle):
    """Steps of up to 63, 64 and 65 tokens per path: the index matcher fuses up to 64 (a lane per
    new position, many more new positions than old ones in the first steps) and appends longer
    steps in a launch of their own; with counts from 0 to n, vocabulary 6, so that the appended
    positions themselves match."""
    rng = np.random.default_rng(6465)
    P, N, T, V, k, L = 2, 5, 400, 6, 2, 8
    motif = rng.integers(0, V, size=9)
    tokens = np.zeros((P, N, T), dtype=np.int32)
    for p in range(P):
        for j in range(N):
            seq = np.tile(np.roll(motif, int(rng.integers(0, 9))), T // 9 + 1)[:T]
            tokens[p, j] = np.where(rng.random(T) < 0.08, rng.integers(0, V, size=T), seq)
    probs = (rng.integers(1, 17, size=tokens.shape) / 16.0).astype(np.float32)
    for n in (63, 64, 65):
        steps = 8
        counts = rng.integers(0, n + 1, size=(steps, P, N)).astype(np.int32)
        for flags, mode in ((INDEX, 0), (INDEX | binding.INCLUDE_SELF, 1), (SCAN, 0)):
            what = "n%d flags%d mode%d" % (n, flags, mode)
            print(what, flush=True)
            got = gpu_replay(tokens, probs, k, L, 0.5, mode, flags, steps=steps, counts=counts,
                             n_per_step=n, how="step")
            assert got["status"] in (0, binding.STATUS_CAPACITY), what
            for t in range(steps):
                want = oracle.draft_all(tokens, probs, got["lens"][t], k, L, 0.5, mode,
                                        include_self=bool(flags & binding.INCLUDE_SELF))
                assert_step_equal(got, want, t, what)


def test_query_len_longer_and_shorter_than_history(oracle):
    """q = min(k, len_i): the first steps of a replay use 1- and 2-token queries; also
    draft() with every query_len up to the maximum on a full history."""
    w = synth.scaled(synth.WORKLOADS["C2"], max_len=300, query_len=8, draft_len=32)
    tokens, probs = synth.make_paths(w)
    dev = torch.device("cuda:0")
    lens = np.full((1, w.n_paths), 300, dtype=np.int32)
    for flags in (INDEX, SCAN):
        ix = binding.Index(1, w.n_paths, 300, w.vocab, 8, 32, 0.25, 0, flags, device=dev)
        ix.append(torch.from_numpy(tokens).to(dev), torch.from_numpy(probs).to(dev), None, 300)
        for k in range(1, 9):
            for L in (1, 7, 32):
                out = ix.draft(k, L)
                want = oracle.draft_all(tokens, probs, lens, k, L, 0.25, 0)
                got = dict(draft=out["tokens"].cpu().numpy()[None], draft_len=out["length"].cpu().numpy()[None],
                           token_scores=out["token_scores"].cpu().numpy()[None],
                           path_scores=out["path_scores"].cpu().numpy()[None])
                assert_step_equal(got, want, 0, "flags=%d k=%d L=%d" % (flags, k, L))


def _one_shot(oracle, paths, probs, k, L, alpha=1.0, mode=0, flags=None, fused=False, pool_mode=0, eps=0):
    """Appends whole (possibly ragged) paths in one call and compares one draft; by default
    under both matchers (returns the last index)."""
    if flags is None:
        for f in (SCAN, INDEX):
            for fu in (False, True):
                if eps and f == INDEX and k < 2:
                    continue                    # one-token queries with one edit are found by scan
                res = _one_shot(oracle, paths, probs, k, L, alpha, mode, f, fu, pool_mode, eps)
        return res
    N = len(paths)
    T = max(len(p) for p in paths)
    tok = np.zeros((1, N, T), dtype=np.int32)
    pr = np.ones((1, N, T), dtype=np.float32) if probs is not None else None
    cnt = np.zeros((1, N), dtype=np.int32)
    for j, p in enumerate(paths):
        tok[0, j, :len(p)] = p
        cnt[0, j] = len(p)
        if probs is not None:
            pr[0, j, :len(p)] = probs[j]
    dev = torch.device("cuda:0")
    ix = binding.Index(1, N, T, int(tok.max()) + 1, max(k, 1), L, alpha, mode, flags, device=dev,
                       max_edits=eps, pool_mode=pool_mode)
    d_tok, d_pr, d_cnt = (torch.from_numpy(tok).to(dev), None if pr is None else torch.from_numpy(pr).to(dev),
                          torch.from_numpy(cnt).to(dev))
    if fused:      # the whole history arrives in the very step that drafts from it
        out = ix.step(d_tok, d_pr, d_cnt, T, k, L)
    else:
        ix.append(d_tok, d_pr, d_cnt, T)
        out = ix.draft(k, L)
    want = oracle.draft_all(tok, pr, cnt, k, L, alpha, mode, eps=eps, pool_mode=pool_mode)
    got = dict(draft=out["tokens"].cpu().numpy()[None], draft_len=out["length"].cpu().numpy()[None],
               token_scores=out["token_scores"].cpu().numpy()[None],
               path_scores=out["path_scores"].cpu().numpy()[None])
    assert_step_equal(got, want, 0)
    assert ix.status() == 0
    return ix, tok, pr, cnt, want


def test_degenerate_constant_paths_streaming_tier(oracle):
    """All tokens equal: (N-1)(T-q) matches, far more than the on-chip match list holds."""
    for N, T in ((4, 700), (16, 1024)):
        ix, tok, pr, cnt, want = _one_shot(oracle, [[5] * T] * N, None, 3, 8)
        assert (want["draft_len"] == 8).all()
        assert want["token_scores"][0, 0, 0] == (N - 1) * (T - 3)
        je, off = ix.dump_matches(3, cap=N * N * T)
        assert off[-1] == N * (N - 1) * (T - 3)
        assert np.array_equal(je[off[1]:off[2]], oracle.matches(tok[0], cnt[0], 1, 3))


def test_many_distinct_edges_overflow_the_lds_table(oracle):
    """A frequent query token followed by random continuations: thousands of distinct
    DAG edges force the layer-by-layer tier, and (second case) its token classes."""
    rng = np.random.default_rng(5)
    for reps, n_paths in ((120, 5), (700, 5)):
        paths, probs = [], []
        for j in range(n_paths):
            body = rng.integers(10, 4000, size=(reps, 6))
            body[:, 0] = 7                                  # the query token recurs every 6 tokens
            paths.append(body.reshape(-1).tolist())
            probs.append((rng.integers(1, 9, size=reps * 6) / 8.0).tolist())
        paths[0] = paths[0][:-5]                            # path 0 ends with the query token 7
        probs[0] = probs[0][:-5]
        for mode in (0, 1):
            _one_shot(oracle, paths, probs, 1, 6, 0.5, mode)


def test_hundreds_of_matches_node_weights_tabulated_first(oracle):
    """Rows of 65 .. 1024 matches in scan mode take the walk that tabulates Eq. 5's node weights
    of all layers first: with few distinct continuations (every instance of a layer on a handful
    of keys), with thousands of distinct ones, with so many that the key set gives up and the
    row is walked layer by layer after all (1000 matches x 8 layers of random tokens), with
    token ids too large for the packed rank, with long drafts, and under edge scoring (which
    never tabulates).  The query token recurs at the head of every block."""
    rng = np.random.default_rng(77)
    for reps, n_paths, lo, hi, L in ((150, 5, 10, 4000, 8), (250, 5, 10, 4000, 8), (150, 5, 10, 3_000_000, 8),
                                     (60, 5, 10, 14, 32), (200, 5, 10, 13, 8), (17, 5, 10, 200, 8)):
        paths, probs = [], []
        for j in range(n_paths):
            body = rng.integers(lo, hi, size=(reps, L + 1))
            body[:, 0] = 7
            paths.append(body.reshape(-1).tolist())
            probs.append((rng.integers(0, 9, size=reps * (L + 1)) / 8.0).tolist())
        paths[0] = paths[0][:-L]                            # path 0 ends with the query token 7
        probs[0] = probs[0][:-L]
        for mode, alpha in ((0, 0.5), (1, 0.5), (0, 1.0), (0, 0.0)):
            print("reps", reps, "tokens below", hi, "L", L, "mode", mode, "alpha", alpha, flush=True)
            for fused in (False, True):
                _one_shot(oracle, paths, probs, 1, L, alpha, mode, SCAN, fused)


def test_one_edit_through_the_index_rows_of_many_distinct_continuations(oracle):
    """One-edit matching through the variant index with rows of 60 .. 200 matches whose
    continuations mostly differ: more than the lane-per-match walks of the one-wave kernel
    take, so the node weights are tabulated first (or, where that does not apply or the key set
    fills up, the per-layer tables are built).  The two query tokens recur at the head of every
    block; some blocks carry a substituted first token (a one-edit match)."""
    rng = np.random.default_rng(78)
    for reps, hi, L in ((16, 4000, 8), (30, 4000, 8), (30, 4000, 16), (50, 14, 8), (30, 3_000_000, 8), (56, 4000, 8)):
        paths, probs = [], []
        for j in range(5):
            body = rng.integers(10, hi, size=(reps, L + 2))
            body[:, 0] = np.where(rng.random(reps) < 0.25, 8, 7)
            body[:, 1] = 9
            paths.append(body.reshape(-1).tolist())
            probs.append((rng.integers(0, 9, size=reps * (L + 2)) / 8.0).tolist())
        paths[0] = paths[0][:-L]                            # path 0 ends with the query tokens 7 9
        probs[0] = probs[0][:-L]
        paths[0][-2] = 7
        for mode, alpha in ((0, 0.5), (1, 0.5), (0, 1.0)):
            print("reps", reps, "tokens below", hi, "L", L, "mode", mode, "alpha", alpha, flush=True)
            for fused in (False, True):
                _one_shot(oracle, paths, probs, 2, L, alpha, mode, INDEX, fused, eps=1)


def test_random_rows_of_hundreds_of_matches(oracle):
    """Differential test of the walks that serve 65 .. 1024 matches per row (and the hand-overs
    to the tiers on both sides): random paths over a few symbols, so that a short query recurs
    hundreds of times with continuations that agree in part; geometry, query and draft length,
    alpha, scoring, tolerance and matcher vary together."""
    rng = np.random.default_rng(4711)
    seen = []
    for case in range(36):
        N = int(rng.integers(2, 9))
        T = int(rng.integers(120, 700))
        V = int(rng.choice([2, 3, 4, 6, 12]))
        k = int(rng.integers(1, 4))
        L = int(rng.choice([1, 3, 8, 10, 16, 32]))
        alpha = float(rng.choice([0.0, 0.3, 1.0]))
        mode = int(rng.integers(0, 2))
        eps = int(rng.integers(0, 2))
        flags = SCAN if (eps and k < 2) or rng.random() < 0.6 else INDEX
        fused = bool(rng.integers(0, 2))
        base = rng.integers(0, V, size=T)
        paths, probs = [], []
        for j in range(N):
            n = int(rng.integers(T // 2, T + 1))
            noise = rng.random(n) < rng.choice([0.0, 0.05, 0.3])
            paths.append(np.where(noise, rng.integers(0, V, size=n), base[:n]).tolist())
            probs.append((rng.integers(0, 17, size=n) / 16.0).tolist())
        print("case", case, "N", N, "T", T, "V", V, "k", k, "L", L, "alpha", alpha, "mode", mode, "eps", eps,
              "flags", flags, "fused", fused, flush=True)
        ix, tok, pr, cnt, want = _one_shot(oracle, paths, probs, k, L, alpha, mode, flags, fused, eps=eps)
        seen.append(int(max(len(oracle.matches(tok[0], cnt[0], i, k, eps)) for i in range(N))))
    assert sum(65 <= m <= 1024 for m in seen) >= 12 and any(m > 1024 for m in seen), sorted(seen)


def test_empty_and_tiny_paths(oracle):
    _one_shot(oracle, [[1, 2, 3], [], [3], [2, 3, 9, 2, 3]], None, 2, 4)
    _one_shot(oracle, [[4], [4, 4], [9]], [[0.5], [0.25, 1.0], [1.0]], 3, 3)
    # nothing appended at all: every draft is empty
    dev = torch.device("cuda:0")
    ix = binding.Index(2, 3, 16, 10, 2, 4, device=dev)
    out = ix.draft(2, 4)
    assert (out["length"].cpu().numpy() == 0).all() and (out["tokens"].cpu().numpy() == -1).all()
    assert (out["token_scores"].cpu().numpy() == 0).all() and (out["path_scores"].cpu().numpy() == 0).all()


def test_hand_worked_example_on_gpu(oracle):
    import json, os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_worked_dag.json")))
    for mode in (0, 1):
        ix, tok, pr, cnt, want = _one_shot(oracle, g["paths"], None, g["k"], g["L"], 1.0, mode)
        assert want["draft"][0, 0].tolist() == g["no_probs"]["mode%d" % mode]["draft"]
    je, off = ix.dump_matches(g["k"])
    assert je[off[0]:off[1]].tolist() == g["matches"]
    duv, cs, eoff = ix.dump_edges(g["k"], g["L"])
    assert [r + [int(c[0])] for r, c in zip(duv[eoff[0]:eoff[1]].tolist(), cs[eoff[0]:eoff[1]])] == g["edges_counts"]


def test_status_bits_and_reset(oracle):
    dev = torch.device("cuda:0")
    ix = binding.Index(1, 2, 8, 100, 2, 4, device=dev)
    t = torch.tensor([[[1, 2, 3, 4, 5, 6], [1, 2, 3, 4, 5, 6]]], dtype=torch.int32, device=dev)
    ix.append(t, None, None, 6)
    assert ix.status() == 0
    with pytest.raises(binding.CsdError) as e:           # 6 + 6 > 8 and the host knows it
        ix.append(t, None, None, 6)
    assert e.value.code == binding.ERR_CAPACITY
    cnt = torch.tensor([[1, 6]], dtype=torch.int32, device=dev)
    ix.append(t, None, cnt, 6)                            # path 1 is clipped by the kernel
    assert ix.status() == binding.STATUS_CAPACITY
    ix.reset()
    assert ix.status() == 0
    bad = torch.tensor([[[100], [-1]]], dtype=torch.int32, device=dev)
    ix.append(bad, None, None, 1)
    assert ix.status() == binding.STATUS_TOKEN_RANGE
    ix.reset()
    # after reset the index behaves like a new one
    ix.append(torch.tensor([[[7, 8, 9, 7], [7, 8, 9, 7]]], dtype=torch.int32, device=dev)[:, :, :4].contiguous(), None, None, 4)
    out = ix.draft(1, 3)
    assert out["tokens"].cpu().numpy()[0, 0].tolist() == [8, 9, 7]


def test_table_full_status_needs_a_constructed_input(oracle):
    """CSD_STATUS_TABLE_FULL, the one documented inexact path: a layer whose continuation tokens
    include more distinct ids of ONE hash class (bits 12..31 of id * 0x9E3779B1) than the
    bounded-memory tier's table holds.  Ids below 2^24 cannot do that; 300 ids below 2^29 built
    to share a class do, in a launch of 2048 rows (whose on-chip table has 256 slots): the draft
    of that row ends early and the status bit is raised.  The scan kernel walks the same row one
    thread per match, without tables, and agrees with the oracle."""
    inv = pow(0x9E3779B1, -1, 1 << 32)
    base = 12345
    ids = []
    for delta in range(-4095, 4096):
        v = (base + delta * inv) % (1 << 32)
        if v < (1 << 29) - 1 and ((v * 0x9E3779B1) % (1 << 32)) >> 12 == ((base * 0x9E3779B1) % (1 << 32)) >> 12:
            ids.append(v)
    ids = sorted(set(ids))[:300]
    assert len(ids) == 300
    a = 7
    T = 2 * len(ids)
    P = 1024                                       # 2048 rows: the one-wave kernel's small layout
    dev = torch.device("cuda:0")
    for vocab, successors in (((1 << 29) - 1, np.array(ids)), (1 << 24, np.arange(100, 400) * 9973 % (1 << 24))):
        tok = np.zeros((P, 2, T), dtype=np.int32)
        tok[:, 0, :3] = [3, 4, a]
        tok[:, 1, 0::2] = 5
        tok[:, 1, 1::2] = 6
        tok[0, 1, 0::2] = a                        # problem 0: `a` followed by 300 different tokens
        tok[0, 1, 1::2] = successors
        cnt = np.tile(np.array([[3, T]], dtype=np.int32), (P, 1))
        want = oracle.draft_all(tok[:1], None, cnt[:1], 1, 4)
        assert want["draft_len"][0, 0] == 4        # 300 successors of weight 1: the lowest id, then `a`, ..
        for flags in (SCAN, INDEX):
            ix = binding.Index(P, 2, T, vocab, 1, 4, 1.0, 0, flags, device=dev)
            ix.append(torch.from_numpy(tok).to(dev), None, torch.from_numpy(cnt).to(dev), T)
            out = ix.draft(1, 4)
            status = ix.status()
            got_len, got_tok = out["length"].cpu().numpy(), out["tokens"].cpu().numpy()
            assert (got_len[1:] == 0).all()        # the other problems: `a` occurs nowhere else
            if flags == INDEX and vocab > (1 << 24):
                assert status == binding.STATUS_TABLE_FULL and got_len[0, 0] == 0
            else:
                assert status == 0 and got_len[0, 0] == 4
                assert got_tok[0, 0].tolist() == want["draft"][0, 0].tolist()
            del ix, out
        torch.cuda.empty_cache()


def test_determinism_two_runs_identical(oracle):
    w = synth.WORKLOADS["C2"]
    tokens, probs = synth.make_paths(w)
    a = gpu_replay(tokens, probs, 3, 8, steps=400)
    b = gpu_replay(tokens, probs, 3, 8, steps=400)
    for key in ("draft", "draft_len", "token_scores", "path_scores"):
        assert np.array_equal(a[key], b[key])
    # the sliced scan hands matches over in whatever order the workgroups finish: the sums are
    # exact integers, so the results must still be the same bits, run after run
    runs = [gpu_replay(tokens, probs, 3, 8, flags=SCAN, steps=300, how="replay", max_edits=1,
                       pool_mode=pool) for pool in (0, 1, 2) for _ in range(3)]
    for pool in range(3):
        for other in runs[3 * pool + 1:3 * pool + 3]:
            for key in ("draft", "draft_len", "token_scores", "path_scores"):
                assert np.array_equal(runs[3 * pool][key], other[key])


def test_many_paths_beyond_one_wave_and_length_cache(oracle):
    """N = 300 paths: more than one 64-lane chunk of heads and more than the 256 lengths
    cached on chip; ragged lengths; both matchers; fused single-token steps and one-shot."""
    rng = np.random.default_rng(11)
    N, T, k, L = 300, 40, 2, 4
    base = rng.integers(0, 30, size=T)
    tokens = np.tile(base, (1, N, 1)).astype(np.int32)
    flip = rng.random(tokens.shape) < 0.2
    tokens[flip] = rng.integers(0, 30, size=int(flip.sum()))
    probs = rng.random(tokens.shape).astype(np.float32)
    for flags, how in ((INDEX, "replay"), (SCAN, "step"), (INDEX, "calls")):
        got = gpu_replay(tokens, probs, k, L, 0.7, 0, flags, how=how)
        assert got["status"] == 0
        for t in range(0, T, 3):
            want = oracle.draft_all(tokens, probs, got["lens"][t], k, L, 0.7, 0)
            assert_step_equal(got, want, t, "N=300 flags=%d %s" % (flags, how))
    ix = got["index"]
    je, off = ix.dump_matches(k, cap=1 << 22)
    lens = got["lens"][-1]
    for i in (0, 63, 64, 255, 256, 299):
        assert np.array_equal(je[off[i]:off[i + 1]], oracle.matches(tokens[0], lens[0], i, k))


def test_maximum_positions_per_problem(oracle):
    """N * max_len = 2^24, the largest geometry the library accepts: positions pack into
    24 + bits, the index has 2^21 buckets.  Only a few tokens are appended (the oracle scans)."""
    N, T, k, L = 4096, 4096, 3, 4
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(3)
    n = 6
    step = rng.integers(0, 5, size=(1, N, n)).astype(np.int32)
    for flags in (INDEX, SCAN):
        ix = binding.Index(1, N, T, 5, k, L, 1.0, 0, flags, device=dev)
        ix.append(torch.from_numpy(step).to(dev), None, None, n)
        out = ix.draft(k, L)
        tok = np.zeros((1, N, T), dtype=np.int32)
        tok[:, :, :n] = step
        lens = np.full((1, N), n, dtype=np.int32)
        rows = [0, 1, 63, 64, 2047, 4095]
        got_tok = out["tokens"].cpu().numpy()
        got_len = out["length"].cpu().numpy()
        got_ts = out["token_scores"].cpu().numpy()
        for i in rows:
            d, nd, ts, ps = oracle.draft(tok[0], None, lens[0], i, k, L)
            assert got_len[0, i] == nd and got_tok[0, i].tolist() == d.tolist(), (flags, i)
            np.testing.assert_allclose(got_ts[0, i], ts, rtol=1e-6)
        assert ix.status() == 0
        del ix, out
        torch.cuda.empty_cache()


# ---------------------------------------------------------------- fuzzy suffix matching (Eq. 4, one edit)
def _fuzzy_replay(oracle, w, check_every, hows, dump_at=(), edges=True):
    tokens, probs = synth.make_paths(w)
    T, k, L = w.max_len, w.query_len, w.draft_len
    steps = sorted(set(list(range(0, T, check_every)) + [0, 1, 2, 3, T - 1]))
    want = {t: oracle.draft_all(tokens, probs, np.full(tokens.shape[:2], t + 1, dtype=np.int32), k, L,
                                1.0, 0, eps=1) for t in steps}
    exact_nonempty = sum(int((oracle.draft_all(tokens, probs, np.full(tokens.shape[:2], t + 1, dtype=np.int32),
                                               k, L, 1.0, 0)["draft_len"] > 0).sum()) for t in steps[::4])
    fuzzy_nonempty = sum(int((want[t]["draft_len"] > 0).sum()) for t in steps[::4])
    assert fuzzy_nonempty > exact_nonempty           # the tolerance finds more
    for flags, how in hows:          # INDEX: the variant index; SCAN: exhaustive comparison
        print("fuzzy replay", w.name, flags, how, flush=True)
        got = gpu_replay(tokens, probs, k, L, 1.0, 0, flags, how=how, max_edits=1)
        assert got["status"] == 0
        for t in steps:
            assert_step_equal(got, want[t], t, "fuzzy %s %d %s" % (w.name, flags, how))
    dev = torch.device("cuda:0")
    for flags, t in [(f, t) for f in (INDEX, SCAN) for t in dump_at]:
        ix = binding.Index(w.n_problems, w.n_paths, T, w.vocab, k, L, 1.0, 0, flags, device=dev, max_edits=1)
        ix.append(torch.from_numpy(np.ascontiguousarray(tokens[:, :, :t])).to(dev),
                  torch.from_numpy(np.ascontiguousarray(probs[:, :, :t])).to(dev), None, t)
        lens_t = np.full(tokens.shape[:2], t, dtype=np.int32)
        for q in range(1, k + 1):
            je, moff = ix.dump_matches(q, cap=1 << 22)
            for i in range(w.n_paths):
                assert np.array_equal(je[moff[i]:moff[i + 1]], oracle.matches(tokens[0], lens_t[0], i, q, 1)), (q, i)
        if not edges:        # rows whose tables exceed the on-chip tier are not dumpable
            continue
        duv, cs, eoff = ix.dump_edges(k, L)
        for i in range(w.n_paths):
            wduv, wcs = oracle.edges(tokens[0], probs[0], lens_t[0], i, k, L, 1)
            assert np.array_equal(duv[eoff[i]:eoff[i + 1]], wduv) and np.array_equal(cs[eoff[i]:eoff[i + 1]], wcs)


def test_fuzzy_c1_every_step(oracle):
    _fuzzy_replay(oracle, synth.WORKLOADS["C1"], 1,
                  ((INDEX, "replay"), (INDEX, "calls"), (SCAN, "replay"), (SCAN, "calls")), dump_at=(7, 256))


def test_fuzzy_c2_sampled_steps(oracle):
    _fuzzy_replay(oracle, synth.WORKLOADS["C2"], 32, ((INDEX, "replay"), (SCAN, "replay"), (INDEX, "step")),
                  dump_at=(300,), edges=False)


def test_fuzzy_c3_longer_query_through_the_index(oracle):
    # query of 4 tokens: five gram variants per position, the fifth filed by the general insert
    _fuzzy_replay(oracle, synth.scaled(synth.WORKLOADS["C3"], max_len=512), 16, ((INDEX, "replay"),),
                  dump_at=(200,), edges=False)


def _fuzzy_sampled(oracle, w, steps, variants, dump=None):
    """One-edit replay of a whole workload compared with the (threaded) oracle at the sampled
    steps; dump = (history length, rows): match sets of those rows at that length."""
    tokens, probs = synth.make_paths(w)
    T, k, L = w.max_len, w.query_len, w.draft_len
    steps = sorted(set(t for t in steps if 0 <= t < T))
    print("oracle, one edit:", w.name, tokens.shape, len(steps), "steps", flush=True)
    want = oracle_steps(oracle, tokens, probs, steps, k, L, 1.0, 0, eps=1)
    assert sum(int((x["draft_len"] > 0).sum()) for x in want.values()) > 0
    dev = torch.device("cuda:0")
    for flags, how in variants:
        print("one-edit replay", w.name, "flags", flags, how, flush=True)
        got = gpu_replay(tokens, probs, k, L, 1.0, 0, flags, how=how, max_edits=1)
        assert got["status"] == 0
        for t in steps:
            assert_step_equal(got, want[t], t, "one edit %s flags=%d %s" % (w.name, flags, how))
        if dump is not None:
            t, rows = dump
            ix = got["index"]
            ix.reset()
            ix.append(torch.from_numpy(np.ascontiguousarray(tokens[:, :, :t])).to(dev),
                      torch.from_numpy(np.ascontiguousarray(probs[:, :, :t])).to(dev), None, t)
            lens_t = np.full(tokens.shape[:2], t, dtype=np.int32)
            je, moff = ix.dump_matches(k, cap=1 << 23)
            for r in rows:
                p_, i_ = divmod(r, w.n_paths)
                assert np.array_equal(je[moff[r]:moff[r + 1]], oracle.matches(tokens[p_], lens_t[p_], i_, k, 1)), \
                    "one edit %s flags=%d matches of row %d" % (w.name, flags, r)
        del got
        torch.cuda.empty_cache()


def test_fuzzy_full_size_c3_c4_c5(oracle):
    """One-edit matching (Eq. 4, the tolerance of the paper's experiments) at the full size of
    C3 and C5 and on 8 problems of C4: sampled steps up to the full history, under the matcher
    CSD_MATCH_AUTO picks (the variant index for C3 and C5, the sliced scan for C4's three-token
    queries) and under the other one (C3, C5: the sliced scan; C4: the index)."""
    AUTO = binding.MATCH_AUTO
    w = synth.WORKLOADS["C3"]
    T = w.max_len
    _fuzzy_sampled(oracle, w, list(range(0, 6)) + list(range(127, T, 128)) + [T - 2, T - 1],
                   ((AUTO, "replay"), (SCAN, "replay")), dump=(700, range(0, w.n_paths, 5)))
    w = synth.WORKLOADS["C5"]
    T = w.max_len
    _fuzzy_sampled(oracle, w, list(range(0, 6)) + list(range(511, T, 512)) + [T - 2, T - 1],
                   ((AUTO, "replay"), (SCAN, "replay")), dump=(1500, range(0, w.n_paths, 9)))
    w = synth.scaled(synth.WORKLOADS["C4"], n_problems=8)
    T = w.max_len
    _fuzzy_sampled(oracle, w, list(range(0, 5)) + list(range(127, T, 128)) + [T - 1],
                   ((AUTO, "replay"), (INDEX, "replay")), dump=(400, range(0, 128, 11)))


def test_fuzzy_auto_picks_the_variant_index_and_many_rows(oracle):
    """One-edit matching where CSD_MATCH_AUTO takes the variant index (queries of 4 tokens, more
    than 128 rows), and launches of 2048 rows under both of AUTO's choices."""
    AUTO = binding.MATCH_AUTO

    def ws(w, flags):
        return binding.workspace_bytes(binding.Config(w.n_problems, w.n_paths, w.max_len, w.vocab, w.query_len,
                                                      w.draft_len, 1.0, 0, flags, 1, 0))
    w = synth.scaled(synth.WORKLOADS["C3"], n_problems=6, max_len=384, pool=96)       # 192 rows, k = 4
    assert ws(w, AUTO) == ws(w, INDEX) != ws(w, SCAN)          # AUTO's workspace holds the variant index
    _fuzzy_sampled(oracle, w, range(0, w.max_len, 8), ((AUTO, "replay"), (AUTO, "calls")),
                   dump=(200, range(0, 192, 17)))
    w = synth.scaled(synth.WORKLOADS["C3"], n_problems=128, n_paths=16, max_len=96, pool=24)   # 2048 rows, k = 4
    assert ws(w, AUTO) == ws(w, INDEX) != ws(w, SCAN)
    _fuzzy_sampled(oracle, w, range(0, w.max_len, 5), ((AUTO, "replay"),), dump=(96, range(0, 2048, 97)))
    w = synth.scaled(synth.WORKLOADS["C4"], n_problems=128, max_len=96, pool=24)      # 2048 rows, k = 3: scan
    assert ws(w, AUTO) == ws(w, SCAN) != ws(w, INDEX)
    _fuzzy_sampled(oracle, w, range(0, w.max_len, 5), ((AUTO, "replay"),), dump=(96, range(0, 2048, 97)))


def test_two_and_three_edits(oracle):
    """Eq. 4 with tolerances above one edit (always by scan): C1 at every step with match sets,
    C2 at sampled steps up to the full history, and random small configurations in which
    geometry, query and draft lengths, scoring, pool, options and call pattern vary together
    (queries no longer than the tolerance match every position)."""
    AUTO = binding.MATCH_AUTO
    dev = torch.device("cuda:0")
    for eps, how in ((2, "replay"), (3, "calls")):
        w = synth.WORKLOADS["C1"]
        tokens, probs = synth.make_paths(w)
        T, k, L = w.max_len, w.query_len, w.draft_len
        want = oracle_steps(oracle, tokens, probs, list(range(T)), k, L, 0.5, 0, eps=eps)
        for flags in (AUTO, SCAN):
            print("edits", eps, "C1 flags", flags, how, flush=True)
            got = gpu_replay(tokens, probs, k, L, 0.5, 0, flags, how=how, max_edits=eps)
            assert got["status"] == 0
            for t in range(T):
                assert_step_equal(got, want[t], t, "C1 %d edits flags=%d" % (eps, flags))
        ix = got["index"]
        lens_t = np.full((1, w.n_paths), T, dtype=np.int32)
        for q in range(1, k + 1):
            je, moff = ix.dump_matches(q, cap=1 << 22)
            for i in range(w.n_paths):
                assert np.array_equal(je[moff[i]:moff[i + 1]], oracle.matches(tokens[0], lens_t[0], i, q, eps)), (eps, q, i)
    w = synth.WORKLOADS["C2"]
    tokens, probs = synth.make_paths(w)
    steps = [0, 1, 2, 3, 5, 200, 500, 800, 1022, 1023]
    want = oracle_steps(oracle, tokens, probs, steps, w.query_len, w.draft_len, 1.0, 0, eps=2)
    print("edits 2 C2", flush=True)
    got = gpu_replay(tokens, probs, w.query_len, w.draft_len, 1.0, 0, AUTO, how="replay", max_edits=2)
    assert got["status"] == 0
    for t in steps:
        assert_step_equal(got, want[t], t, "C2 two edits")
    del got
    rng = np.random.default_rng(2503)
    for case in range(90):
        P, N = int(rng.integers(1, 3)), int(rng.integers(1, 7))
        T = int(rng.integers(4, 70))
        V = int(rng.choice([3, 5, 40]))
        k, L = int(rng.integers(1, 9)), int(rng.integers(1, 17))
        eps, pool_mode, mode = int(rng.integers(2, 4)), int(rng.integers(0, 3)), int(rng.integers(0, 2))
        flags = int(rng.choice([AUTO, SCAN]))
        include_self, backoff = bool(case % 3 == 1), bool(case % 4 == 2)
        flags |= (binding.INCLUDE_SELF if include_self else 0) | (binding.QUERY_BACKOFF if backoff else 0)
        n_per_step = int(rng.choice([1, 1, 3]))
        how = str(rng.choice(["calls", "step"]))
        segs = [rng.integers(0, V, size=int(rng.integers(2, 9))) for _ in range(4)]
        tokens = np.zeros((P, N, T), dtype=np.int32)
        for p in range(P):
            for j in range(N):
                seq = np.concatenate([segs[int(x)] for x in rng.integers(0, 4, size=T)])[:T]
                tokens[p, j] = np.where(rng.random(T) < 0.15, rng.integers(0, V, size=T), seq)
        probs = (rng.integers(1, 17, size=tokens.shape) / 16.0).astype(np.float32)
        steps_n = T // n_per_step
        counts = rng.integers(0, n_per_step + 1, size=(steps_n, P, N)).astype(np.int32) if n_per_step > 1 else None
        what = "edits case %d: P%d N%d T%d V%d k%d L%d eps%d pool%d mode%d flags%d n%d %s" % (
            case, P, N, T, V, k, L, eps, pool_mode, mode, flags, n_per_step, how)
        print(what, flush=True)
        got = gpu_replay(tokens, probs, k, L, 0.75, mode, flags, steps=steps_n, counts=counts,
                         n_per_step=n_per_step, how=how, max_edits=eps, pool_mode=pool_mode)
        assert got["status"] in (0, binding.STATUS_CAPACITY), what
        for t in range(steps_n):
            want_t = oracle.draft_all(tokens, probs, got["lens"][t], k, L, 0.75, mode, eps=eps, pool_mode=pool_mode,
                                      include_self=include_self, backoff=backoff)
            assert_step_equal(got, want_t, t, what)
    cfg = binding.Config(1, 4, 64, 100, 3, 5, 1.0, 0, INDEX, 2, 0)
    with pytest.raises(binding.CsdError):
        binding.workspace_bytes(cfg)                       # more than one edit through the index: not built


def test_fuzzy_small_cases(oracle):
    """Hand cases and tiny random inputs, including queries of one token (every position of
    every other path is within one edit of it) and matches at index 0."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(21)
    cases = [([[9, 1, 2, 3], [1, 7, 3, 50, 0, 1, 3, 51, 0, 1, 2, 8, 3, 52, 0, 4, 4, 4, 53]], 3, 4),
             ([[5], [6, 7, 8], [5, 5]], 1, 3), ([[1, 2], [2, 9], [], [1, 9, 2, 4]], 2, 2)]
    for _ in range(60):
        n = int(rng.integers(2, 5))
        cases.append(([rng.integers(0, 4, size=int(rng.integers(0, 20))).tolist() for _ in range(n)],
                      int(rng.integers(1, 5)), int(rng.integers(1, 6))))
    for _ in range(40):      # longer paths over three symbols, queries up to the maximum length
        n = int(rng.integers(2, 6))
        cases.append(([rng.integers(0, 3, size=int(rng.integers(0, 48))).tolist() for _ in range(n)],
                      int(rng.integers(1, 9)), int(rng.integers(1, 6))))
    for (paths, k, L), flags in [(c, f) for c in cases for f in ((INDEX if c[1] >= 2 else 0), SCAN)]:
        N, T = len(paths), max(1, max(len(p) for p in paths))
        tok = np.zeros((1, N, T), dtype=np.int32)
        cnt = np.array([[len(p) for p in paths]], dtype=np.int32)
        for j, p in enumerate(paths):
            tok[0, j, :len(p)] = p
        pr = (rng.integers(1, 9, size=tok.shape) / 8.0).astype(np.float32)
        ix = binding.Index(1, N, T, 64, k, L, 0.5, 0, flags, device=dev, max_edits=1)
        ix.append(torch.from_numpy(tok).to(dev), torch.from_numpy(pr).to(dev), torch.from_numpy(cnt).to(dev), T)
        out = ix.draft(k, L)
        want = oracle.draft_all(tok, pr, cnt, k, L, 0.5, 0, eps=1)
        got = dict(draft=out["tokens"].cpu().numpy()[None], draft_len=out["length"].cpu().numpy()[None],
                   token_scores=out["token_scores"].cpu().numpy()[None],
                   path_scores=out["path_scores"].cpu().numpy()[None])
        assert_step_equal(got, want, 0, "fuzzy case %s k=%d L=%d flags=%d" % (paths, k, L, flags))
        je, off = ix.dump_matches(k)
        for i in range(N):
            assert np.array_equal(je[off[i]:off[i + 1]], oracle.matches(tok[0], cnt[0], i, k, 1)), (paths, k, i)
        assert ix.status() == 0


def test_fuzzy_ragged_multi_token_steps(oracle):
    """Steps that append 0..4 tokens per path: the scan then meets positions whose compared
    tokens are partly history and partly this launch's input."""
    w = synth.WORKLOADS["C1"]
    tokens, probs = synth.make_paths(w)
    steps = w.max_len // 2
    counts = synth.make_ragged_counts(w, 4, steps)
    want = None
    for flags, how in ((SCAN, "step"), (SCAN, "calls"), (INDEX, "step"), (INDEX, "calls")):
        got = gpu_replay(tokens, probs, w.query_len, w.draft_len, flags=flags, steps=steps, counts=counts,
                         n_per_step=4, how=how, max_edits=1)
        assert got["status"] in (0, binding.STATUS_CAPACITY)
        if want is None:
            want = [oracle.draft_all(tokens, probs, got["lens"][t], w.query_len, w.draft_len, 1.0, 0, eps=1)
                    for t in range(steps)]
        for t in range(steps):
            assert_step_equal(got, want[t], t, "fuzzy ragged %d %s" % (flags, how))


# ---------------------------------------------------------------- tree and list pools (the ablation's variants)
@pytest.mark.parametrize("pool_mode", [binding.POOL_TREE, binding.POOL_LIST])
def test_pool_modes_replay(oracle, pool_mode):
    for name, every, variants in (("C1", 1, ((INDEX, "replay"), (SCAN, "step"), (INDEX, "calls"))),
                                  ("C2", 8, ((INDEX, "replay"), (SCAN, "replay")))):
        w = synth.WORKLOADS[name]
        tokens, probs = synth.make_paths(w)
        T, k, L = w.max_len, w.query_len, w.draft_len
        targets = np.stack([synth.make_noisy_targets(w, tokens, t + 1, L) for t in range(T)])
        steps = sorted(set(list(range(0, T, every)) + [T - 1]))
        for alpha, use_probs in ((1.0, True), (0.5, True), (1.0, False)):
            pr = probs if use_probs else None
            want = {t: oracle.draft_all(tokens, pr, np.full(tokens.shape[:2], t + 1, dtype=np.int32), k, L,
                                        alpha, 0, targets[t], pool_mode=pool_mode) for t in steps}
            if name == "C2":      # with enough candidates the pool structures give different drafts
                dag = {t: oracle.draft_all(tokens, pr, np.full(tokens.shape[:2], t + 1, dtype=np.int32), k, L,
                                           alpha, 0) for t in steps}
                assert sum(not np.array_equal(dag[t]["draft"], want[t]["draft"]) for t in dag) >= 5
            for flags, how in variants:
                print("pool", pool_mode, name, "alpha", alpha, "probs", use_probs, flags, how, flush=True)
                got = gpu_replay(tokens, pr, k, L, alpha, 0, flags, targets=targets, how=how,
                                 pool_mode=pool_mode)
                assert got["status"] == 0
                for t in steps:
                    assert_step_equal(got, want[t], t, "pool %d %s %d %s" % (pool_mode, name, flags, how))


@pytest.mark.parametrize("pool_mode", [binding.POOL_TREE, binding.POOL_LIST])
def test_pool_modes_small_and_degenerate_cases(oracle, pool_mode):
    rng = np.random.default_rng(99 + pool_mode)
    for _ in range(40):
        n = int(rng.integers(2, 6))
        paths = [rng.integers(0, 4, size=int(rng.integers(0, 40))).tolist() for _ in range(n)]
        probs = [(rng.integers(1, 9, size=len(p)) / 8.0).tolist() for p in paths]
        k, L = int(rng.integers(1, 5)), int(rng.integers(1, 9))
        _one_shot(oracle, paths, probs, k, L, float(rng.integers(0, 5)) / 4, 0, pool_mode=pool_mode,
                  eps=int(rng.integers(0, 2)))
    # more matches than the on-chip list holds: candidates are re-found and compare whole prefixes
    _one_shot(oracle, [[5] * 700] * 4, None, 3, 8, pool_mode=pool_mode)
    # a frequent query token followed by random continuations: one depth of the tree holds
    # thousands of distinct children
    body = [np.random.default_rng(j).integers(10, 4000, size=(500, 6)) for j in range(5)]
    for b in body:
        b[:, 0] = 7
    paths = [b.reshape(-1).tolist() for b in body]
    paths[0] = paths[0][:-5]
    _one_shot(oracle, paths, None, 1, 6, pool_mode=pool_mode)


# ---------------------------------------------------------------- the propose / verify / accept loop
def _accept_loop_case(oracle, w, n_steps, flags, eps=0, pool_mode=0, use_probs=True, warm=None,
                      min_scratch=False, steps_per_launch=1):
    tokens, probs = synth.make_paths(w)
    pr = probs if use_probs else None
    dev = torch.device("cuda:0")
    P, N, T, k, L = w.n_problems, w.n_paths, w.max_len, w.query_len, w.draft_len
    ix = binding.Index(P, N, T, w.vocab, k, L, 1.0, 0, flags, device=dev, max_edits=eps, pool_mode=pool_mode)
    if steps_per_launch > 1:
        ix.set_steps_per_launch(steps_per_launch)
    lens0 = np.zeros((P, N), np.int32)
    if warm is not None:                          # start from ragged, partly filled paths
        lens0 = warm.astype(np.int32)
        n0 = int(lens0.max())
        ix.append(torch.from_numpy(np.ascontiguousarray(tokens[:, :, :n0])).to(dev),
                  None if pr is None else torch.from_numpy(np.ascontiguousarray(pr[:, :, :n0])).to(dev),
                  torch.from_numpy(lens0).to(dev), n0)
    got = ix.accept_loop(n_steps, torch.from_numpy(tokens).to(dev),
                         None if pr is None else torch.from_numpy(pr).to(dev), k, L,
                         min_scratch=min_scratch)
    want = oracle.accept_loop(tokens, pr, lens0, k, L, n_steps, eps=eps, pool_mode=pool_mode)
    what = "%s flags=%d eps=%d pool=%d min_scratch=%d steps_per_launch=%d" % (
        w.name, flags, eps, pool_mode, min_scratch, steps_per_launch)
    print("accept loop", what, flush=True)
    assert np.array_equal(got["path_len"].cpu().numpy(), want["path_len"]), what
    assert np.array_equal(got["length"].cpu().numpy(), want["draft_len"]), what
    assert np.array_equal(got["tokens"].cpu().numpy(), want["draft"]), what
    assert np.array_equal(got["accept"].cpu().numpy(), want["accept_len"]), what
    assert ix.status() in (0, binding.STATUS_CAPACITY)
    return want


def test_accept_loop_diverging_path_lengths(oracle):
    c1, c2, c4 = (synth.WORKLOADS[n] for n in ("C1", "C2", "C4"))
    for flags in (INDEX, SCAN):
        want = _accept_loop_case(oracle, c1, 200, flags)
        assert want["accept_len"].sum() > 0 and want["path_len"][-1].max() > want["path_len"][-1].min()
        _accept_loop_case(oracle, c1, 120, flags, use_probs=False,
                          warm=np.array([[40, 3, 0, 17]]))
    # with the minimum of scratch memory the index matcher takes two launches per step
    _accept_loop_case(oracle, c1, 200, INDEX, min_scratch=True)
    _accept_loop_case(oracle, c1, 120, INDEX, use_probs=False, warm=np.array([[40, 3, 0, 17]]), min_scratch=True)
    # longer drafts (the loop's kernels for up to 16 and up to 32 draft tokens), more paths than the
    # staged step holds (N * (L + 1) > 1024), a query of 4
    c3 = synth.WORKLOADS["C3"]
    _accept_loop_case(oracle, synth.scaled(c3, max_len=300), 80, INDEX)
    _accept_loop_case(oracle, synth.scaled(c2, max_len=400, draft_len=16), 100, INDEX)
    _accept_loop_case(oracle, synth.scaled(c2, n_paths=64, max_len=200, draft_len=32), 60, INDEX)
    _accept_loop_case(oracle, c1, 200, SCAN, eps=1)
    _accept_loop_case(oracle, c1, 200, INDEX, pool_mode=binding.POOL_TREE)
    _accept_loop_case(oracle, c1, 200, SCAN, eps=1, pool_mode=binding.POOL_LIST)
    want = _accept_loop_case(oracle, c2, 700, INDEX)          # runs every path to its full length
    assert (want["final_len"] == c2.max_len).all()
    _accept_loop_case(oracle, synth.scaled(c4, n_problems=6), 60, INDEX)


def test_device_side_loops_many_steps_per_launch(oracle):
    """csd_set_steps_per_launch: csd_replay and csd_accept_loop with a device-side loop (one
    workgroup per problem, a wave per path, a barrier between steps) against the oracle at
    every step: whole replays in one launch and in chunks, 64 problems at once, the general
    kernels (tree and list pools, own history), longer drafts, a query of 4, no probabilities;
    and configurations the loop does not serve (32 paths; one-edit matching), which must fall
    back to a launch per step with the same results."""
    c1, c2, c3, c4 = (synth.WORKLOADS[n] for n in ("C1", "C2", "C3", "C4"))

    def replay_case(w, spl, use_probs=True, mode=0, pool_mode=0, flags=INDEX, eps=0, accept=True, **extras):
        tokens, probs = synth.make_paths(w)
        if not use_probs:
            probs = None
        T = w.max_len
        targets = np.stack([synth.make_noisy_targets(w, tokens, t + 1, w.draft_len) for t in range(T)]) if accept else None
        what = "device loop %s steps_per_launch=%d probs=%s mode=%d pool=%d flags=%d eps=%d" % (
            w.name, spl, use_probs, mode, pool_mode, flags, eps)
        print(what, flush=True)
        want = oracle_steps(oracle, tokens, probs, list(range(T)), w.query_len, w.draft_len, 0.75, mode, targets,
                            eps=eps, pool_mode=pool_mode, **extras)
        got = gpu_replay(tokens, probs, w.query_len, w.draft_len, 0.75, mode, flags, targets=targets, how="replay",
                         max_edits=eps, pool_mode=pool_mode, steps_per_launch=spl)
        assert got["status"] == 0
        for t in range(T):
            assert_step_equal(got, want[t], t, what)

    replay_case(c1, 1000)
    replay_case(c1, 7, use_probs=False, mode=1, accept=False)
    replay_case(c2, 1024)
    replay_case(c2, 100, mode=1)
    replay_case(c4, 256)
    replay_case(synth.scaled(c3, n_paths=16, max_len=600), 64)                      # query of 4, drafts of 10
    replay_case(synth.scaled(c2, max_len=300, draft_len=32), 300)
    replay_case(c1, 64, pool_mode=binding.POOL_TREE)
    replay_case(c1, 64, pool_mode=binding.POOL_LIST)
    replay_case(c1, 64, flags=INDEX | binding.INCLUDE_SELF, include_self=True)
    replay_case(synth.scaled(c3, max_len=200), 64)                                  # 32 paths: a launch per step
    replay_case(c1, 64, flags=binding.MATCH_AUTO, eps=1)                            # one edit: a launch per step
    for w, steps, spl in ((c1, 200, 50), (c2, 700, 700), (c2, 300, 64), (synth.scaled(c4, n_problems=6), 120, 30),
                          (synth.scaled(c2, max_len=400, draft_len=16), 100, 100),
                          (synth.scaled(c2, max_len=300, draft_len=32), 60, 8)):
        want = _accept_loop_case(oracle, w, steps, INDEX, steps_per_launch=spl)
        assert want["accept_len"].sum() > 0
    _accept_loop_case(oracle, c1, 120, INDEX, use_probs=False, warm=np.array([[40, 3, 0, 17]]), steps_per_launch=33)
    _accept_loop_case(oracle, c1, 200, INDEX, pool_mode=binding.POOL_TREE, steps_per_launch=64)


def test_large_batch_uses_the_small_on_chip_layout(oracle):
    """2048+ rows per launch run the one-wave kernel with its small LDS layout (more rows
    resident per CU).  Rows that do not fit it (two problems of constant paths: thousands of
    matches; rows with many distinct continuations) must take the bounded-memory tier."""
    w = synth.scaled(synth.WORKLOADS["C4"], n_problems=130, max_len=192)
    tokens, probs = synth.make_paths(w)
    tokens[7] = 11                                         # constant paths
    tokens[99, :, :] = tokens[99, :1, :]                   # identical paths
    rng = np.random.default_rng(3)
    tokens[50, :, ::3] = 5                                 # a frequent token with varied successors
    tokens[50, :, 1::3] = rng.integers(100, 130, size=tokens[50, :, 1::3].shape)
    assert tokens.shape[0] * tokens.shape[1] >= 2048
    T, k, L = w.max_len, w.query_len, w.draft_len
    targets = np.stack([synth.make_noisy_targets(w, tokens, t + 1, L) for t in range(T)])
    got = gpu_replay(tokens, probs, k, L, flags=INDEX, targets=targets, how="replay")
    assert got["status"] == 0
    for t in sorted(set(list(range(0, T, 24)) + [T - 1])):
        lens_t = np.full(tokens.shape[:2], t + 1, dtype=np.int32)
        want = oracle.draft_all(tokens, probs, lens_t, k, L, 1.0, 0, targets[t])
        assert_step_equal(got, want, t, "large batch")


def test_random_configurations_against_the_oracle(oracle):
    """Differential test over random small configurations: geometry, query and draft lengths,
    alpha, scoring, tolerance, pool structure, matcher and call pattern all vary together."""
    rng = np.random.default_rng(20250305)
    for case in range(250):
        P, N = int(rng.integers(1, 4)), int(rng.integers(1, 9))
        T = int(rng.integers(4, 90))
        V = int(rng.choice([3, 5, 40, 1000]))
        k, L = int(rng.integers(1, 9)), int(rng.integers(1, 33))
        eps, pool_mode, mode = int(rng.integers(0, 2)), int(rng.integers(0, 3)), int(rng.integers(0, 2))
        alpha = float(rng.integers(0, 9)) / 8
        flags = int(rng.choice([0, SCAN, INDEX]))
        if eps and flags == INDEX and k < 2:
            flags = 0
        include_self, backoff = bool(case % 3 == 1), bool(case % 4 == 2)   # the options, in a third / a quarter
        flags |= (binding.INCLUDE_SELF if include_self else 0) | (binding.QUERY_BACKOFF if backoff else 0)
        n_per_step = int(rng.choice([1, 1, 2, 5]))
        how = str(rng.choice(["calls", "step"]))
        use_probs = bool(rng.integers(0, 2))
        # paths: a few shared segments in random order, with noise, so that matches exist
        segs = [rng.integers(0, V, size=int(rng.integers(2, 9))) for _ in range(4)]
        tokens = np.zeros((P, N, T), dtype=np.int32)
        for p in range(P):
            for j in range(N):
                seq = np.concatenate([segs[int(x)] for x in rng.integers(0, 4, size=T)])[:T]
                noise = rng.random(T) < 0.1
                tokens[p, j] = np.where(noise, rng.integers(0, V, size=T), seq)
        probs = (rng.integers(1, 17, size=tokens.shape) / 16.0).astype(np.float32) if use_probs else None
        steps = T // n_per_step
        counts = rng.integers(0, n_per_step + 1, size=(steps, P, N)).astype(np.int32) if n_per_step > 1 else None
        what = "case %d: P%d N%d T%d V%d k%d L%d eps%d pool%d mode%d alpha%.3f flags%d n%d %s probs%d" % (
            case, P, N, T, V, k, L, eps, pool_mode, mode, alpha, flags, n_per_step, how, use_probs)
        print(what, flush=True)
        got = gpu_replay(tokens, probs, k, L, alpha, mode, flags, steps=steps, counts=counts,
                         n_per_step=n_per_step, how=how, max_edits=eps, pool_mode=pool_mode)
        assert got["status"] in (0, binding.STATUS_CAPACITY), what
        for t in range(steps):
            want = oracle.draft_all(tokens, probs, got["lens"][t], k, L, alpha, mode, eps=eps, pool_mode=pool_mode,
                                    include_self=include_self, backoff=backoff)
            assert_step_equal(got, want, t, what)


def test_match_counts_across_the_walk_forms(oracle):
    """Rows whose match counts sweep from 0 to hundreds within one replay, so that every form
    of the DAG walk (lanes = instances, lanes = one, two or four matches, LDS tables) and the
    hand-overs between them (8 | 9, 64 | 65, 128 | 129 and 256 | 257 matches at L = 8, fewer for
    longer drafts) are crossed many times,
    under both scoring modes, the tree pool, and both matchers."""
    rng = np.random.default_rng(8964)
    P, N, T, V, k = 2, 8, 240, 3, 2
    motif = rng.integers(0, V, size=12)
    tokens = np.zeros((P, N, T), dtype=np.int32)
    for p in range(P):
        for j in range(N):
            seq = np.tile(np.roll(motif, int(rng.integers(0, 12))), T // 12 + 1)[:T]
            noise = rng.random(T) < (0.02 + 0.03 * j)
            tokens[p, j] = np.where(noise, rng.integers(0, V, size=T), seq)
    probs = (rng.integers(1, 17, size=tokens.shape) / 16.0).astype(np.float32)
    seen = set()
    for L, mode, pool_mode, flags in [(8, 0, 0, INDEX), (8, 1, 0, INDEX), (8, 0, 1, INDEX), (8, 0, 0, SCAN),
                                      (8, 1, 1, SCAN), (1, 0, 0, INDEX), (4, 1, 0, INDEX), (16, 0, 0, INDEX),
                                      (32, 1, 0, INDEX), (32, 0, 1, INDEX), (16, 0, 0, SCAN)]:
        what = "L%d mode%d pool%d flags%d" % (L, mode, pool_mode, flags)
        print(what, flush=True)
        got = gpu_replay(tokens, probs, k, L, 0.75, mode, flags, pool_mode=pool_mode)
        for t in range(T):
            lens_t = np.full((P, N), t + 1, dtype=np.int32)
            want = oracle.draft_all(tokens, probs, lens_t, k, L, 0.75, mode, pool_mode=pool_mode)
            assert_step_equal(got, want, t, what)
    # the sweep is what the test is for: count the matches of every row and step on the CPU
    for t in range(k, T):
        for j in range(N):
            q = tokens[0, j, t - k + 1:t + 1]
            m = 0
            for o in range(N):
                if o == j:
                    continue
                h = tokens[0, o, :t + 1]
                for e in range(k, t + 1):
                    m += int(np.array_equal(h[e - k:e], q))
            seen.add(m if m <= 9 else 10 if m <= 64 else 65 if m <= 128 else 129 if m <= 256 else 257)
    assert {0, 1, 2, 4, 8, 9, 10, 65, 129, 257} <= seen, sorted(seen)


@pytest.mark.parametrize("include_self,backoff", [(True, False), (False, True), (True, True)])
def test_self_history_and_query_back_off(oracle, include_self, backoff):
    """The two retrieval-style options (neither is in the paper): every step of C1 and sampled
    steps of C2 under both matchers, all pools and both tolerances; one path on its own."""
    opts = (binding.INCLUDE_SELF if include_self else 0) | (binding.QUERY_BACKOFF if backoff else 0)
    w = synth.WORKLOADS["C1"]
    tokens, probs = synth.make_paths(w)
    T = w.max_len
    for matcher, eps, pool_mode, mode in [(0, 0, 0, 0), (SCAN, 0, 0, 1), (INDEX, 0, 0, 0), (INDEX, 0, 1, 0),
                                          (SCAN, 0, 2, 0), (SCAN, 1, 0, 0), (INDEX, 1, 0, 0), (0, 1, 1, 0)]:
        what = "C1 opts%d matcher%d eps%d pool%d mode%d" % (opts, matcher, eps, pool_mode, mode)
        print(what, flush=True)
        got = gpu_replay(tokens, probs, w.query_len, w.draft_len, 1.0, mode, matcher | opts, max_edits=eps,
                         pool_mode=pool_mode)
        for t in range(T):
            lens_t = np.full(tokens.shape[:2], t + 1, dtype=np.int32)
            want = oracle.draft_all(tokens, probs, lens_t, w.query_len, w.draft_len, 1.0, mode, eps=eps,
                                    pool_mode=pool_mode, include_self=include_self, backoff=backoff)
            assert_step_equal(got, want, t, what)
    w = synth.WORKLOADS["C2"]
    tokens, probs = synth.make_paths(w)
    for matcher in (0, INDEX):
        what = "C2 opts%d matcher%d" % (opts, matcher)
        print(what, flush=True)
        got = gpu_replay(tokens, probs, w.query_len, w.draft_len, 1.0, 0, matcher | opts, steps=400)
        for t in list(range(0, 40)) + list(range(43, 400, 17)):
            lens_t = np.full(tokens.shape[:2], t + 1, dtype=np.int32)
            want = oracle.draft_all(tokens, probs, lens_t, w.query_len, w.draft_len, 1.0, 0,
                                    include_self=include_self, backoff=backoff)
            assert_step_equal(got, want, t, what)
    # one path alone: nothing to search without its own history
    rng = np.random.default_rng(5)
    motif = rng.integers(0, 50, size=7)
    tokens = np.tile(motif, 12)[None, None, :80].astype(np.int32)
    tokens[0, 0, rng.integers(0, 80, size=6)] = 99
    for matcher in (SCAN, INDEX):
        got = gpu_replay(tokens, None, 3, 6, 1.0, 0, matcher | opts)
        n_drafts = 0
        for t in range(80):
            lens_t = np.full((1, 1), t + 1, dtype=np.int32)
            want = oracle.draft_all(tokens, None, lens_t, 3, 6, 1.0, 0, include_self=include_self, backoff=backoff)
            assert_step_equal(got, want, t, "single path opts%d matcher%d" % (opts, matcher))
            n_drafts += int(want["draft_len"][0, 0] > 0)
        assert (n_drafts > 40) == include_self


def test_scores_are_bit_equal_to_the_oracle(oracle):
    """Both sides hold a score as the same exact integer and round it to float once, so the
    floats agree in every bit (the other tests allow 1e-6 relative): C1 and the first 300
    steps of C2, with probabilities and a fractional alpha, so that the sums have low bits."""
    for name, steps, alpha in (("C1", None, 0.625), ("C2", 300, 0.3), ("C1", None, 1.0)):
        w = synth.WORKLOADS[name]
        tokens, probs = synth.make_paths(w)
        steps = steps or w.max_len
        got = gpu_replay(tokens, probs, w.query_len, w.draft_len, alpha, 0, 0, steps=steps)
        for t in range(steps):
            lens_t = np.full(tokens.shape[:2], t + 1, dtype=np.int32)
            want = oracle.draft_all(tokens, probs, lens_t, w.query_len, w.draft_len, alpha, 0)
            assert got["token_scores"][t].tobytes() == want["token_scores"].tobytes(), (name, t)
            assert got["path_scores"][t].tobytes() == want["path_scores"].tobytes(), (name, t)
