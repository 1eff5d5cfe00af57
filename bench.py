#!/usr/bin/env python3
"""Benchmark of the consensus-draft hot path on one MI355X.

One "step" = append one token to every path + draft for all N paths + greedy
accept length, in ONE launch, on workload C2 (N = 16 paths x 1024 tokens, vocab
32000, query 3, draft 8, generation probabilities supplied, alpha = 1).  Inputs
are staged in HBM before anything is timed.

What is timed.  The metric is quoted at N = 16 x 1024 tokens, so the timed region
is the LAST K steps of the 1024-step replay, where the histories are (nearly)
full: the device is synchronised, the first T - K steps of the replay run untimed
(they are the warm-up: at least W steps), then K steps are timed with HIP events
on the launch stream (the first event sits on the stream directly behind the
untimed steps: the timed steps run back to back behind earlier work, as in a
decode loop), and the device is synchronised again.  With a synchronisation
directly before the timed steps they would start on an idle device, whose first
launches are slower: that figure is reported too (`..._after_device_idle`), it is
not the headline.  All of it is repeated R times (default 30);
`value` and `ms_per_step` are the median over the repeats, `us_per_step_p50/p99`
their percentiles.  The match counts behind the roofline's byte count and the
CPU baseline are taken on those same K steps.

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build runs on one
GPU.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "draft steps/sec (all N paths) and µs/step at N=16×1024 tok; % HBM roofline"
HBM_PEAK_GBS = 8000.0
POOLS = {"dag": 0, "tree": 1, "list": 2}


def algorithmic_bytes(n_paths, k, L, kmax, matches_per_step):
    """Bytes the method has to move per step (not the bytes a scan would touch).
    Per path: step input (token + probability), history store (token + quantised
    probability), its meta row read and written (length + kmax tail tokens), one index
    entry (posting + fill count), one 64-byte index bucket for the lookup, the outputs
    (L draft tokens + L scores + length + path score), L targets and the accept length.
    Per match: its posting, the k verify tokens, L continuation tokens with probabilities."""
    b_path = 8 + 8 + 8 * (1 + kmax) + 8 + 64 + (8 * L + 8) + (4 * L + 4)
    b_match = 4 + 4 * k + 8 * L
    return n_paths * b_path + matches_per_step * b_match


def committed_traffic(kernel, variant):
    """HBM bytes per launch of the step kernel from the committed rocprofv3 counter runs of
    this command (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy kernel of known size);
    the second value names the file."""
    name = "%s_%s_traffic.json" % (kernel, variant)
    try:
        with open(os.path.join(ROOT, "profiles", name)) as f:
            return json.load(f)["traffic_bytes_per_launch"], "profiles/" + name
    except (OSError, KeyError, ValueError):
        return None, None


def percentile(xs, q):
    xs = sorted(xs)
    return xs[min(len(xs) - 1, int(round(q * (len(xs) - 1))))]


class Replay:
    """One workload staged in HBM, with an index and output buffers for a whole replay."""

    def __init__(self, torch, binding, synth, name, dev, max_edits=0, matcher="auto", pool="dag",
                 include_self=False, backoff=False):
        self.torch, self.binding = torch, binding
        self.w = w = synth.WORKLOADS[name]
        self.tokens, self.probs = synth.make_paths(w)
        P, N, T, L = w.n_problems, w.n_paths, w.max_len, w.draft_len
        self.P, self.N, self.T, self.k, self.L = P, N, T, w.query_len, L
        self.max_edits, self.matcher, self.pool = max_edits, matcher, pool
        self.include_self, self.backoff = include_self, backoff
        self.d_tok = torch.from_numpy(np.ascontiguousarray(self.tokens.transpose(2, 0, 1))).to(dev)   # [T][P][N]
        self.d_pr = torch.from_numpy(np.ascontiguousarray(self.probs.transpose(2, 0, 1))).to(dev)
        # targets of step t: every path's own next L tokens (-1 beyond the end), [T][P][N][L]
        padded = np.concatenate([self.tokens, np.full((P, N, L), -1, np.int32)], axis=2)
        tg = np.stack([padded[:, :, 1 + d:1 + d + T] for d in range(L)], axis=-1)       # [P][N][T][L]
        self.targets = np.ascontiguousarray(tg.transpose(2, 0, 1, 3))
        self.d_tg = torch.from_numpy(self.targets).to(dev)
        self.flags = {"auto": 0, "scan": 1, "index": 2}[matcher]
        self.flags |= (binding.INCLUDE_SELF if include_self else 0) | (binding.QUERY_BACKOFF if backoff else 0)
        self.ix = binding.Index(P, N, T, w.vocab, self.k, L, 1.0, 0, self.flags, device=dev,
                                max_edits=max_edits, pool_mode=POOLS[pool])
        mk = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        self.outs = dict(tokens=mk((T, P, N, L), torch.int32), length=mk((T, P, N), torch.int32),
                         token_scores=mk((T, P, N, L), torch.float32), path_scores=mk((T, P, N), torch.float32))
        self.accs = mk((T, P, N), torch.int32)
        rows = P * N
        by_scan = matcher == "scan" or (matcher == "auto" and backoff) or (
            max_edits > 0 and matcher == "auto" and not (self.k >= 4 and (rows > 128 or N * T >= 1 << 14)))
        self.kernel = "step_scan_kernel" if by_scan else "step_wave_kernel"
        self.variant = (w.name + ("_one_edit" if max_edits else "") + ("" if pool == "dag" else "_" + pool)
                        + ("_self" if include_self else "") + ("_backoff" if backoff else ""))

    def steps(self, first, count, fused=True):
        """Steps first .. first + count - 1 of the replay, issued by the library's host loop."""
        if count <= 0:
            return
        s = slice(first, first + count)
        outs = {name: t[s] for name, t in self.outs.items()}
        self.ix.replay(count, self.d_tok[s], self.d_pr[s], self.k, self.L, out=outs, targets=self.d_tg[s],
                       accept_out=self.accs[s], fused=fused)

    def time_tail(self, K, repeats, fused=True, idle_before=False):
        """Per-step microseconds of the last K steps of the replay, once per repeat, by HIP
        events on the launch stream.  The device is synchronised before the replay starts and
        after its last step; the first event is recorded on the stream directly behind the
        untimed steps, so the timed steps run as they do in a decode loop: back to back behind
        earlier work.  idle_before: synchronise once more directly before the timed steps, so
        that they start on an idle device (its first launches are then slower)."""
        torch = self.torch
        by_event = []
        for _ in range(repeats):
            self.ix.reset()
            torch.cuda.synchronize()
            self.steps(0, self.T - K, fused)
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            if idle_before:
                torch.cuda.synchronize()
            ev0.record()
            self.steps(self.T - K, K, fused)
            ev1.record()
            torch.cuda.synchronize()
            by_event.append(ev0.elapsed_time(ev1) / K * 1e3)
        return by_event

    def matches_in_tail(self, K, samples):
        """Mean number of matches per step (all rows) over `samples` of the last K steps, counted
        through the debug dump of the match sets (untimed)."""
        self.ix.reset()
        self.steps(0, self.T - K)
        want = set(np.linspace(self.T - K, self.T - 1, num=min(samples, K)).astype(int).tolist())
        total = 0
        for t in range(self.T - K, self.T):
            self.steps(t, 1)
            if t in want:
                _, off = self.ix.dump_matches(self.k, cap=1 << 22)
                total += int(off[-1])
        return total / len(want)

    def describe(self):
        w = self.w
        return ("%s: P=%d problems x N=%d paths x %d tokens, vocab %d, query %d, draft %d, probs supplied, "
                "alpha 1, max_edits %d, pool %s%s%s; step = append 1 token/path + draft all paths + accept"
                % (w.name, self.P, self.N, self.T, w.vocab, self.k, self.L, self.max_edits, self.pool,
                   ", own history" if self.include_self else "", ", query back-off" if self.backoff else ""))


def batch_points(binding, torch, dev, w, tokens, probs, matches_per_problem_step, flags, max_edits, problems,
                 S=256):
    """Step time with P copies of the workload's first problem in one index (the problems are
    independent; every copy has its own memory).  S steps from an empty index per point."""
    N, T, k, L = w.n_paths, w.max_len, w.query_len, w.draft_len
    S = min(S, T)
    points = []
    for P in problems:
        tok = np.ascontiguousarray(np.broadcast_to(tokens[0, :, :S].T[:, None, :], (S, P, N)))
        pr = np.ascontiguousarray(np.broadcast_to(probs[0, :, :S].T[:, None, :], (S, P, N)))
        d_tok, d_pr = torch.from_numpy(tok).to(dev), torch.from_numpy(pr).to(dev)
        ix = binding.Index(P, N, T, w.vocab, k, L, 1.0, 0, flags, device=dev, max_edits=max_edits)
        outs = dict(tokens=torch.empty((S, P, N, L), dtype=torch.int32, device=dev),
                    length=torch.empty((S, P, N), dtype=torch.int32, device=dev),
                    token_scores=torch.empty((S, P, N, L), dtype=torch.float32, device=dev),
                    path_scores=torch.empty((S, P, N), dtype=torch.float32, device=dev))
        ix.replay(S, d_tok, d_pr, k, L, out=outs)                 # warm-up
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            ix.reset()
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            ev0.record()
            ix.replay(S, d_tok, d_pr, k, L, out=outs)
            ev1.record()
            torch.cuda.synchronize()
            us = ev0.elapsed_time(ev1) / S * 1e3
            best = us if best is None else min(best, us)
        # matches grow about linearly with history: a replay of S of T steps sees S/T of the mean
        b = algorithmic_bytes(N * P, k, L, k, matches_per_problem_step * P * S / T) - 4 * L * N * P
        points.append({"problems": P, "rows": P * N, "steps_from_empty": S, "us_per_step": best,
                       "problem_steps_per_s": P / best * 1e6, "algorithmic_GBps": b / best / 1e3})
        del ix, outs, d_tok, d_pr
        torch.cuda.empty_cache()
    return points


def batch_points_full_history(binding, torch, dev, w, tokens, probs, matches_per_problem_step, flags, max_edits,
                              problems, K=128):
    """The same batches at FULL history: P copies of the workload's first problem, T - K steps
    replayed untimed, then the last K steps timed (best of two)."""
    N, T, k, L = w.n_paths, w.max_len, w.query_len, w.draft_len
    points = []
    for P in problems:
        tok = np.ascontiguousarray(np.broadcast_to(tokens[0].T[:, None, :], (T, P, N)))
        pr = np.ascontiguousarray(np.broadcast_to(probs[0].T[:, None, :], (T, P, N)))
        d_tok, d_pr = torch.from_numpy(tok).to(dev), torch.from_numpy(pr).to(dev)
        ix = binding.Index(P, N, T, w.vocab, k, L, 1.0, 0, flags, device=dev, max_edits=max_edits)
        outs = dict(tokens=torch.empty((K, P, N, L), dtype=torch.int32, device=dev),
                    length=torch.empty((K, P, N), dtype=torch.int32, device=dev),
                    token_scores=torch.empty((K, P, N, L), dtype=torch.float32, device=dev),
                    path_scores=torch.empty((K, P, N), dtype=torch.float32, device=dev))
        best = None
        for _ in range(2):
            ix.reset()
            ix.replay(T - K, d_tok[:T - K], d_pr[:T - K], k, L)
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            ev0.record()
            ix.replay(K, d_tok[T - K:], d_pr[T - K:], k, L, out=outs)
            ev1.record()
            torch.cuda.synchronize()
            us = ev0.elapsed_time(ev1) / K * 1e3
            best = us if best is None else min(best, us)
        b = algorithmic_bytes(N * P, k, L, k, matches_per_problem_step * P) - 4 * L * N * P
        points.append({"problems": P, "rows": P * N, "timed_steps": K, "history": "%d..%d" % (T - K + 1, T),
                       "us_per_step": best, "problem_steps_per_s": P / best * 1e6,
                       "algorithmic_GBps": b / best / 1e3})
        del ix, outs, d_tok, d_pr
        torch.cuda.empty_cache()
    return points


def cpu_baseline(oracle, r, K, budget_s, threads):
    """The oracle on the last K steps of the replay (the timed region's steps), repeated until
    about budget_s seconds have passed: steps per second on `threads` host threads."""
    T = r.T
    lens = np.empty((K, r.P, r.N), dtype=np.int32)
    lens[:] = (np.arange(T - K, T, dtype=np.int32) + 1)[:, None, None]
    tg = np.ascontiguousarray(r.targets[T - K:])
    done, spent = 0, 0.0
    while spent < budget_s:
        c0 = time.perf_counter()
        oracle.draft_many(r.tokens, r.probs, lens, r.k, r.L, 1.0, 0, tg, eps=r.max_edits,
                          pool_mode=POOLS[r.pool], include_self=r.include_self, backoff=r.backoff,
                          threads=threads)
        spent += time.perf_counter() - c0
        done += K
    return done / spent, done


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128, help="K: timed steps at the end of the replay")
    ap.add_argument("--warmup", type=int, default=64,
                    help="W: least number of untimed steps before the timed ones (the replay's first "
                         "T - K steps run untimed in any case)")
    ap.add_argument("--repeats", type=int, default=30, help="R: how often the timed region is measured")
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--max-edits", type=int, default=0,
                    help="edit tolerance of the suffix match (0 = exact, the headline; 1 = one edit)")
    ap.add_argument("--matcher", choices=("auto", "scan", "index"), default="auto")
    ap.add_argument("--pool", choices=tuple(POOLS), default="dag",
                    help="organisation of the candidate pool (dag = the method, the headline; tree and "
                         "list are the variants of the paper's ablation)")
    ap.add_argument("--include-self", action="store_true",
                    help="also search a path's own history (not in the paper; not the headline)")
    ap.add_argument("--backoff", action="store_true",
                    help="shorten a query without matches until it has some (not in the paper; not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the timed region (what the profiler runs use): no other workloads, "
                         "launch patterns, accept loop, batch points or CPU baseline")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also time the step with 1..4096 copies of the workload's first problem in one "
                         "index (throughput against batch size; the default run has two of these points)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 64 MiB copy kernel (reference for traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
                 "(no multi-GPU sharding or collectives in this path)" % args.gpus)

    import torch
    from paper_2503_05330_amd import binding, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    binding.load()
    dev = torch.device("cuda:0")
    r = Replay(torch, binding, synth, args.workload, dev, args.max_edits, args.matcher, args.pool,
               args.include_self, args.backoff)
    P, N, T, k, L = r.P, r.N, r.T, r.k, r.L
    W = max(0, args.warmup)
    K = max(1, min(args.steps, T - min(W, T - 1)))
    R = max(1, args.repeats)

    if args.calibrate_copy:
        src = torch.zeros(64 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        binding.debug_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    r.steps(0, T)                                     # one whole replay first: code and data are warm
    torch.cuda.synchronize()
    by_event = r.time_tail(K, R)
    us = percentile(by_event, 0.5)
    after_idle = r.time_tail(K, R, idle_before=True)
    matches_per_step = r.matches_in_tail(K, 32)
    b_step = algorithmic_bytes(N * P, k, L, k, matches_per_step)
    achieved = b_step / (us * 1e-6) / 1e9
    traffic, traffic_file = committed_traffic(r.kernel, r.variant)
    res = {
        "metric": METRIC, "value": 1e6 / us, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "untimed_steps_before_each_timed_region": T - K,
        "ms_per_step": us * 1e-3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": r.describe(),
                   "timed_region": "steps %d..%d of the %d-step replay (history length %d..%d tokens per path), "
                                   "after %d untimed steps; median of %d repeats, HIP events"
                                   % (T - K + 1, T, T, T - K + 1, T, T - K, R)},
        "repeats": R,
        "us_per_step": us, "us_per_step_p50": us, "us_per_step_p99": percentile(by_event, 0.99),
        "us_per_step_min": min(by_event), "us_per_step_max": max(by_event),
        "us_per_step_mean": float(np.mean(by_event)),
        "us_per_step_after_device_idle_p50": percentile(after_idle, 0.5),
        "us_per_step_after_device_idle_p99": percentile(after_idle, 0.99),
        "percentiles_over": "the R repeats of the K-step timed region (each sample: mean per step of one "
                            "repeat); per-launch percentiles of the kernel are in profiles/",
        "matches_per_step": matches_per_step,
        "algorithmic_bytes_per_step": b_step,
        "roofline": {"bound": "hbm", "kernel": "csd::%s (one launch per step: append+draft+accept)" % r.kernel,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_file,
                     "algorithmic_bytes_per_launch": b_step, "avg_launch_us": us,
                     "note": "bytes and time are those of the same K timed steps; the step is bound by "
                             "launch and memory latency, not by bandwidth"},
    }
    if args.headline_only:
        if args.batch_sweep:
            res["batch"] = batch_points(binding, torch, dev, r.w, r.tokens, r.probs, matches_per_step / P, r.flags,
                                        args.max_edits, (1, 4, 16, 64, 256, 1024, 4096))
        print(json.dumps(res))
        return

    # the same steps as three launches each (append, draft, accept), and issued from Python per call
    ev3 = r.time_tail(K, min(R, 5), fused=False)
    res["us_per_step_three_launches"] = percentile(ev3, 0.5)
    out1 = {name: t[0] for name, t in r.outs.items()}
    per_call = []
    for _ in range(min(R, 5)):
        r.ix.reset()
        r.steps(0, T - K)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for t in range(T - K, T):
            r.ix.step(r.d_tok[t], r.d_pr[t], None, 1, k, L, out=out1, targets=r.d_tg[t], accept_out=r.accs[0])
        torch.cuda.synchronize()
        per_call.append((time.perf_counter() - t1) / K * 1e6)
    res["us_per_step_python_per_call"] = percentile(per_call, 0.5)

    # the whole replay from an empty index (history lengths 1..T): a labelled secondary figure
    whole = []
    for _ in range(5):
        r.ix.reset()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ev0.record()
        r.steps(0, T)
        ev1.record()
        torch.cuda.synchronize()
        whole.append(ev0.elapsed_time(ev1) / T * 1e3)
    res["us_per_step_mean_over_whole_replay"] = percentile(whole, 0.5)

    # the propose / verify / accept loop with each path's own future as the model: paths accept
    # different numbers of tokens, so their lengths diverge and steps append several tokens
    d_future_tok = torch.from_numpy(r.tokens).to(dev)
    d_future_pr = torch.from_numpy(r.probs).to(dev)
    r.ix.reset()
    loop = r.ix.accept_loop(T, d_future_tok, d_future_pr, k, L)               # warm-up
    torch.cuda.synchronize()
    loop_us = []
    for _ in range(5):
        r.ix.reset()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ev0.record()
        loop = r.ix.accept_loop(T, d_future_tok, d_future_pr, k, L, out=loop)
        ev1.record()
        torch.cuda.synchronize()
        loop_us.append(ev0.elapsed_time(ev1) / T * 1e3)
    path_len = loop["path_len"].cpu().numpy().reshape(T, -1)
    growing = np.concatenate([np.ones((1, path_len.shape[1]), bool), path_len[:-1] < T])
    res["accept_loop"] = {"us_per_step": percentile(loop_us, 0.5),
                          "steps_until_all_paths_full": int(growing.any(axis=1).sum()),
                          "mean_accept_len_while_growing":
                              float(loop["accept"].cpu().numpy().reshape(T, -1)[growing].mean()),
                          "note": "csd_accept_loop over %d steps: draft -> accept against the path's own "
                                  "future -> append accepted + 1; synthetic stand-in for the model" % T}
    # the same two host-free loops with the device-side loop (many steps per launch): reported
    # beside the per-launch figures, never instead of them
    r.ix.set_steps_per_launch(1 << 20)
    dev_tail = r.time_tail(K, min(R, 10))
    dev_loop_us = []
    for _ in range(5):
        r.ix.reset()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ev0.record()
        loop = r.ix.accept_loop(T, d_future_tok, d_future_pr, k, L, out=loop)
        ev1.record()
        torch.cuda.synchronize()
        dev_loop_us.append(ev0.elapsed_time(ev1) / T * 1e3)
    r.ix.set_steps_per_launch(1)
    res["device_side_loop"] = {
        "replay_us_per_step_at_full_history": percentile(dev_tail, 0.5),
        "accept_loop_us_per_step": percentile(dev_loop_us, 0.5),
        "note": "csd_set_steps_per_launch: csd_replay / csd_accept_loop as ONE launch for all their steps "
                "(a workgroup per problem, a wave per path, a barrier between steps); same steps and "
                "timing as `value` and accept_loop.us_per_step; not the per-call headline"}
    del loop, d_future_tok, d_future_pr

    # the other workloads, one-edit matching and two batch sizes: step time at full history
    def tail_of(name, **kw):
        x = Replay(torch, binding, synth, name, dev, **kw)
        Kx = min(128, x.T // 4)
        x.steps(0, x.T)
        torch.cuda.synchronize()
        ev = x.time_tail(Kx, 5)
        m = x.matches_in_tail(Kx, 8)
        bx = algorithmic_bytes(x.N * x.P, x.k, x.L, x.k, m)
        u = percentile(ev, 0.5)
        return {"us_per_step_at_full_history": u, "us_min": min(ev), "us_max": max(ev), "timed_steps": Kx,
                "repeats": 5, "matches_per_step": m, "algorithmic_bytes_per_step": bx,
                "algorithmic_GBps": bx / u / 1e3, "problem_steps_per_s": x.P / u * 1e6,
                "kernel": "csd::" + x.kernel, "workload": x.describe()}
    if args.workload == "C2" and args.max_edits == 0 and args.pool == "dag" and args.matcher == "auto" \
            and not args.include_self and not args.backoff:
        per = {}
        for name in ("C1", "C2", "C3", "C4", "C5"):
            per[name] = tail_of(name)
        res["per_workload"] = per
        res["one_edit"] = {"C2": tail_of("C2", max_edits=1), "C3": tail_of("C3", max_edits=1),
                           "C5": tail_of("C5", max_edits=1),
                           "note": "Eq. 4 with one edit, the tolerance of the paper's experiments, under the "
                                   "matcher CSD_MATCH_AUTO picks"}
        problems = (1, 4, 16, 64, 256, 1024, 4096) if args.batch_sweep else (64, 4096)
        res["batch"] = batch_points(binding, torch, dev, r.w, r.tokens, r.probs, matches_per_step / P, r.flags,
                                    args.max_edits, problems)
        res["batch_at_full_history"] = batch_points_full_history(
            binding, torch, dev, r.w, r.tokens, r.probs, matches_per_step / P, r.flags, args.max_edits,
            (64, 1024, 4096) if args.batch_sweep else (1024, 4096))
    elif args.batch_sweep:
        res["batch"] = batch_points(binding, torch, dev, r.w, r.tokens, r.probs, matches_per_step / P, r.flags,
                                    args.max_edits, (1, 4, 16, 64, 256, 1024, 4096))

    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        cores = oracle.host_threads()
        all_cores, n_all = cpu_baseline(oracle, r, K, 8.0, cores)
        one_core, n_one = cpu_baseline(oracle, r, K, 8.0, 1)
        sample = "the %d timed steps (history %d..%d) of the %s replay" % (K, T - K + 1, T, r.w.name)
        res["cpu_baseline"] = {"value": all_cores, "unit": "steps/s", "cores": cores, "kind": "oracle",
                               "sample": "%s, %d passes, %d host threads" % (sample, n_all // K, cores)}
        res["cpu_baseline_1t"] = {"value": one_core, "unit": "steps/s", "cores": 1, "kind": "oracle",
                                  "sample": "%s, %d passes, one thread" % (sample, n_one // K)}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
