#!/usr/bin/env python3
"""Benchmark of the consensus-draft hot path on one MI355X.

One "step" = append one token to every path + draft for all N paths + greedy
accept length, on workload C2 (N = 16 paths x 1024 tokens, vocab 32000, query 3,
draft 8, generation probabilities supplied, alpha = 1).  Inputs are staged in HBM
before the timed region.  The timed region replays K consecutive decode steps
from an empty index (the mean therefore covers history lengths 1..K).

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused:
this build runs on one GPU.
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


def measured_traffic(kernel, workload):
    """HBM bytes per launch of the step kernel from the committed rocprofv3 counter runs
    (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy kernel of known size)."""
    path = os.path.join(ROOT, "profiles", "%s_%s_traffic.json" % (kernel, workload))
    try:
        with open(path) as f:
            return json.load(f)["traffic_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def batch_sweep(binding, torch, dev, w, tokens, probs, matches_per_problem_step, flags, max_edits):
    """Step time with P copies of the workload's first problem in one index (the problems are
    independent; every copy has its own memory).  256 steps from an empty index per point."""
    N, T, k, L = w.n_paths, w.max_len, w.query_len, w.draft_len
    S = min(256, T)
    points = []
    for P in (1, 4, 16, 64, 256, 1024, 4096):
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
        ix.reset()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        ix.replay(S, d_tok, d_pr, k, L, out=outs)
        ev1.record()
        torch.cuda.synchronize()
        us = ev0.elapsed_time(ev1) / S * 1e3
        # matches grow about linearly with history: a replay of S of T steps sees S/T of the mean
        b = algorithmic_bytes(N * P, k, L, k, matches_per_problem_step * P * S / T) - 4 * L * N * P
        points.append({"problems": P, "rows": P * N, "us_per_step": us,
                       "problem_steps_per_s": P / us * 1e6, "algorithmic_GBps": b / us / 1e3})
        del ix, outs, d_tok, d_pr
    return points


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1024)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--max-edits", type=int, default=0,
                    help="edit tolerance of the suffix match (0 = exact, the headline; 1 = fuzzy, by scan)")
    ap.add_argument("--matcher", choices=("auto", "scan", "index"), default="auto")
    ap.add_argument("--pool", choices=("dag", "tree", "list"), default="dag",
                    help="organisation of the candidate pool (dag = the method, the headline; tree and "
                         "list are the variants of the paper's ablation)")
    ap.add_argument("--include-self", action="store_true",
                    help="also search a path's own history (not in the paper; not the headline)")
    ap.add_argument("--backoff", action="store_true",
                    help="shorten a query without matches until it has some (not in the paper; not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also time the step with 1..4096 copies of the workload's first problem in one "
                         "index (throughput against batch size)")
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
    w = synth.WORKLOADS[args.workload]
    tokens, probs = synth.make_paths(w)
    P, N, T, k, L = w.n_problems, w.n_paths, w.max_len, w.query_len, w.draft_len
    K, W = args.steps, args.warmup

    # step-major staging in HBM: [T][P][N]
    d_tok = torch.from_numpy(np.ascontiguousarray(tokens.transpose(2, 0, 1))).to(dev)
    d_pr = torch.from_numpy(np.ascontiguousarray(probs.transpose(2, 0, 1))).to(dev)
    tg = np.stack([synth.make_targets(tokens, min(t + 1, T), L) for t in range(T)])
    d_tg = torch.from_numpy(tg).to(dev)
    flags = {"auto": 0, "scan": 1, "index": 2}[args.matcher]
    flags |= (binding.INCLUDE_SELF if args.include_self else 0) | (binding.QUERY_BACKOFF if args.backoff else 0)
    ix = binding.Index(P, N, T, w.vocab, k, L, 1.0, 0, flags,
                       device=dev, max_edits=args.max_edits,
                       pool_mode={"dag": 0, "tree": 1, "list": 2}[args.pool])
    out = dict(tokens=torch.empty((P, N, L), dtype=torch.int32, device=dev),
               length=torch.empty((P, N), dtype=torch.int32, device=dev),
               token_scores=torch.empty((P, N, L), dtype=torch.float32, device=dev),
               path_scores=torch.empty((P, N), dtype=torch.float32, device=dev))
    acc = torch.empty((P, N), dtype=torch.int32, device=dev)

    outs = dict(tokens=torch.empty((T, P, N, L), dtype=torch.int32, device=dev),
                length=torch.empty((T, P, N), dtype=torch.int32, device=dev),
                token_scores=torch.empty((T, P, N, L), dtype=torch.float32, device=dev),
                path_scores=torch.empty((T, P, N), dtype=torch.float32, device=dev))
    accs = torch.empty((T, P, N), dtype=torch.int32, device=dev)

    def run_steps(n_steps, fused=True):
        """n_steps consecutive decode steps issued by the library's host loop (one fused
        launch per step); the replay restarts from an empty index whenever the paths are full."""
        done = 0
        while done < n_steps:
            m = min(T, n_steps - done)
            ix.reset()
            ix.replay(m, d_tok, d_pr, k, L, out=outs, targets=d_tg, accept_out=accs, fused=fused)
            done += m

    if args.calibrate_copy:
        src = torch.zeros(64 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        binding.debug_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    run_steps(W)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    run_steps(K)
    ev1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    launch_ms = ev0.elapsed_time(ev1) / K          # HIP events on the launch stream

    # the same steps as three launches each (append, draft, accept), and from Python per call
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    run_steps(min(K, T), fused=False)
    torch.cuda.synchronize()
    dt_unfused = (time.perf_counter() - t1) / min(K, T)
    ix.reset()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for t in range(min(K, T)):
        ix.step(d_tok[t], d_pr[t], None, 1, k, L, out=out, targets=d_tg[t], accept_out=acc)
    torch.cuda.synchronize()
    dt_python = (time.perf_counter() - t1) / min(K, T)

    # steady state at full history: the last 128 steps of a replay
    tail = min(128, T)
    ix.reset()
    ix.replay(T - tail, d_tok, d_pr, k, L, out=outs, targets=d_tg, accept_out=accs)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ix.replay(tail, d_tok[T - tail:], d_pr[T - tail:], k, L, out=outs, targets=d_tg[T - tail:],
              accept_out=accs)
    torch.cuda.synchronize()
    dt_tail = time.perf_counter() - t1

    # the propose / verify / accept loop with each path's own future as the model: paths accept
    # different numbers of tokens, so their lengths diverge and steps append several tokens
    d_future_tok = torch.from_numpy(tokens).to(dev)
    d_future_pr = torch.from_numpy(probs).to(dev)
    loop_steps = T
    ix.reset()
    loop = ix.accept_loop(loop_steps, d_future_tok, d_future_pr, k, L)       # warm-up
    torch.cuda.synchronize()
    ix.reset()
    t1 = time.perf_counter()
    loop = ix.accept_loop(loop_steps, d_future_tok, d_future_pr, k, L, out=loop)
    torch.cuda.synchronize()
    dt_loop = time.perf_counter() - t1
    path_len = loop["path_len"].cpu().numpy().reshape(loop_steps, -1)
    growing = np.concatenate([np.ones((1, path_len.shape[1]), bool), path_len[:-1] < T])
    steps_to_finish = int(growing.any(axis=1).sum())
    accept_mean = float(loop["accept"].cpu().numpy().reshape(loop_steps, -1)[growing].mean())

    # measured match counts (untimed, through the debug dump) -> algorithmic bytes
    ix.reset()
    m_total, m_samples = 0, 0
    for t in range(T):
        ix.append(d_tok[t], d_pr[t], None, 1)
        if t % 32 == 31:
            _, off = ix.dump_matches(k)
            m_total += int(off[-1])
            m_samples += 1
    matches_per_step = m_total / max(m_samples, 1)
    b_step = algorithmic_bytes(N * P, k, L, k, matches_per_step)
    achieved = b_step / (launch_ms * 1e-3) / 1e9

    # which kernel the configuration runs (the library's choice, mirrored here for the report)
    rows = P * N
    by_scan = args.matcher == "scan" or (args.matcher == "auto" and args.backoff) or (
        args.max_edits > 0 and args.matcher == "auto" and not (k >= 4 and rows > 128))
    kernel = "step_scan_kernel" if by_scan else "step_wave_kernel"
    variant = w.name + ("_one_edit" if args.max_edits else "") + ("" if args.pool == "dag" else "_" + args.pool)
    variant += ("_self" if args.include_self else "") + ("_backoff" if args.backoff else "")
    res = {
        "metric": METRIC, "value": K / dt, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": dt / K * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "%s: P=%d problems x N=%d paths x %d tokens, vocab %d, query %d, draft %d, "
                               "probs supplied, alpha 1, max_edits %d, pool %s%s%s; step = append 1 token/path + "
                               "draft all paths + accept" % (w.name, P, N, T, w.vocab, k, L, args.max_edits,
                                                             args.pool, ", own history" if args.include_self else "",
                                                             ", query back-off" if args.backoff else "")},
        "us_per_step_mean_over_replay": dt / K * 1e6,
        "us_per_step_at_full_history": dt_tail / tail * 1e6,
        "us_per_step_three_launches": dt_unfused * 1e6,
        "us_per_step_python_per_call": dt_python * 1e6,
        "accept_loop": {"us_per_step": dt_loop / loop_steps * 1e6, "steps_until_all_paths_full": steps_to_finish,
                        "mean_accept_len_while_growing": accept_mean,
                        "note": "csd_accept_loop: draft -> accept against the path's own future -> append "
                                "accepted + 1; synthetic stand-in for the model"},
        "matches_per_step": matches_per_step,
        "algorithmic_bytes_per_step": b_step,
        "roofline": {"bound": "hbm", "kernel": "csd::%s (one launch per step: append+draft+accept)" % kernel,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(kernel, variant),
                     "algorithmic_bytes_per_launch": b_step, "avg_launch_us": launch_ms * 1e3},
    }

    if args.batch_sweep:
        res["batch_sweep"] = batch_sweep(binding, torch, dev, w, tokens, probs, matches_per_step / P, flags,
                                         args.max_edits)

    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        reps, n_done, t_cpu = 0, 0, 0.0
        while t_cpu < 10.0 and reps < 64:
            c0 = time.perf_counter()
            for t in range(T):
                lens = np.full((P, N), t + 1, dtype=np.int32)
                oracle.draft_all(tokens, probs, lens, k, L, 1.0, 0, tg[t], eps=args.max_edits,
                                 pool_mode={"dag": 0, "tree": 1, "list": 2}[args.pool],
                                 include_self=args.include_self, backoff=args.backoff)
            t_cpu += time.perf_counter() - c0
            n_done += T
            reps += 1
        res["cpu_baseline"] = {"value": n_done / t_cpu, "unit": "steps/s", "cores": 1, "kind": "oracle",
                               "sample": "all %d steps of the %s replay, %d repeat(s), single thread"
                                         % (T, w.name, reps)}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
