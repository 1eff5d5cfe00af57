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


def algorithmic_bytes(N, k, L, kmax, matches_per_step):
    """Bytes the method has to move per step (not the bytes a scan would touch):
    per path: step input + history store + index entries, one 64-byte index bucket per
    query, the outputs; per match: its posting, the tokens compared, L continuation
    tokens with their probabilities."""
    b_app = 4 + 4 + 4 + 4 + 8 * kmax
    b_lkp = 64
    b_out = 8 * L + 8 + 4 * L + 4          # draft tokens+scores, length+path score, targets, accept
    b_match = 4 + 4 * k + L * (4 + 4)
    per_step = N * (b_app + b_lkp + b_out) + matches_per_step * b_match
    draft_only = N * (b_lkp + 8 * L + 8) + matches_per_step * b_match
    return per_step, draft_only


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1024)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    ix = binding.Index(P, N, T, w.vocab, k, L, 1.0, 0, 0, device=dev)
    out = dict(tokens=torch.empty((P, N, L), dtype=torch.int32, device=dev),
               length=torch.empty((P, N), dtype=torch.int32, device=dev),
               token_scores=torch.empty((P, N, L), dtype=torch.float32, device=dev),
               path_scores=torch.empty((P, N), dtype=torch.float32, device=dev))
    acc = torch.empty((P, N), dtype=torch.int32, device=dev)

    def run_steps(n_steps, events=None):
        """n_steps consecutive decode steps; the replay restarts from an empty
        index whenever the paths are full."""
        t = 0
        for s in range(n_steps):
            if t == T:
                ix.reset()
                t = 0
            ix.append(d_tok[t], d_pr[t], None, 1)
            if events is not None:
                events[s][0].record()
            ix.draft(k, L, out=out)
            if events is not None:
                events[s][1].record()
            ix.accept(out["tokens"], out["length"], d_tg[t], L, out=acc)
            t += 1

    run_steps(W)
    ix.reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(K)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # steady state at full history: the last 128 steps of a replay
    ix.reset()
    tail = min(128, T)
    for t in range(T - tail):
        ix.append(d_tok[t], d_pr[t], None, 1)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for t in range(T - tail, T):
        ix.append(d_tok[t], d_pr[t], None, 1)
        ix.draft(k, L, out=out)
        ix.accept(out["tokens"], out["length"], d_tg[t], L, out=acc)
    torch.cuda.synchronize()
    dt_tail = time.perf_counter() - t1

    # dominant kernel (draft): HIP events on the launch stream around every draft launch
    ix.reset()
    Ke = min(K, T)
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(Ke)]
    run_steps(Ke, events)
    torch.cuda.synchronize()
    draft_ms = float(np.mean([a.elapsed_time(b) for a, b in events]))

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
    b_step, b_draft = algorithmic_bytes(N * P, k, L, k, matches_per_step)
    achieved = b_draft / (draft_ms * 1e-3) / 1e9

    res = {
        "metric": METRIC, "value": K / dt, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": dt / K * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "%s: P=%d problems x N=%d paths x %d tokens, vocab %d, query %d, draft %d, "
                               "probs supplied, alpha 1; step = append 1 token/path + draft all paths + accept"
                               % (w.name, P, N, T, w.vocab, k, L)},
        "us_per_step_mean_over_replay": dt / K * 1e6,
        "us_per_step_at_full_history": dt_tail / tail * 1e6,
        "matches_per_step": matches_per_step,
        "algorithmic_bytes_per_step": b_step,
        "roofline": {"bound": "hbm", "kernel": "draft_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": b_draft, "avg_launch_us": draft_ms * 1e3},
    }

    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        reps, n_done, t_cpu = 0, 0, 0.0
        while t_cpu < 10.0 and reps < 64:
            c0 = time.perf_counter()
            for t in range(T):
                lens = np.full((P, N), t + 1, dtype=np.int32)
                oracle.draft_all(tokens, probs, lens, k, L, 1.0, 0, tg[t])
            t_cpu += time.perf_counter() - c0
            n_done += T
            reps += 1
        res["cpu_baseline"] = {"value": n_done / t_cpu, "unit": "steps/s", "cores": 1, "kind": "oracle",
                               "sample": "all %d steps of the %s replay, %d repeat(s), single thread"
                                         % (T, w.name, reps)}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
