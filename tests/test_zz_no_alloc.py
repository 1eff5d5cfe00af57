"""The entry point that allocates nothing (csd_accept_loop_noalloc) against csd_accept_loop,
through the C-ABI: two calls in a row on one GPU, the second with a smaller input, so that the
second call finds the first one's contents in the library's fixed scratch array."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2503_05330_amd import binding, synth

pytestmark = pytest.mark.gpu


def _both(w, steps, dev):
    tokens, probs = synth.make_paths(w)
    P, N, T, k, L = w.n_problems, w.n_paths, w.max_len, w.query_len, w.draft_len
    d_tok, d_pr = torch.from_numpy(tokens).to(dev), torch.from_numpy(probs).to(dev)
    ref_ix = binding.Index(P, N, T, w.vocab, k, L, 1.0, 0, binding.MATCH_INDEX, device=dev)
    ref = ref_ix.accept_loop(steps, d_tok, d_pr, k, L)
    ix = binding.Index(P, N, T, w.vocab, k, L, 1.0, 0, binding.MATCH_INDEX, device=dev)
    out = {name: torch.full_like(ref[name], -7) for name in ("tokens", "length", "accept", "path_len")}
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    ix.accept_loop_noalloc(steps, d_tok, d_pr, k, L, out)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated"
    for name in ("tokens", "length", "accept", "path_len"):
        assert torch.equal(out[name], ref[name]), "%s %s differs" % (w.name, name)
    assert ix.status() == ref_ix.status() == 0
    assert int(out["accept"].max()) > 0 and min(steps, T - 1) < int(out["path_len"].max()) <= T
    return ix


def test_noalloc_accept_loop_matches_the_allocating_one():
    dev = torch.device("cuda:0")
    print("noalloc C4 x 8 problems", flush=True)
    big = synth.scaled(synth.WORKLOADS["C4"], n_problems=8)          # 128 rows, L = 8
    _both(big, 400, dev)
    print("noalloc C1 (smaller, same array)", flush=True)
    small = synth.WORKLOADS["C1"]                                    # 4 rows, L = 5
    ix = _both(small, 256, dev)
    # beyond the fixed array: rejected before anything is enqueued
    print("noalloc limit", flush=True)
    rows = binding.NOALLOC_SCRATCH_BYTES // (2 * (3 * 32 + 3) * 4) + 1
    huge = binding.Index(rows, 1, 64, 100, 3, 32, 1.0, 0, binding.MATCH_INDEX, device=dev)
    fut = torch.zeros((rows, 1, 64), dtype=torch.int32, device=dev)
    out = dict(tokens=torch.empty((1, rows, 1, 32), dtype=torch.int32, device=dev))
    for name in ("length", "accept", "path_len"):
        out[name] = torch.empty((1, rows, 1), dtype=torch.int32, device=dev)
    with pytest.raises(binding.CsdError) as err:
        huge.accept_loop_noalloc(1, fut, None, 3, 32, out)
    assert err.value.code == binding.ERR_SCRATCH_LIMIT
    assert "scratch" in binding.strerror(binding.ERR_SCRATCH_LIMIT)
