"""Replay helpers shared by the GPU parity tests: feed a synthetic path set to
the HIP library step by step, and compute the same steps with the CPU oracle."""
import numpy as np
import torch

from paper_2503_05330_amd import binding


def gpu_replay(tokens, probs, k, L, alpha=1.0, score_mode=0, flags=0, steps=None, targets=None,
               counts=None, n_per_step=1, how="calls", max_edits=0, pool_mode=0, steps_per_launch=1):
    """Appends n_per_step tokens per path per step (or counts[t] of them) and drafts after
    every step.  Returns host arrays indexed by step, plus the final status bits.
    how: "calls"  = csd_append + csd_draft (+ csd_accept) per step,
         "step"   = one fused csd_step per step,
         "replay" / "replay_unfused" = one csd_replay call for all steps (n_per_step == 1,
                    no counts).
    steps_per_launch > 1: csd_replay runs its device-side loop where the configuration allows."""
    P, N, T = tokens.shape
    steps = steps if steps is not None else T // n_per_step
    dev = torch.device("cuda:0")
    ix = binding.Index(P, N, T, int(tokens.max()) + 1 if tokens.size else 1, k, L, alpha,
                       score_mode, flags, device=dev, max_edits=max_edits, pool_mode=pool_mode)
    if steps_per_launch > 1:
        ix.set_steps_per_launch(steps_per_launch)
    out_tok = torch.empty((steps, P, N, L), dtype=torch.int32, device=dev)
    out_len = torch.empty((steps, P, N), dtype=torch.int32, device=dev)
    out_ts = torch.empty((steps, P, N, L), dtype=torch.float32, device=dev)
    out_ps = torch.empty((steps, P, N), dtype=torch.float32, device=dev)
    out_acc = torch.empty((steps, P, N), dtype=torch.int32, device=dev) if targets is not None else None
    lens = np.zeros((steps, P, N), dtype=np.int32)
    cur = np.zeros((P, N), dtype=np.int64)
    n = n_per_step
    if how.startswith("replay"):
        assert n == 1 and counts is None
        d_tok = torch.from_numpy(np.ascontiguousarray(tokens[:, :, :steps].transpose(2, 0, 1))).to(dev)
        d_pr = None if probs is None else torch.from_numpy(
            np.ascontiguousarray(probs[:, :, :steps].transpose(2, 0, 1))).to(dev)
        d_tg = None if targets is None else torch.from_numpy(np.ascontiguousarray(targets[:steps])).to(dev)
        out = dict(tokens=out_tok, length=out_len, token_scores=out_ts, path_scores=out_ps)
        ix.replay(steps, d_tok, d_pr, k, L, out=out, targets=d_tg, accept_out=out_acc,
                  fused=(how == "replay"))
        lens[:] = (np.arange(steps) + 1)[:, None, None]
        steps_to_run = 0
    else:
        steps_to_run = steps
    for t in range(steps_to_run):
        cnt = counts[t].astype(np.int64) if counts is not None else np.full((P, N), n, np.int64)
        cnt = np.minimum(cnt, T - cur)
        # gather each path's next n tokens (ragged: path-local read position)
        idx = np.minimum(cur[..., None] + np.arange(n), T - 1)
        step_tok = np.take_along_axis(tokens, idx, axis=2).astype(np.int32)
        d_tok = torch.from_numpy(np.ascontiguousarray(step_tok)).to(dev)
        d_pr = None
        if probs is not None:
            d_pr = torch.from_numpy(np.ascontiguousarray(np.take_along_axis(probs, idx, axis=2))).to(dev)
        d_cnt = torch.from_numpy(cnt.astype(np.int32)).to(dev) if counts is not None else None
        cur = cur + cnt
        lens[t] = cur
        out = dict(tokens=out_tok[t], length=out_len[t], token_scores=out_ts[t], path_scores=out_ps[t])
        d_tg = torch.from_numpy(targets[t]).to(dev) if targets is not None else None
        if how == "step":
            ix.step(d_tok, d_pr, d_cnt, n, k, L, out=out, targets=d_tg,
                    accept_out=out_acc[t] if targets is not None else None)
        else:
            ix.append(d_tok, d_pr, d_cnt, n)
            ix.draft(k, L, out=out)
            if targets is not None:
                ix.accept(out_tok[t], out_len[t], d_tg, L, out=out_acc[t])
    status = ix.status()
    res = dict(draft=out_tok.cpu().numpy(), draft_len=out_len.cpu().numpy(),
               token_scores=out_ts.cpu().numpy(), path_scores=out_ps.cpu().numpy(),
               accept_len=out_acc.cpu().numpy() if out_acc is not None else None,
               lens=lens, status=status, index=ix)
    return res


def assert_step_equal(got, want, t, what=""):
    """Bit-exact on tokens / lengths / accept lengths; scores within 1e-6 relative."""
    for key in ("draft", "draft_len"):
        if not np.array_equal(got[key][t], want[key]):
            bad = np.argwhere(got[key][t] != want[key])[0]
            raise AssertionError("%s step %d: %s differs at %s: gpu %s oracle %s" % (
                what, t, key, bad, got[key][t][tuple(bad[:2])], want[key][tuple(bad[:2])]))
    if want.get("accept_len") is not None:
        assert np.array_equal(got["accept_len"][t], want["accept_len"]), "%s step %d accept" % (what, t)
    for key in ("token_scores", "path_scores"):
        np.testing.assert_allclose(got[key][t], want[key], rtol=1e-6, atol=0,
                                   err_msg="%s step %d %s" % (what, t, key))
