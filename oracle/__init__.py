"""Loader for the CPU oracle (csd_oracle.cpp) — TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.
The GPU package never does.  This module compiles the C++ file with g++ and
wraps its `extern "C"` functions with numpy array marshalling; it contains no
arithmetic of its own.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csd_oracle.cpp")
_SANITIZE = os.environ.get("CSD_ORACLE_SANITIZE") == "1"
_LIB = os.path.join(_HERE, "libcsd_oracle_san.so" if _SANITIZE else "libcsd_oracle.so")
_lib = None

_i32p = ctypes.POINTER(ctypes.c_int32)
_u64p = ctypes.POINTER(ctypes.c_uint64)
_f32p = ctypes.POINTER(ctypes.c_float)


def _extra_flags():
    """CSD_ORACLE_SANITIZE=1 builds the oracle (into a library of its own) with the address and
    undefined-behaviour sanitizers: host code only.  A Python process can load that library
    only with libasan preloaded; tests/test_oracle_pins.py runs the pins that way."""
    if _SANITIZE:
        return ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                "-fno-omit-frame-pointer"]
    return []


def host_threads() -> int:
    """Threads the threaded oracle entry point uses by default: the cores this process may run
    on, at most 16 (a GPU machine's CPU share)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(n, 16))


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (plain -O2, no GPU toolchain)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++14", "-pthread", *_extra_flags(), "-shared", "-fPIC",
                               "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_quantize_prob.restype = ctypes.c_uint32
        lib.oracle_quantize_prob.argtypes = [ctypes.c_float]
        lib.oracle_alpha_q.restype = ctypes.c_uint32
        lib.oracle_alpha_q.argtypes = [ctypes.c_double]
        lib.oracle_edit_distance.restype = ctypes.c_int32
        lib.oracle_edit_distance.argtypes = [_i32p, ctypes.c_int32, _i32p, ctypes.c_int32]
        lib.oracle_matches.restype = ctypes.c_int64
        lib.oracle_matches.argtypes = [_i32p, _i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _i32p, ctypes.c_int64]
        lib.oracle_edges.restype = ctypes.c_int64
        lib.oracle_edges.argtypes = [_i32p, _f32p, _i32p, ctypes.c_int32, ctypes.c_int32,
                                     ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                     ctypes.c_int32, _i32p, _u64p, ctypes.c_int64]
        lib.oracle_draft.restype = ctypes.c_int32
        lib.oracle_draft.argtypes = [_i32p, _f32p, _i32p, ctypes.c_int32, ctypes.c_int32,
                                     ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                     ctypes.c_uint32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                     _i32p, _f32p, _f32p]
        lib.oracle_accept.restype = ctypes.c_int32
        lib.oracle_accept.argtypes = [_i32p, ctypes.c_int32, _i32p]
        lib.oracle_draft_all.restype = None
        lib.oracle_draft_all.argtypes = [_i32p, _f32p, _i32p, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_uint32, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_int32, _i32p, _i32p, _f32p, _f32p,
                                         _i32p, _i32p]
        lib.oracle_draft_many.restype = None
        lib.oracle_draft_many.argtypes = [_i32p, _f32p, _i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_uint32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_int32, _i32p, _i32p, _f32p, _f32p, _i32p, _i32p]
        lib.oracle_accept_loop.restype = None
        lib.oracle_accept_loop.argtypes = [_i32p, _f32p, _i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_uint32,
                                           ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           _i32p, _i32p, _i32p, _i32p]
        _lib = lib
    return _lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_i32p)


def _f32(a):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_f32p)


def quantize_prob(p: float) -> int:
    return int(_load().oracle_quantize_prob(ctypes.c_float(p)))


def alpha_q(alpha: float) -> int:
    return int(_load().oracle_alpha_q(float(alpha)))


def edit_distance(a, b) -> int:
    a, ap = _i32(list(a) + [0])
    b, bp = _i32(list(b) + [0])
    return int(_load().oracle_edit_distance(ap, len(a) - 1, bp, len(b) - 1))


def _extras(include_self, backoff) -> int:
    return (1 if include_self else 0) | (2 if backoff else 0)


def matches(tok, length, i, k, eps=0, include_self=False):
    """(j, e) rows of path i's match set for one problem: tok [N][max_len], length [N]."""
    tok, tp = _i32(tok)
    length, lp = _i32(length)
    N, max_len = tok.shape
    lib = _load()
    cap = max(1, N * max_len)
    out = np.empty((cap, 2), dtype=np.int32)
    n = lib.oracle_matches(tp, lp, N, max_len, i, k, eps, _extras(include_self, False),
                           out.ctypes.data_as(_i32p), cap)
    return out[:n].copy()


def edges(tok, prob, length, i, k, L, eps=0, include_self=False):
    """Edge rows of path i's DAG: (duv int32 [n][3], cs uint64 [n][2]) sorted by (d, u, v)."""
    tok, tp = _i32(tok)
    prob, pp = _f32(prob)
    length, lp = _i32(length)
    N, max_len = tok.shape
    lib = _load()
    ex = _extras(include_self, False)
    n = lib.oracle_edges(tp, pp, lp, N, max_len, i, k, eps, ex, L, None, None, 0)
    duv = np.empty((max(n, 1), 3), dtype=np.int32)
    cs = np.empty((max(n, 1), 2), dtype=np.uint64)
    lib.oracle_edges(tp, pp, lp, N, max_len, i, k, eps, ex, L, duv.ctypes.data_as(_i32p),
                     cs.ctypes.data_as(_u64p), n)
    return duv[:n].copy(), cs[:n].copy()


def draft(tok, prob, length, i, k, L, alpha=1.0, score_mode=0, eps=0, pool_mode=0, include_self=False,
          backoff=False):
    """Draft of path i for one problem -> (tokens [L], draft_len, token_scores [L], path_score).
    pool_mode: 0 = DAG (the method), 1 = prefix tree, 2 = list (the ablation's variants)."""
    tok, tp = _i32(tok)
    prob, pp = _f32(prob)
    length, lp = _i32(length)
    N, max_len = tok.shape
    d = np.empty(L, dtype=np.int32)
    ts = np.empty(L, dtype=np.float32)
    ps = ctypes.c_float(0.0)
    lib = _load()
    n = lib.oracle_draft(tp, pp, lp, N, max_len, i, k, eps, L, lib.oracle_alpha_q(float(alpha)),
                         score_mode, pool_mode, _extras(include_self, backoff), d.ctypes.data_as(_i32p),
                         ts.ctypes.data_as(_f32p), ctypes.byref(ps))
    return d, int(n), ts, np.float32(ps.value)


def accept(draft_tokens, draft_len, target) -> int:
    d, dp = _i32(draft_tokens)
    t, tp = _i32(target)
    return int(_load().oracle_accept(dp, int(draft_len), tp))


def draft_all(tok, prob, length, k, L, alpha=1.0, score_mode=0, target=None, eps=0, pool_mode=0,
              include_self=False, backoff=False):
    """All paths of all problems: tok [P][N][max_len], prob same or None, length [P][N].

    Returns dict(draft [P][N][L], draft_len [P][N], token_scores [P][N][L],
    path_scores [P][N], accept_len [P][N] or None)."""
    tok, tp = _i32(tok)
    prob, pp = _f32(prob)
    length, lp = _i32(length)
    P, N, max_len = tok.shape
    d = np.empty((P, N, L), dtype=np.int32)
    dl = np.empty((P, N), dtype=np.int32)
    ts = np.empty((P, N, L), dtype=np.float32)
    ps = np.empty((P, N), dtype=np.float32)
    lib = _load()
    if target is not None:
        target, tgp = _i32(target)
        al = np.empty((P, N), dtype=np.int32)
        alp = al.ctypes.data_as(_i32p)
    else:
        tgp, al, alp = None, None, None
    lib.oracle_draft_all(tp, pp, lp, P, N, max_len, k, eps, L, lib.oracle_alpha_q(float(alpha)),
                         score_mode, pool_mode, _extras(include_self, backoff), d.ctypes.data_as(_i32p),
                         dl.ctypes.data_as(_i32p), ts.ctypes.data_as(_f32p), ps.ctypes.data_as(_f32p), tgp, alp)
    return dict(draft=d, draft_len=dl, token_scores=ts, path_scores=ps, accept_len=al)


def draft_many(tok, prob, lengths, k, L, alpha=1.0, score_mode=0, targets=None, eps=0, pool_mode=0,
               include_self=False, backoff=False, threads=None):
    """draft_all for S independent history states of one path set, on `threads` host threads
    (default: host_threads()).  tok [P][N][max_len], lengths [S][P][N], targets [S][P][N][L] or
    None.  Returns the dict of draft_all with a leading S axis on every array."""
    tok, tp = _i32(tok)
    prob, pp = _f32(prob)
    lengths, lp = _i32(lengths)
    P, N, max_len = tok.shape
    S = lengths.shape[0]
    assert lengths.shape == (S, P, N)
    d = np.empty((S, P, N, L), dtype=np.int32)
    dl = np.empty((S, P, N), dtype=np.int32)
    ts = np.empty((S, P, N, L), dtype=np.float32)
    ps = np.empty((S, P, N), dtype=np.float32)
    lib = _load()
    if targets is not None:
        targets, tgp = _i32(targets)
        assert targets.shape == (S, P, N, L)
        al = np.empty((S, P, N), dtype=np.int32)
        alp = al.ctypes.data_as(_i32p)
    else:
        tgp, al, alp = None, None, None
    n_threads = host_threads() if threads is None else int(threads)
    lib.oracle_draft_many(tp, pp, lp, S, P, N, max_len, k, eps, L, lib.oracle_alpha_q(float(alpha)),
                          score_mode, pool_mode, _extras(include_self, backoff), n_threads,
                          d.ctypes.data_as(_i32p), dl.ctypes.data_as(_i32p), ts.ctypes.data_as(_f32p),
                          ps.ctypes.data_as(_f32p), tgp, alp)
    return dict(draft=d, draft_len=dl, token_scores=ts, path_scores=ps, accept_len=al)


def accept_loop(future_tok, future_prob, length, k, L, n_steps, alpha=1.0, score_mode=0, eps=0, pool_mode=0,
                include_self=False, backoff=False):
    """The propose / verify / accept loop with every path's own future standing in for the
    model.  future_tok [P][N][max_len], length [P][N] = lengths on entry.  Returns dict(draft
    [S][P][N][L], draft_len, accept_len, path_len [S][P][N], final_len [P][N])."""
    tok, tp = _i32(future_tok)
    prob, pp = _f32(future_prob)
    length = np.array(length, dtype=np.int32, copy=True, order="C")
    P, N, max_len = tok.shape
    assert L <= 64
    d = np.empty((n_steps, P, N, L), dtype=np.int32)
    dl = np.empty((n_steps, P, N), dtype=np.int32)
    al = np.empty((n_steps, P, N), dtype=np.int32)
    pl = np.empty((n_steps, P, N), dtype=np.int32)
    lib = _load()
    lib.oracle_accept_loop(tp, pp, length.ctypes.data_as(_i32p), P, N, max_len, k, eps, L,
                           lib.oracle_alpha_q(float(alpha)), score_mode, pool_mode,
                           _extras(include_self, backoff), n_steps,
                           d.ctypes.data_as(_i32p), dl.ctypes.data_as(_i32p), al.ctypes.data_as(_i32p),
                           pl.ctypes.data_as(_i32p))
    return dict(draft=d, draft_len=dl, accept_len=al, path_len=pl, final_len=length)
