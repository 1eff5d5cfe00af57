"""Thin ctypes binding over the csd C-ABI (include/csd.h).

Argument marshalling only: every step of the drafting path runs in the HIP
kernels of libcsd.so.  PyTorch supplies device memory and the stream.  There is
no CPU fallback: if the library is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from .build import LIBRARY, build_library

MATCH_AUTO, MATCH_SCAN, MATCH_INDEX = 0, 1, 2
INCLUDE_SELF, QUERY_BACKOFF = 4, 8      # options OR-ed to a MATCH_* value
POOL_DAG, POOL_TREE, POOL_LIST = 0, 1, 2
STATUS_CAPACITY, STATUS_TOKEN_RANGE, STATUS_TABLE_FULL = 1, 2, 4
OK, ERR_INVALID_ARG, ERR_CAPACITY, ERR_WORKSPACE, ERR_HIP, ERR_UNIMPLEMENTED = 0, -1, -2, -3, -4, -5
ERR_SCRATCH_LIMIT = -6
NOALLOC_SCRATCH_BYTES = 1 << 20

EXPORTS = ["csd_workspace_bytes", "csd_create", "csd_destroy", "csd_reset", "csd_append",
           "csd_draft", "csd_accept", "csd_step", "csd_replay", "csd_accept_loop", "csd_accept_loop_noalloc", "csd_set_steps_per_launch", "csd_status",
           "csd_dump_matches",
           "csd_dump_edges", "csd_debug_copy", "csd_strerror"]


class Config(ctypes.Structure):
    _fields_ = [("n_problems", ctypes.c_int32), ("n_paths", ctypes.c_int32),
                ("max_len", ctypes.c_int32), ("vocab", ctypes.c_int32),
                ("max_query_len", ctypes.c_int32), ("max_draft_len", ctypes.c_int32),
                ("alpha", ctypes.c_float), ("score_mode", ctypes.c_int32),
                ("flags", ctypes.c_int32), ("max_edits", ctypes.c_int32),
                ("pool_mode", ctypes.c_int32)]


class CsdError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__("%s failed: %s (%d)" % (what, strerror(code), code))
        self.code = code


_lib = None
_vp = ctypes.c_void_p


def load() -> ctypes.CDLL:
    """Loads libcsd.so (building it first only if it has never been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIBRARY):
            build_library()
        lib = ctypes.CDLL(LIBRARY)
        i32, i64 = ctypes.c_int32, ctypes.c_int64
        cfgp = ctypes.POINTER(Config)
        lib.csd_workspace_bytes.argtypes = [cfgp, ctypes.POINTER(ctypes.c_size_t)]
        lib.csd_create.argtypes = [cfgp, _vp, ctypes.c_size_t, _vp, ctypes.POINTER(_vp)]
        lib.csd_destroy.argtypes = [_vp]
        lib.csd_reset.argtypes = [_vp, _vp]
        lib.csd_append.argtypes = [_vp, _vp, _vp, _vp, i32, _vp]
        lib.csd_draft.argtypes = [_vp, i32, i32, _vp, _vp, _vp, _vp, _vp]
        lib.csd_accept.argtypes = [_vp, _vp, _vp, _vp, i32, _vp, _vp]
        lib.csd_step.argtypes = [_vp, _vp, _vp, _vp, i32, i32, i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
        lib.csd_replay.argtypes = [_vp, i32, _vp, _vp, i32, i32, _vp, _vp, _vp, _vp, _vp, _vp, i32, _vp]
        lib.csd_accept_loop.argtypes = [_vp, i32, _vp, _vp, i32, i32, _vp, ctypes.c_size_t, _vp, _vp, _vp, _vp,
                                        _vp]
        lib.csd_accept_loop_noalloc.argtypes = [_vp, i32, _vp, _vp, i32, i32, _vp, _vp, _vp, _vp, _vp]
        lib.csd_set_steps_per_launch.argtypes = [_vp, i32]
        lib.csd_status.argtypes = [_vp, ctypes.POINTER(ctypes.c_uint32), _vp]
        lib.csd_dump_matches.argtypes = [_vp, i32, _vp, _vp, i64, _vp]
        lib.csd_dump_edges.argtypes = [_vp, i32, i32, _vp, _vp, _vp, i64, _vp]
        lib.csd_debug_copy.argtypes = [_vp, _vp, ctypes.c_size_t, _vp]
        lib.csd_strerror.argtypes = [ctypes.c_int]
        lib.csd_strerror.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name != "csd_strerror":
                getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def strerror(code: int) -> str:
    return load().csd_strerror(code).decode()


def debug_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Plain device copy of known size (calibration of hardware traffic counters)."""
    nbytes = src.numel() * src.element_size()
    rc = load().csd_debug_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream())
    if rc != OK:
        raise CsdError(rc, "csd_debug_copy")


def workspace_bytes(cfg: Config) -> int:
    out = ctypes.c_size_t(0)
    rc = load().csd_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out))
    if rc != OK:
        raise CsdError(rc, "csd_workspace_bytes")
    return out.value


def _ptr(t: Optional[torch.Tensor], dtype, numel: Optional[int] = None):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("expected a contiguous device tensor of dtype %s" % dtype)
    if numel is not None and t.numel() < numel:
        raise ValueError("tensor has %d elements, needs %d" % (t.numel(), numel))
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Index:
    """The draft pool of P problems x N paths on the current device."""

    def __init__(self, n_problems, n_paths, max_len, vocab, max_query_len, max_draft_len,
                 alpha=1.0, score_mode=0, flags=MATCH_AUTO, device="cuda", max_edits=0,
                 pool_mode=POOL_DAG):
        self.cfg = Config(n_problems, n_paths, max_len, vocab, max_query_len, max_draft_len,
                          alpha, score_mode, flags, max_edits, pool_mode)
        self.P, self.N = n_problems, n_paths
        self.rows = n_problems * n_paths
        self.device = torch.device(device)
        nbytes = workspace_bytes(self.cfg)
        # +256 so that a 256-byte aligned start always exists inside the buffer
        self._buf = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self._buf.data_ptr()
        self._ws = (base + 255) // 256 * 256
        self._h = _vp()
        rc = load().csd_create(ctypes.byref(self.cfg), self._ws, nbytes, _stream(),
                               ctypes.byref(self._h))
        if rc != OK:
            raise CsdError(rc, "csd_create")

    def close(self):
        if getattr(self, "_h", None):
            load().csd_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: module globals may already be gone
            pass

    def _check(self, rc, what):
        if rc != OK:
            raise CsdError(rc, what)

    def set_steps_per_launch(self, steps: int):
        """Steps per launch of replay() and accept_loop() (1 = a launch per step)."""
        self._check(load().csd_set_steps_per_launch(self._h, steps), "csd_set_steps_per_launch")

    def reset(self):
        self._check(load().csd_reset(self._h, _stream()), "csd_reset")

    def append(self, tokens, probs=None, counts=None, n=None):
        """tokens [P][N][n] int32, probs same float32 or None, counts [P][N] int32 or None."""
        if n is None:
            n = tokens.numel() // self.rows
        self._check(load().csd_append(self._h, _ptr(tokens, torch.int32, self.rows * n),
                                      _ptr(probs, torch.float32, self.rows * n),
                                      _ptr(counts, torch.int32, self.rows), n, _stream()),
                    "csd_append")

    def draft(self, query_len, draft_len, out=None, scores=True):
        """Returns dict(tokens [P][N][L], length [P][N], token_scores, path_scores)."""
        P, N, L = self.P, self.N, draft_len
        if out is None:
            out = dict(tokens=torch.empty((P, N, L), dtype=torch.int32, device=self.device),
                       length=torch.empty((P, N), dtype=torch.int32, device=self.device),
                       token_scores=torch.empty((P, N, L), dtype=torch.float32,
                                                device=self.device) if scores else None,
                       path_scores=torch.empty((P, N), dtype=torch.float32,
                                               device=self.device) if scores else None)
        self._check(load().csd_draft(self._h, query_len, draft_len,
                                     _ptr(out["tokens"], torch.int32, self.rows * L),
                                     _ptr(out["length"], torch.int32, self.rows),
                                     _ptr(out.get("token_scores"), torch.float32, self.rows * L),
                                     _ptr(out.get("path_scores"), torch.float32, self.rows),
                                     _stream()), "csd_draft")
        return out

    def accept(self, draft_tokens, draft_len_t, targets, draft_len, out=None):
        if out is None:
            out = torch.empty((self.P, self.N), dtype=torch.int32, device=self.device)
        self._check(load().csd_accept(self._h, _ptr(draft_tokens, torch.int32, self.rows * draft_len),
                                      _ptr(draft_len_t, torch.int32, self.rows),
                                      _ptr(targets, torch.int32, self.rows * draft_len), draft_len,
                                      _ptr(out, torch.int32, self.rows), _stream()), "csd_accept")
        return out

    def _outputs(self, L, scores, lead=()):
        P, N = self.P, self.N
        mk = lambda shape, dt: torch.empty(tuple(lead) + shape, dtype=dt, device=self.device)
        return dict(tokens=mk((P, N, L), torch.int32), length=mk((P, N), torch.int32),
                    token_scores=mk((P, N, L), torch.float32) if scores else None,
                    path_scores=mk((P, N), torch.float32) if scores else None)

    def step(self, tokens, probs, counts, n, query_len, draft_len, out=None, targets=None,
             accept_out=None, scores=True):
        """One fused decode step (append + draft [+ accept]) in one launch."""
        L = draft_len
        if out is None:
            out = self._outputs(L, scores)
        if targets is not None and accept_out is None:
            accept_out = torch.empty((self.P, self.N), dtype=torch.int32, device=self.device)
        self._check(load().csd_step(self._h, _ptr(tokens, torch.int32, self.rows * n),
                                    _ptr(probs, torch.float32, self.rows * n),
                                    _ptr(counts, torch.int32, self.rows), n, query_len, L,
                                    _ptr(out["tokens"], torch.int32, self.rows * L),
                                    _ptr(out["length"], torch.int32, self.rows),
                                    _ptr(out.get("token_scores"), torch.float32, self.rows * L),
                                    _ptr(out.get("path_scores"), torch.float32, self.rows),
                                    _ptr(targets, torch.int32, self.rows * L),
                                    _ptr(accept_out, torch.int32, self.rows), _stream()), "csd_step")
        out["accept"] = accept_out
        return out

    def replay(self, n_steps, tokens, probs, query_len, draft_len, out=None, targets=None,
               accept_out=None, fused=True, scores=True):
        """n_steps decode steps from a host loop inside the library.
        tokens / probs [n_steps][P][N]; outputs get a leading n_steps axis."""
        L, S = draft_len, n_steps
        if out is None:
            out = self._outputs(L, scores, lead=(S,))
        if targets is not None and accept_out is None:
            accept_out = torch.empty((S, self.P, self.N), dtype=torch.int32, device=self.device)
        self._check(load().csd_replay(self._h, S, _ptr(tokens, torch.int32, S * self.rows),
                                      _ptr(probs, torch.float32, S * self.rows), query_len, L,
                                      _ptr(out["tokens"], torch.int32, S * self.rows * L),
                                      _ptr(out["length"], torch.int32, S * self.rows),
                                      _ptr(out.get("token_scores"), torch.float32, S * self.rows * L),
                                      _ptr(out.get("path_scores"), torch.float32, S * self.rows),
                                      _ptr(targets, torch.int32, S * self.rows * L),
                                      _ptr(accept_out, torch.int32, S * self.rows),
                                      1 if fused else 0, _stream()), "csd_replay")
        out["accept"] = accept_out
        return out

    def accept_loop(self, n_steps, future_tokens, future_probs, query_len, draft_len, out=None,
                    min_scratch=False):
        """n_steps of the propose / verify / accept loop with each path's own future
        (future_tokens / future_probs [P][N][max_len]) standing in for the model.  Returns
        dict(tokens [S][P][N][L], length, accept, path_len [S][P][N]).  min_scratch: hand over
        the minimum of scratch memory instead of twice as much (same results, more launches)."""
        L, S = draft_len, n_steps
        if out is None:
            out = dict(tokens=torch.empty((S, self.P, self.N, L), dtype=torch.int32, device=self.device))
            for name in ("length", "accept", "path_len"):
                out[name] = torch.empty((S, self.P, self.N), dtype=torch.int32, device=self.device)
        cells = self.rows * self.cfg.max_len
        nbytes = (1 if min_scratch else 2) * self.rows * (3 * L + 3) * 4   # twice the minimum: one launch per step
        scratch = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self._check(load().csd_accept_loop(self._h, S, _ptr(future_tokens, torch.int32, cells),
                                           _ptr(future_probs, torch.float32, cells), query_len, L,
                                           scratch.data_ptr(), nbytes,
                                           _ptr(out["tokens"], torch.int32, S * self.rows * L),
                                           _ptr(out["length"], torch.int32, S * self.rows),
                                           _ptr(out["accept"], torch.int32, S * self.rows),
                                           _ptr(out["path_len"], torch.int32, S * self.rows), _stream()),
                    "csd_accept_loop")
        out["_scratch"] = scratch        # enqueued work still uses it
        return out

    def accept_loop_noalloc(self, n_steps, future_tokens, future_probs, query_len, draft_len, out):
        """csd_accept_loop_noalloc: the same loop with the step buffers in the library's fixed
        device array.  `out` (as returned by accept_loop) must be given: nothing is allocated."""
        L, S = draft_len, n_steps
        cells = self.rows * self.cfg.max_len
        self._check(load().csd_accept_loop_noalloc(
            self._h, S, _ptr(future_tokens, torch.int32, cells), _ptr(future_probs, torch.float32, cells),
            query_len, L, _ptr(out["tokens"], torch.int32, S * self.rows * L),
            _ptr(out["length"], torch.int32, S * self.rows), _ptr(out["accept"], torch.int32, S * self.rows),
            _ptr(out["path_len"], torch.int32, S * self.rows), _stream()), "csd_accept_loop_noalloc")
        return out

    def status(self) -> int:
        flags = ctypes.c_uint32(0)
        self._check(load().csd_status(self._h, ctypes.byref(flags), _stream()), "csd_status")
        return flags.value

    def dump_matches(self, query_len, cap=None):
        """(je int32 [n][2], off int32 [P*N+1]) on the host; rows in canonical order."""
        cap = cap if cap is not None else 1 << 20
        je = torch.empty((max(cap, 1), 2), dtype=torch.int32, device=self.device)
        off = torch.empty(self.rows + 1, dtype=torch.int32, device=self.device)
        self._check(load().csd_dump_matches(self._h, query_len, je.data_ptr(), off.data_ptr(), cap,
                                            _stream()), "csd_dump_matches")
        off = off.cpu().numpy()
        return je[:off[-1]].cpu().numpy(), off

    def dump_edges(self, query_len, draft_len, cap=None):
        """(duv int32 [n][3], cs uint64 [n][2], off int32 [P*N+1]) on the host."""
        cap = cap if cap is not None else 1 << 20
        duv = torch.empty((max(cap, 1), 3), dtype=torch.int32, device=self.device)
        cs = torch.empty((max(cap, 1), 2), dtype=torch.int64, device=self.device)
        off = torch.empty(self.rows + 1, dtype=torch.int32, device=self.device)
        self._check(load().csd_dump_edges(self._h, query_len, draft_len, duv.data_ptr(),
                                          cs.data_ptr(), off.data_ptr(), cap, _stream()),
                    "csd_dump_edges")
        off = off.cpu().numpy()
        n = off[-1]
        return duv[:n].cpu().numpy(), cs[:n].cpu().numpy().view("uint64"), off
