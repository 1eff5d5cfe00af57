"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, sizes its workspace, and rejects bad
arguments before anything is enqueued."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2503_05330_amd import binding
    return binding.load()


def test_exports_every_declared_symbol(lib):
    from paper_2503_05330_amd import binding
    header = open(os.path.join(ROOT, "include", "csd.h")).read()
    declared = sorted(set(re.findall(r"^(?:int|const char\*)\s+(csd_[a-z_]+)\s*\(", header, re.M)))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(lib, name), "libcsd.so does not export " + name
    assert sorted(binding.EXPORTS) == declared


def test_workspace_size_and_validation(lib):
    from paper_2503_05330_amd import binding as b
    good = dict(n_problems=1, n_paths=16, max_len=1024, vocab=32000, max_query_len=3,
                max_draft_len=8, alpha=1.0, score_mode=0, flags=0)
    n = b.workspace_bytes(b.Config(**good))
    assert n >= 2 * 16 * 1024 * 4 and n % 256 == 0
    out = ctypes.c_size_t(0)
    bad_cases = [dict(n_problems=0), dict(n_paths=-1), dict(max_len=0), dict(vocab=0),
                 dict(vocab=1 << 29), dict(max_query_len=0), dict(max_query_len=9),
                 dict(max_draft_len=0), dict(max_draft_len=33), dict(alpha=1.5),
                 dict(alpha=float("nan")), dict(score_mode=2), dict(n_paths=4097, max_len=4096)]
    for bad in bad_cases:
        cfg = b.Config(**{**good, **bad})
        assert lib.csd_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)) == b.ERR_INVALID_ARG, bad
    for unknown in (16, 3, 3 | b.INCLUDE_SELF, -1):        # an unknown option bit; no such matcher
        cfg = b.Config(**{**good, "flags": unknown})
        assert lib.csd_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)) == b.ERR_UNIMPLEMENTED, unknown
    for bad, code in ((dict(max_edits=-1), b.ERR_INVALID_ARG), (dict(max_edits=4), b.ERR_UNIMPLEMENTED),
                      (dict(max_edits=2, flags=b.MATCH_INDEX), b.ERR_UNIMPLEMENTED),
                      (dict(max_edits=1, flags=b.MATCH_INDEX, max_query_len=1), b.ERR_UNIMPLEMENTED),
                      (dict(pool_mode=-1), b.ERR_INVALID_ARG), (dict(pool_mode=3), b.ERR_INVALID_ARG)):
        cfg = b.Config(**{**good, **bad})
        assert lib.csd_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)) == code, bad
    for fine in (dict(max_edits=1), dict(max_edits=2), dict(max_edits=3, flags=b.MATCH_SCAN),
                 dict(max_edits=1, flags=b.MATCH_INDEX), dict(pool_mode=b.POOL_TREE),
                 dict(pool_mode=b.POOL_LIST, max_edits=1), dict(flags=b.INCLUDE_SELF),
                 dict(flags=b.MATCH_INDEX | b.QUERY_BACKOFF), dict(flags=b.MATCH_SCAN | b.INCLUDE_SELF | b.QUERY_BACKOFF)):
        cfg = b.Config(**{**good, **fine})
        assert lib.csd_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)) == b.OK, fine
    assert lib.csd_workspace_bytes(None, ctypes.byref(out)) == b.ERR_INVALID_ARG
    assert lib.csd_workspace_bytes(ctypes.byref(b.Config(**good)), None) == b.ERR_INVALID_ARG


def test_null_and_misaligned_arguments_are_rejected(lib):
    from paper_2503_05330_amd import binding as b
    cfg = b.Config(1, 4, 64, 100, 3, 5, 1.0, 0, 0)
    h = ctypes.c_void_p()
    assert lib.csd_create(ctypes.byref(cfg), None, 1 << 20, None, ctypes.byref(h)) == b.ERR_INVALID_ARG
    assert lib.csd_create(ctypes.byref(cfg), 256, 16, None, ctypes.byref(h)) == b.ERR_WORKSPACE
    assert lib.csd_create(ctypes.byref(cfg), 257, 1 << 20, None, ctypes.byref(h)) == b.ERR_WORKSPACE
    assert lib.csd_create(ctypes.byref(cfg), 256, 1 << 20, None, None) == b.ERR_INVALID_ARG
    assert h.value is None
    for fn, args in ((lib.csd_destroy, (None,)), (lib.csd_reset, (None, None)),
                     (lib.csd_append, (None, None, None, None, 1, None)),
                     (lib.csd_draft, (None, 1, 1, None, None, None, None, None)),
                     (lib.csd_accept, (None, None, None, None, 1, None, None)),
                     (lib.csd_accept_loop, (None, 1, None, None, 1, 1, None, 0, None, None, None, None, None)),
                     (lib.csd_accept_loop_noalloc, (None, 1, None, None, 1, 1, None, None, None, None, None)),
                     (lib.csd_status, (None, None, None)),
                     (lib.csd_dump_matches, (None, 1, None, None, 0, None)),
                     (lib.csd_dump_edges, (None, 1, 1, None, None, None, 0, None))):
        assert fn(*args) == b.ERR_INVALID_ARG
    for code in (0, -1, -2, -3, -4, -5, -6, -99):
        assert isinstance(b.strerror(code), str) and b.strerror(code)


def test_binding_has_no_cpu_fallback():
    """The product path must not import the oracle."""
    pkg = os.path.join(ROOT, "paper_2503_05330_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp", ".cuh", ".hpp", ".inc")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"import\s+oracle|from\s+oracle|csd_oracle|oracle[/.]", text), \
                    f + " reaches for the oracle"


def test_bound_behind_the_table_full_status_bit():
    """csd.h promises that CSD_STATUS_TABLE_FULL cannot occur with vocab <= 2^24: token ids are
    split into 2^20 classes by bits 12..31 of id * 0x9E3779B1 mod 2^32, so two ids of one class
    differ by delta / 0x9E3779B1 (mod 2^32) for some |delta| < 4096.  Counting the deltas whose
    quotient is smaller than the vocabulary bounds a class's population; two keys per id must
    fit the smallest table (256 slots)."""
    src = open(os.path.join(ROOT, "paper_2503_05330_amd", "csrc", "csd_dag.cuh")).read()
    assert "0x9E3779B1u) >> 12 & (n_class - 1)" in src          # the class function the header describes
    common = open(os.path.join(ROOT, "paper_2503_05330_amd", "csrc", "csd_common.cuh")).read()
    assert "kMaxClassBits = 20" in common and "LdsT<256, 256, 512, 1, 64> LdsWaveSmall" in common
    inv = pow(0x9E3779B1, -1, 1 << 32)

    def most_ids_in_a_class(vocab):
        n = 1
        for delta in range(-4095, 4096):
            d = (delta * inv) % (1 << 32)
            d -= (1 << 32) if d >= (1 << 31) else 0
            n += 1 if delta != 0 and abs(d) < vocab else 0
        return n
    assert most_ids_in_a_class(1 << 24) == 65 and 2 * 65 <= 256
    assert most_ids_in_a_class((1 << 29) - 1) == 2045
    assert most_ids_in_a_class(152064) == 1                   # the largest vocabulary of the workloads
