"""CPU-only checks of the C ABI: the shared library loads, exports every function that
include/ziplm.h declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2302_04089_amd import ziplm
    return ziplm.lib()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ziplm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ziplm_[a-z_]+)\s*\(", text)))


def test_header_functions_are_exported(L):
    from paper_2302_04089_amd import ziplm
    names = _declared_functions()
    assert len(names) == 23
    assert sorted(ziplm.EXPORTS) == names
    for n in names:
        assert getattr(L, n) is not None


def _signature(name):
    """Parameter list of `name` as declared in the header, comments and line breaks removed."""
    text = open(os.path.join(ROOT, "include", "ziplm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    m = re.search(r"\b%s\s*\(([^)]*)\)\s*;" % re.escape(name), text)
    assert m, name
    return re.sub(r"\s+", " ", m.group(1)).strip()


def test_design_table_of_exports_matches_the_header():
    """The design doc holds one table row per exported function (its signature and how it differs from the
    boundary the build plan started from); every declared function has a row, no row names a function
    that is not declared, and each row quotes the parameter list the header declares."""
    design = open(os.path.join(ROOT, "DESIGN.md")).read()
    rows = re.findall(r"^\| `(ziplm_[a-z_]+)` \| `([^`]*)` \|", design, flags=re.M)
    assert sorted(r[0] for r in rows) == _declared_functions()
    for name, params in rows:
        assert params == _signature(name), name


def test_library_reads_no_environment_variable_and_keeps_no_global_state():
    """The product sources call neither getenv nor a process-wide lock, and the only device allocation is the
    exchange-area helper."""
    csrc = os.path.join(ROOT, "paper_2302_04089_amd", "csrc")
    text = "".join(open(os.path.join(csrc, f)).read() for f in sorted(os.listdir(csrc)) if f.endswith((".hip", ".h")))
    code = re.sub(r"//[^\n]*|/\*.*?\*/", "", text, flags=re.S)
    assert "getenv" not in code and "std::mutex" not in code
    assert len(re.findall(r"\bhip(?:Ext)?Malloc\w*\s*\(", code)) == 1 and "hipFree" not in code


def test_version_and_status_strings(L):
    assert L.ziplm_version() >= 100
    seen = set()
    for code in (0, -1, -2, -3, -4, -5):
        s = L.ziplm_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert L.ziplm_status_string(12345) == b"unknown status"


def test_workspace_sizes_are_aligned_and_monotone(L):
    assert L.ziplm_hinv_workspace_bytes(0) == 0
    a, b = L.ziplm_hinv_workspace_bytes(768), L.ziplm_hinv_workspace_bytes(3072)
    assert 0 < a < b and a % 256 == 0 and b % 256 == 0
    # three padded fp32 squares
    assert b >= 3 * 3072 * 3072 * 4
    p1 = L.ziplm_prune_workspace_bytes(768, 3072, 1, 0)
    assert p1 >= 3072 * 3072 * 8 and p1 % 256 == 0
    assert L.ziplm_prune_workspace_bytes(768, 768, 64, 0) >= 768 * 768 * 8
    assert L.ziplm_prune_workspace_bytes(768, 770, 64, 0) == 0      # not divisible
    assert L.ziplm_hessian_workspace_bytes(3072, 0) == 0
    assert L.ziplm_hessian_workspace_bytes(3072, 16384) % 256 == 0


def test_argument_errors_return_before_any_device_work(L):
    one = ctypes.c_void_p(256)       # never dereferenced: validation fails first
    assert L.ziplm_hessian_accumulate(None, one, 4, 4, 4, 0, 2.0, None, 0, None) == -1
    assert L.ziplm_hessian_accumulate(one, None, 4, 4, 4, 0, 2.0, None, 0, None) == -1
    assert L.ziplm_hessian_accumulate(one, one, 4, 8, 4, 0, 2.0, None, 0, None) == -1      # ldx < n_tok
    assert L.ziplm_hessian_accumulate(one, one, 4, 8, 8, 7, 2.0, None, 0, None) == -1      # layout
    assert L.ziplm_hessian_accumulate(one, one, 0, 8, 8, 0, 2.0, None, 0, None) == -1
    assert L.ziplm_hessian_accumulate(one, None, 4, 0, 0, 0, 2.0, None, 0, None) == 0      # empty batch
    assert L.ziplm_hinv(None, one, 4, 0.01, None, None, one, 1 << 30, None) == -1
    assert L.ziplm_hinv(one, one, 4, -1.0, None, None, one, 1 << 30, None) == -1
    assert L.ziplm_hinv(one, one, 4, 0.01, None, None, None, 0, None) == -3
    assert L.ziplm_hinv(one, one, 4, 0.01, None, None, ctypes.c_void_p(8), 1 << 30, None) == -3   # misaligned
    assert L.ziplm_hinv(one, one, 4, 0.01, None, None, one, 16, None) == -3                        # too small
    pr = L.ziplm_structured_obs_prune
    big = 1 << 40
    assert pr(None, one, 2, 8, 1, 1, one, one, None, 0, None, None, None, None, 0, one, big, None) == -1
    assert pr(one, one, 2, 8, 3, 1, one, one, None, 0, None, None, None, None, 0, one, big, None) == -1     # 8 % 3
    assert pr(one, one, 2, 8, 1, 9, one, one, None, 0, None, None, None, None, 0, one, big, None) == -1     # n_remove > G
    assert pr(one, one, 2, 8, 1, 1, None, one, None, 0, None, None, None, None, 0, one, big, None) == -1    # no order_out
    assert pr(one, one, 2, 8, 1, 1, one, one, None, 1, None, None, None, None, 0, one, big, None) == -1     # snapshots w/o arrays
    steps = (ctypes.c_int32 * 1)(5)
    assert pr(one, one, 2, 8, 1, 1, one, one, None, 1, steps, one, None, None, 0, one, big, None) == -1     # step > n_remove
    assert pr(one, one, 2, 256, 128, 1, one, one, None, 0, None, None, None, None, 0, one, big, None) == -5 # group too large
    assert pr(one, one, 2, 8, 1, 1, one, one, None, 0, None, None, None, None, 0, None, 0, None) == -3
    assert pr(one, one, 2, 8, 1, 1, one, one, None, 0, None, None, None, one, 16, one, big, None) == -3     # exchange too small
    assert pr(one, one, 2, 8, 1, 1, one, one, None, 0, None, None, None, ctypes.c_void_p(8), big, one, big, None) == -3
    # exchange area: only the single-column loop has one, sized per launch of up to four layers
    xb = L.ziplm_prune_exchange_bytes
    assert xb(1, 768, 3072, 64) == 0 and xb(0, 768, 3072, 1) == 0
    x1, x4, x12 = xb(1, 768, 3072, 1), xb(4, 768, 3072, 1), xb(12, 768, 3072, 1)
    assert 0 < x1 <= 8 << 20 and x1 % 256 == 0 and x1 <= x4 == x12
    assert L.ziplm_exchange_alloc(0, ctypes.byref(ctypes.c_void_p())) == -1
    assert L.ziplm_exchange_alloc(1 << 20, None) == -1
    pe = L.ziplm_structured_obs_prune_eager
    assert L.ziplm_prune_eager_workspace_bytes(768, 3072, 0) >= 3072 * 3072 * 8
    assert pe(None, one, 2, 8, 1, one, one, None, 0, None, None, None, one, big, None) == -1
    assert pe(one, one, 2, 8, 9, one, one, None, 0, None, None, None, one, big, None) == -1               # n_remove > d_col
    assert pe(one, one, 2, 8, 1, one, one, None, 0, None, None, None, None, 0, None) == -3
    st = L.ziplm_selftest_bounded_wait
    info = ctypes.c_int(0)
    assert st(None, one, 2, 8, one, one, ctypes.byref(info), one, big, None) == -1
    assert st(one, one, 2, 8, one, one, None, one, big, None) == -1                                      # info is the result
    assert st(one, one, 2, 8, one, one, ctypes.byref(info), None, 0, None) == -3
    pb = L.ziplm_structured_obs_prune_batch
    assert L.ziplm_prune_batch_workspace_bytes(12, 768, 768, 64, 0) == 12 * L.ziplm_prune_workspace_bytes(768, 768, 64, 0)
    # single columns: a batch runs as a sequence of launches of a few layers each, which share the workspace
    one_layer = L.ziplm_prune_workspace_bytes(768, 3072, 1, 0)
    assert L.ziplm_prune_batch_workspace_bytes(1, 768, 3072, 1, 0) == one_layer
    assert 0 < L.ziplm_prune_batch_workspace_bytes(12, 768, 3072, 1, 0) <= 4 * one_layer
    assert L.ziplm_prune_batch_workspace_bytes(12, 768, 3072, 1, 0) == L.ziplm_prune_batch_workspace_bytes(4, 768, 3072, 1, 0)
    assert pb(one, one, 0, 64, 64, 8, 8, 4, 1, one, one, 0, None, None, None, None, 0, one, big, None) == -1    # no layers
    assert pb(one, one, 2, 63, 64, 8, 8, 4, 1, one, one, 0, None, None, None, None, 0, one, big, None) == -1    # stride too small
    assert pb(one, one, 2, 64, 64, 8, 8, 1, 9, one, one, 0, None, None, None, None, 0, one, big, None) == -1    # single columns: n_remove > G
    assert pb(one, one, 2, 64, 64, 8, 8, 1, 1, one, one, 0, None, None, None, None, 0, None, 0, None) == -3
    assert pb(one, one, 2, 256 * 256, 256 * 256, 8, 256, 128, 1, one, one, 0, None, None, None, None, 0, one, big, None) == -5   # group too large
    assert pb(one, one, 2, 64, 64, 8, 8, 4, 3, one, one, 0, None, None, None, None, 0, one, big, None) == -1    # n_remove > G
    assert pb(one, one, 2, 64, 64, 8, 8, 4, 1, one, one, 0, None, None, None, None, 0, None, 0, None) == -3
    assert pb(one, one, 2, 64, 64, 8, 8, 1, 1, one, one, 0, None, None, None, one, 16, one, big, None) == -3    # exchange too small
    me = L.ziplm_module_error
    assert L.ziplm_module_error_workspace_bytes(0, 8) == 0
    need = L.ziplm_module_error_workspace_bytes(768, 3072)
    assert need >= 6 * 24 * 8 and need % 256 == 0
    assert me(None, one, 2, 8, 0.0, one, one, big, None) == -1
    assert me(one, one, 2, 8, 0.0, None, one, big, None) == -1
    assert me(one, one, 2, 0, 0.0, one, one, big, None) == -1
    assert me(one, one, 2, 8, -1.0, one, one, big, None) == -1          # negative dampening
    assert me(one, one, 2, 8, 0.0, one, None, 0, None) == -3
    assert L.ziplm_prior(None, 4, one, one, None) == -1
    assert L.ziplm_prior(one, 4, None, one, None) == -1
    assert L.ziplm_prior(one, -1, one, one, None) == -1
    assert L.ziplm_prior(None, 0, one, None, None) == 0                 # empty run


def test_database_grid_of_the_paper():
    """Section 3.2, "Runtime awareness": 0..N heads removed; intermediate sizes 3072 * 0.9^i, i = 0..42.
    Truncation reproduces the sizes 1322, 302, 130 and 76 of the paper's example latency table (Appendix E)."""
    from paper_2302_04089_amd import ziplm
    assert ziplm.database_steps(12, "heads") == list(range(13))
    steps = ziplm.database_steps(3072, "columns")
    sizes = [3072 - s for s in steps]
    assert len(steps) == 43 and steps[0] == 0 and steps == sorted(set(steps))
    for printed in (3072, 1322, 302, 130, 76):
        assert printed in sizes
    assert min(sizes) == int(3072 * 0.9 ** 42) == 36
    small = ziplm.database_steps(8, "columns")          # duplicates collapse, never more removals than columns
    assert small == sorted(set(small)) and small[-1] <= 8
    with pytest.raises(ValueError):
        ziplm.database_steps(8, "rows")


def test_bench_refuses_more_than_one_gpu():
    """The build runs on one GPU; asking the benchmark for more ends with a message, before any device is touched."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert out.returncode == 2 and "one GPU" in out.stderr
