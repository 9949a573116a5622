"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects
bad arguments before any HIP call (so these run on a machine without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    import paper_2501_08071_amd as pkg
    pkg.lib  # force the load
    return pkg


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(attn_[a-z0-9_]+)\s*\(", text)))


def declared_rowops_symbols():
    text = open(os.path.join(ROOT, "include", "rowops.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:rowops_|softmax_rows_|rmsnorm_)[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(P):
    names = declared_symbols()
    assert {"attn_fwd", "attn_fwd_o16", "attn_supported", "attn_status_str"} <= set(names)
    for n in names:
        assert hasattr(P.lib, n), f"{n} is declared in attn.h but not exported"
    names = declared_rowops_symbols()
    assert names == ["rmsnorm_fwd", "rowops_path", "rowops_status_str", "softmax_rows_fwd"]
    for n in names:
        assert hasattr(P.lib, n), f"{n} is declared in rowops.h but not exported"
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "gemm.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(gemm_[a-z0-9_]+)\s*\(", text)))
    assert names == ["gemm_leakyrelu_fwd", "gemm_path", "gemm_status_str"]
    for n in names:
        assert hasattr(P.lib, n), f"{n} is declared in gemm.h but not exported"
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "probe.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(probe_[a-z0-9_]+)\s*\(", text)))
    assert names == ["probe_empty", "probe_issue_share", "probe_l2_read", "probe_mfma", "probe_softmax_valu"]
    for n in names:
        assert hasattr(P.lib, n), f"{n} is declared in probe.h but not exported"
    assert not any(n.startswith("probe") or "probe" in n for n in declared_symbols())   # measuring aids stay out of attn.h
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["attn.h", "gemm.h", "probe.h", "rowops.h"]


def test_gemm_paths_status_and_bad_arguments(P):
    seen = {P.gemm_status_str(st) for st in (0, -1, -2, -3, -4, -6, -7)}
    assert len(seen) == 7 and "unknown status" not in seen and P.gemm_status_str(-5) == "unknown status"
    for dt in (0, 1):
        assert P.gemm_path(1, 512, 512, 2048, dt) == 5           # the paper's shape: 256 tiles of 32 x 32, K split inside the workgroup
        assert P.gemm_path(1, 512, 512, 128, dt) == 3 and P.gemm_path(1, 1024, 512, 512, dt) == 3   # K too short; too many tiles
        assert P.gemm_path(1, 4096, 4096, 4096, dt) == 1 and P.gemm_path(4, 1024, 1024, 64, dt) == 2
        assert P.gemm_path(1, 2048, 2048, 2048, dt) == 2 and P.gemm_path(1, 3584, 3584, 32, dt) == 1
        assert P.gemm_path(1, 64, 64, 48, dt) == 4 and P.gemm_path(1, 64, 12, 64, dt) == 4 and P.gemm_path(1, 8, 8, 0, dt) == 4
        assert P.gemm_path(1, 8, 8, 1 << 23, dt) == 4
        assert P.gemm_path(0, 0, 0, 0, dt) == 4                  # valid and empty
        assert P.gemm_path(-1, 8, 8, 8, dt) == 0 and P.gemm_path(1, 1 << 20, 8, 1 << 20, dt) == 0
    assert P.gemm_path(1, 8, 8, 32, 2) == 0
    ok = 4096
    f = P.gemm_leakyrelu_fwd_raw
    assert f(0, ok, ok, 1, 8, 8, 32, 0.01, 0, 0) == -1 and f(ok, 0, ok, 1, 8, 8, 32, 0.01, 0, 0) == -1
    assert f(ok, ok, 0, 1, 8, 8, 32, 0.01, 0, 0) == -1 and f(0, 0, 0, 1, 8, 8, 0, 0.01, 0, 0) == -1
    assert f(ok, ok, ok, -1, 8, 8, 32, 0.01, 0, 0) == -2 and f(ok, ok, ok, 1, 8, -8, 32, 0.01, 0, 0) == -2
    assert f(ok, ok, ok, 1, 1 << 16, 8, 1 << 16, 0.01, 0, 0) == -2 and f(ok, ok, ok, 70000, 8, 8, 32, 0.01, 0, 0) == -2
    assert f(ok, ok, ok, 1, 8, 8, 32, 0.01, 5, 0) == -3
    assert f(ok, ok, ok, 1, 8, 8, 32, float("inf"), 0, 0) == -4 and f(ok, ok, ok, 1, 8, 8, 32, float("nan"), 0, 0) == -4
    assert f(ok + 8, ok, ok, 1, 8, 8, 32, 0.01, 0, 0) == -6 and f(ok, ok, ok + 2, 1, 8, 8, 32, 0.01, 0, 0) == -6
    assert f(0, 0, 0, 0, 8, 8, 32, 0.01, 0, 0) == 0 and f(0, 0, 0, 1, 0, 8, 32, 0.01, 0, 0) == 0 and f(0, 0, 0, 1, 8, 0, 32, 0.01, 0, 0) == 0


def test_rowops_status_strings_and_paths(P):
    seen = {P.rowops_status_str(st) for st in (0, -1, -2, -3, -4, -6, -7)}
    assert len(seen) == 7 and "unknown status" not in seen
    assert P.rowops_status_str(-5) == "unknown status" and P.rowops_status_str(3) == "unknown status"
    for op in (0, 1):
        for dt in (0, 1):
            assert P.rowops_path(op, 8, dt) == 1 and P.rowops_path(op, 64, dt) == 1 and P.rowops_path(op, 4096, dt) == 1
            assert P.rowops_path(op, 16384, dt) == 1 and P.rowops_path(op, 16392, dt) == 2
            assert P.rowops_path(op, 1, dt) == 2 and P.rowops_path(op, 4095, dt) == 2 and P.rowops_path(op, 1 << 24, dt) == 2
            assert P.rowops_path(op, 0, dt) == 0 and P.rowops_path(op, (1 << 24) + 8, dt) == 0
        assert P.rowops_path(op, 64, 2) == 0
    assert P.rowops_path(2, 64, 0) == 0


def test_rowops_bad_arguments_rejected_without_a_gpu(P):
    ok = 4096  # any non-null 16-byte aligned address: validation fails before it is touched
    sm, rn = P.softmax_rows_fwd_raw, P.rmsnorm_fwd_raw
    assert sm(0, ok, 4, 64, 0, 0) == -1 and sm(ok, 0, 4, 64, 0, 0) == -1
    assert sm(ok, ok, -1, 64, 0, 0) == -2 and sm(ok, ok, 4, 0, 0, 0) == -2 and sm(ok, ok, 4, (1 << 24) + 1, 0, 0) == -2
    assert sm(ok, ok, 1 << 30, 1 << 20, 0, 0) == -2
    assert sm(ok, ok, 4, 64, 2, 0) == -3 and sm(ok, ok, 4, 64, -1, 0) == -3
    assert sm(ok + 2, ok, 4, 64, 0, 0) == -6 and sm(ok, ok + 8, 4, 64, 0, 0) == -6
    assert sm(0, 0, 0, 64, 0, 0) == 0          # an empty input is valid and launches nothing
    assert rn(0, ok, ok, 4, 64, 1e-6, 0, 0) == -1 and rn(ok, 0, ok, 4, 64, 1e-6, 0, 0) == -1 and rn(ok, ok, 0, 4, 64, 1e-6, 0, 0) == -1
    assert rn(ok, ok, ok, -2, 64, 1e-6, 0, 0) == -2 and rn(ok, ok, ok, 4, -64, 1e-6, 0, 0) == -2
    assert rn(ok, ok, ok, 4, 64, 1e-6, 7, 0) == -3
    assert rn(ok, ok, ok, 4, 64, -1e-6, 0, 0) == -4 and rn(ok, ok, ok, 4, 64, float("nan"), 0, 0) == -4
    assert rn(ok, ok, ok, 4, 64, float("inf"), 0, 0) == -4
    assert rn(ok, ok + 4, ok, 4, 64, 1e-6, 0, 0) == -6
    assert rn(0, 0, 0, 0, 64, 1e-6, 0, 0) == 0


def test_probes_reject_bad_arguments(P):
    f = P.lib.probe_mfma
    assert f(None, 1, 1, 0, 0, None) == -1 and f(4096, 0, 1, 0, 0, None) == -1 and f(4096, 1, 0, 0, 0, None) == -1
    assert f(4096, 1, 1, 2, 0, None) == -1 and f(4096, 1 << 20, 1, 0, 0, None) == -1
    g = P.lib.probe_softmax_valu
    assert g(None, 1, 1, 0, None) == -1 and g(4096, 0, 1, 0, None) == -1 and g(4096, 1, 0, 1, None) == -1
    h = P.lib.probe_l2_read
    assert h(None, 4096, 1024, 8, 1, None) == -1 and h(4096, None, 1024, 8, 1, None) == -1
    assert h(4096, 4096, 1000, 8, 1, None) == -1 and h(4096, 4096, 0, 8, 1, None) == -1      # not whole steps
    assert h(4096 + 4, 4096, 1024, 8, 1, None) == -1 and h(4096, 4096, 1024, 0, 1, None) == -1
    e = P.lib.probe_empty
    assert e(0, 64, None) == -1 and e(1, 0, None) == -1 and e(1, 2048, None) == -1
    i = P.lib.probe_issue_share
    assert i(None, 1, 1, 1, 1, None) == -1 and i(4096, 0, 1, 1, 1, None) == -1 and i(4096, 1, 0, 1, 1, None) == -1
    assert i(4096, 1, 1, 1, 3, None) == -1 and i(4096, 1, 1, 0, 0, None) == -1 and i(4096 + 4, 1, 1, 1, 1, None) == -1


def test_status_strings(P):
    seen = set()
    for st in range(0, -8, -1):
        s = P.attn_status_str(st)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert P.attn_status_str(-99) == "unknown status"


def test_supported_matrix(P):
    for D in (32, 64, 128):
        for dt in (0, 1):
            for causal in (False, True):
                assert P.attn_supported(1, D, dt, causal) and P.attn_supported(16384, D, dt, causal)
                small, large = P.attn_kernel_name(1, 1, 128, D, dt, causal), P.attn_kernel_name(8, 64, 4096, D, dt, causal)
                assert small == f"attn_fwd_kernel<{dt}, {D}, {'true' if causal else 'false'}, 4>"
                assert large == f"attn_fwd_kernel<{dt}, {D}, {'true' if causal else 'false'}, 8>"
                assert P.attn_tile_rows(D, dt, causal) % 32 == 0 and P.attn_tile_keys(D, dt, causal) > 0
                assert P.attn_launch_rows(1, 1, 128, D, dt, causal) == 128 and P.attn_launch_rows(8, 64, 4096, D, dt, causal) == 256
                assert P.attn_launch_rows(1, 128, 256, D, dt, causal) == 128 and P.attn_launch_rows(1, 129, 256, D, dt, causal) == 256
                assert P.attn_launch_rows(0, 1, 128, D, dt, causal) == 0
    assert P.attn_launch_rows(1, 1, 128, 96, 0, False) == 0
    assert not P.attn_supported(128, 16, 0, False) and not P.attn_supported(128, 256, 0, False)
    assert not P.attn_supported(128, 64, 2, False)
    assert not P.attn_supported(0, 64, 0, False)
    assert P.attn_kernel_name(1, 1, 128, 96, 0, False) is None and P.attn_kernel_name(0, 1, 128, 64, 0, False) is None


@pytest.mark.parametrize("entry", ["attn_fwd_raw", "attn_fwd_o16_raw"])
def test_bad_arguments_rejected_without_a_gpu(P, entry):
    ok = 4096  # any non-null 16-byte aligned address: validation fails before it is touched
    f = getattr(P, entry)
    assert f(0, ok, ok, ok, ok, 1, 1, 8, 64, 0, 1.0, 0, 0) == -1
    assert f(ok, 0, ok, ok, ok, 1, 1, 8, 64, 0, 1.0, 0, 0) == -1
    assert f(ok, ok, 0, ok, ok, 1, 1, 8, 64, 0, 1.0, 0, 0) == -1
    assert f(ok, ok, ok, 0, ok, 1, 1, 8, 64, 0, 1.0, 0, 0) == -1
    assert f(ok, ok, ok, ok, ok, 0, 1, 8, 64, 0, 1.0, 0, 0) == -2
    assert f(ok, ok, ok, ok, ok, 1, -1, 8, 64, 0, 1.0, 0, 0) == -2
    assert f(ok, ok, ok, ok, ok, 1, 1, 0, 64, 0, 1.0, 0, 0) == -2
    assert f(ok, ok, ok, ok, ok, 1, 1, 8, 0, 0, 1.0, 0, 0) == -2
    assert f(ok, ok, ok, ok, ok, 1 << 20, 1 << 20, 8, 64, 0, 1.0, 0, 0) == -2
    assert f(ok, ok, ok, ok, ok, 1, 1, 8, 64, 0, 1.0, 2, 0) == -3
    assert f(ok, ok, ok, ok, ok, 1, 1, 8, 64, 0, float("nan"), 0, 0) == -4
    assert f(ok, ok, ok, ok, ok, 1, 1, 8, 64, 0, float("inf"), 0, 0) == -4
    assert f(ok, ok, ok, ok, ok, 1, 1, 8, 96, 0, 1.0, 0, 0) == -5
    assert f(ok + 8, ok, ok, ok, ok, 1, 1, 8, 64, 0, 1.0, 0, 0) == -7    # -6 is a refused launch, which needs a GPU to happen


def test_queries_from_two_threads_agree(P):
    """The query entry points and the argument checks keep no lazily built state: two host threads that call them at the
    same time get the answers of a single thread."""
    import threading

    def answers():
        out = []
        for _ in range(200):
            for D in (32, 64, 128, 96):
                for dt in (0, 1):
                    for causal in (0, 1):
                        out.append((P.attn_kernel_name(1, 3, 500, D, dt, causal), P.attn_kernel_name(4, 64, 500, D, dt, causal),
                                    P.attn_launch_rows(2, 2, 999, D, dt, causal), P.attn_tile_keys(D, dt, causal),
                                    P.attn_fwd_raw(4096, 4096, 4096, 4096 + 8, 0, 1, 1, 8, D, causal, 1.0, dt, 0),
                                    P.attn_fwd_raw(4096, 4096, 0, 4096, 0, 1, 1, 8, D, causal, 1.0, dt, 0),
                                    P.attn_status_str(-7)))
        return out

    want = answers()
    got = [None, None]

    def run(i):
        got[i] = answers()

    ts = [threading.Thread(target=run, args=(i,)) for i in range(2)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    assert got[0] == want and got[1] == want


def test_library_links_only_the_hip_runtime():
    """No torch types cross the boundary: the library must not depend on libtorch."""
    import subprocess
    lib = os.path.join(ROOT, "paper_2501_08071_amd", "libattn_gfx950.so")
    out = subprocess.run(["ldd", lib], capture_output=True, text=True).stdout
    assert "torch" not in out and "libc10" not in out
    assert "amdhip64" in out
