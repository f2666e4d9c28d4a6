"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and its pure
host functions (plan, task order, lock-free queue, argument errors) agree with the oracle."""
import ctypes
import os
import re

import pytest

from paper_1511_04348_amd import binding as tg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(tg.LIB_PATH):
        from paper_1511_04348_amd import build
        build.build()
    return tg.load()


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "tgemm.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b((?:tgemm|mlp)_[a-z_]+)\s*\(", hdr))
    assert declared == set(tg.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_sizes():
    assert ctypes.sizeof(tg.tgemm_opts) == 44
    assert ctypes.sizeof(tg.tgemm_task) == 64
    assert ctypes.sizeof(tg.tgemm_stats) == 96
    assert ctypes.sizeof(tg.tgemm_trace_rec) == 48
    assert ctypes.sizeof(tg.tgemm_mlp_trace_rec) == 48


@pytest.mark.parametrize("M,N,K,T", [(1000, 1000, 1000, 256), (8000, 8000, 8000, 1024), (65536, 65536, 65536, 4096),
                                     (7, 13, 5, 3), (5, 5, 5, 8), (4096, 10000, 16384, 1024), (1, 1, 1, 1), (0, 4, 4, 2)])
def test_plan_matches_oracle_bit_exact(lib, oracle, M, N, K, T):
    got = tg.tgemm_plan(M, N, K, T)
    exp = oracle.plan_tiles(M, N, K, T)
    assert len(got) == len(exp)
    for g, e in zip(got, exp):
        assert g == e


def test_task_order_matches_oracle(lib, oracle):
    from oracle.lru import task_order
    for n_i, n_j in [(1, 1), (3, 4), (16, 16), (5, 1), (1, 7)]:
        assert tg.tgemm_task_order(n_i, n_j, tg.TGEMM_ORDER_ROW_MAJOR) == task_order(n_i, n_j, "row_major")
        assert tg.tgemm_task_order(n_i, n_j, tg.TGEMM_ORDER_SERPENTINE) == task_order(n_i, n_j, "serpentine")
        for strip in (1, 2, 3, 7, 100):
            got = tg.tgemm_task_order(n_i, n_j, tg.TGEMM_ORDER_STRIPS, strip)
            assert got == task_order(n_i, n_j, "strips", strip)
            assert sorted(got) == list(range(n_i * n_j))


@pytest.mark.parametrize("n,p,c", [(0, 1, 1), (1, 1, 1), (1000, 1, 1), (200000, 4, 4), (50000, 1, 6), (50000, 6, 1)])
def test_queue_every_id_exactly_once(lib, n, p, c):
    counts = tg.tgemm_queue_selftest(n, p, c)
    assert len(counts) == n and all(x == 1 for x in counts)


def test_argument_errors_without_gpu(lib):
    n = ctypes.c_int64()
    assert lib.tgemm_plan(4, 4, 4, 0, None, 0, ctypes.byref(n)) == tg.TGEMM_EARG
    assert b"tgemm_plan" in lib.tgemm_last_error()
    assert lib.tgemm_plan(4, 4, 4, 2, None, 0, None) == tg.TGEMM_EARG
    assert lib.tgemm_run(None, None, None, None, 1, 1, 1, 1, 0, 0) == tg.TGEMM_EARG
    assert lib.tgemm_create(None, 0, None, None) == tg.TGEMM_EARG
    assert lib.tgemm_destroy(None) == tg.TGEMM_OK
    assert lib.tgemm_task_order(2, 2, 9, 1, (ctypes.c_int64 * 4)()) == tg.TGEMM_EARG
    assert lib.tgemm_task_order(2, 2, tg.TGEMM_ORDER_STRIPS, 0, (ctypes.c_int64 * 4)()) == tg.TGEMM_EARG
    assert tg.tgemm_strerror(tg.TGEMM_EBUDGET).startswith("hbm_budget")


def test_invalidate_rejects_null_arguments(lib):
    assert lib.tgemm_invalidate(None, None) == tg.TGEMM_EARG


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(tg, "_lib", None)
    monkeypatch.setattr(tg, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        tg.load()


def test_header_is_plain_c_and_links_from_c(lib, tmp_path):
    """include/tgemm.h compiles as C99 and as C++11 with -pedantic, and a plain C program linked
    against the library sees the struct sizes the binding mirrors and can call host-only entry points."""
    import shutil
    import subprocess
    gcc, gxx = shutil.which("gcc"), shutil.which("g++")
    if gcc is None or gxx is None:
        pytest.skip("no gcc / g++")
    inc = os.path.join(ROOT, "include")
    src = os.path.join(ROOT, "tests", "native", "abi_from_c.c")
    for cmd in ([gcc, "-std=c99", "-x", "c"], [gxx, "-std=c++11", "-x", "c++"]):
        r = subprocess.run(cmd + ["-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-fsyntax-only", src],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout
    exe = str(tmp_path / "abi_from_c")
    libdir = os.path.dirname(tg.LIB_PATH)
    r = subprocess.run([gcc, "-std=c99", "-I", inc, src, "-o", exe, "-L", libdir, "-ltgemm", "-Wl,-rpath," + libdir],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode == 0, r.stdout
    out = r.stdout.splitlines()
    sizes = [ctypes.sizeof(t) for t in (tg.tgemm_opts, tg.tgemm_task, tg.tgemm_stats, tg.tgemm_trace_rec, tg.tgemm_mlp_trace_rec,
                                        tg.tgemm_balance, tg.tgemm_segment)]
    assert out[0] == "sizes " + " ".join(str(s) for s in sizes)
    assert out[1] == "order 0 1 2 3 7 6 5 4 8 9 10 11"
    assert out[2] == "balance 1 768 193 447"
    assert out[3].startswith("bad order -> %d" % tg.TGEMM_EARG)
