"""Host-side checks of the C ABI: the library loads, exports what the header
declares, and rejects bad problem descriptions without touching a GPU."""

import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "themis.h")


@pytest.fixture(scope="module")
def T():
    from paper_2407_14843_amd import themis
    if not os.path.exists(themis.LIB_PATH):
        from paper_2407_14843_amd import build
        build.build()
    return themis


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(themis_[a-z_]+)\s*\(", src)))


def test_exports_match_header(T):
    names = _declared_functions()
    assert len(names) >= 8
    lib = ctypes.CDLL(T.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in themis.h but not exported"
    assert sorted(T.EXPORTS) == names


def test_struct_size_matches_header(T):
    # 4 + 16 + 4 + 4 int32 fields
    assert ctypes.sizeof(T.ThemisProblem) == 4 * (4 + 16 + 4 + 4)


def test_version(T):
    assert T.lib().themis_version() >= 100


def _good(T):
    return T.make_problem(64, 3, 8, [1, 2, 4, 8, 16], 8, 1000, 300_000)


def test_check_problem_accepts_good(T):
    p = _good(T)
    assert T.check_problem(p) == T.OK
    assert T.workspace_bytes(p) > 64 * 3 * 40 * 8


@pytest.mark.parametrize("mutate,code", [
    (lambda p: setattr(p, "n_inst", 0), "ERR_SHAPE"),
    (lambda p: setattr(p, "n_stage", 0), "ERR_SHAPE"),
    (lambda p: setattr(p, "c_max", 0), "ERR_SHAPE"),
    (lambda p: setattr(p, "tick_us", 0), "ERR_SHAPE"),
    (lambda p: setattr(p, "slo_max_us", -1), "ERR_SHAPE"),
    (lambda p: setattr(p, "coef_shared", 2), "ERR_SHAPE"),
    (lambda p: p.reserved.__setitem__(0, 7), "ERR_SHAPE"),
    (lambda p: setattr(p, "prune", 4), "ERR_SHAPE"),
    (lambda p: setattr(p, "prune", -1), "ERR_SHAPE"),
    (lambda p: setattr(p, "queue_model", 3), "ERR_SHAPE"),
    (lambda p: setattr(p, "queue_model", -1), "ERR_SHAPE"),
    (lambda p: setattr(p, "profile_form", 2), "ERR_SHAPE"),
    (lambda p: setattr(p, "n_batch", 0), "ERR_BATCH"),
    (lambda p: setattr(p, "n_batch", 17), "ERR_BATCH"),
    (lambda p: p.batch_sizes.__setitem__(2, 2), "ERR_BATCH"),       # not increasing
    (lambda p: p.batch_sizes.__setitem__(4, 2048), "ERR_BATCH"),    # too large
    (lambda p: p.batch_sizes.__setitem__(0, 0), "ERR_BATCH"),
    (lambda p: setattr(p, "r_max", 2000), "ERR_RANGE"),             # 3*2000*8 > 32767
    (lambda p: setattr(p, "tick_us", 1), "ERR_RANGE"),              # 300000 ticks
    (lambda p: setattr(p, "n_inst", 2**31 // 100), "ERR_SHAPE"),    # flat index overflow
])
def test_check_problem_rejects(T, mutate, code):
    p = _good(T)
    mutate(p)
    assert T.check_problem(p) == getattr(T, code)
    assert T.workspace_bytes(p) == 0


def test_null_problem(T):
    assert T.lib().themis_check_problem(None) == T.ERR_NULL
    assert T.lib().themis_workspace_bytes(None) == 0


def test_limits_are_inclusive(T):
    p = T.make_problem(1, 1, 1, [1], 32767, 1, 32767)
    assert T.check_problem(p) == T.OK
    p = T.make_problem(1, 1, 1, [1], 32767, 1, 32768)
    assert T.check_problem(p) == T.ERR_RANGE
    p = T.make_problem(1, 2, 1, [1], 32767, 1, 100)
    assert T.check_problem(p) == T.ERR_RANGE


def test_workspace_grows_with_problem(T):
    a = T.workspace_bytes(T.make_problem(64, 3, 8, [1, 2], 8, 1000, 300_000))
    b = T.workspace_bytes(T.make_problem(128, 3, 8, [1, 2], 8, 1000, 300_000))
    c = T.workspace_bytes(T.make_problem(64, 3, 8, [1, 2], 8, 500, 300_000))
    assert b > a and c > a and a % 256 == 0


def test_fallback_workspace_is_larger(T):
    p = T.make_problem(100, 3, 8, [1, 2], 8, 1000, 300_000)
    base, fb = T.workspace_bytes(p), T.fallback_workspace_bytes(p)
    assert fb % 256 == 0 and fb >= base + (3 + 3) * 100 * 4
    bad = T.make_problem(1, 2, 1, [1], 32767, 1, 100)
    assert T.fallback_workspace_bytes(bad) == 0


def test_fallback_argument_checks_on_host(T):
    """Null pointers and a short or misaligned workspace are refused before
    anything is launched (so this runs without a GPU)."""
    import ctypes
    p = T.make_problem(4, 2, 2, [1, 2], 4, 1000, 100_000)
    f = T.lib().themis_solve_vertical_fallback
    one = ctypes.c_void_p(256)  # never dereferenced: the call fails first
    args = [one] * 4
    outs = [one] * 9
    assert f(ctypes.byref(p), None, one, one, one, *outs, one, 1 << 30, None) == T.ERR_NULL
    assert f(ctypes.byref(p), *args, *([one] * 8 + [None]), one, 1 << 30, None) == T.ERR_NULL
    assert f(ctypes.byref(p), *args, *outs, one, 256, None) == T.ERR_WORKSPACE
    assert f(ctypes.byref(p), *args, *outs, ctypes.c_void_p(264), 1 << 30, None) == \
        T.ERR_WORKSPACE
    assert f(ctypes.byref(p), *args, *outs, None, 1 << 30, None) == T.ERR_WORKSPACE
    bad = T.make_problem(4, 2, 2, [2, 1], 4, 1000, 100_000)
    assert f(ctypes.byref(bad), *args, *outs, one, 1 << 30, None) not in (T.OK, T.ERR_WORKSPACE)


def test_stability_workspace_and_argument_checks(T):
    import ctypes
    p = T.make_problem(100, 3, 8, [1, 2], 8, 1000, 300_000)
    assert T.stability_workspace_bytes(p) >= T.workspace_bytes(p) + (3 + 9) * 100 * 4
    f = T.lib().themis_check_stability
    one = ctypes.c_void_p(256)
    assert f(ctypes.byref(p), one, one, None, one, None, *([one] * 5), one, 1 << 30, None) == \
        T.ERR_NULL
    assert f(ctypes.byref(p), one, one, one, one, None, *([one] * 5), one, 256, None) == \
        T.ERR_WORKSPACE


def test_distinct_solve_workspace_and_argument_checks(T):
    import ctypes
    p = T.make_problem(100, 3, 8, [1, 2], 8, 1000, 300_000)
    # two words per instance and a table of 256 slots (the least power of two >= 2 N)
    assert T.memo_workspace_bytes(p) >= T.workspace_bytes(p) + 2 * 100 * 4 + 256 * 4
    big = T.make_problem(70_000, 3, 8, [1, 2], 8, 1000, 300_000)
    assert T.memo_workspace_bytes(big) >= T.workspace_bytes(big) + 2 * 70_000 * 4 + (1 << 18) * 4
    f = T.lib().themis_solve_distinct
    one = ctypes.c_void_p(256)
    # replica counts are optional (absent = joint); everything else is required
    assert f(ctypes.byref(p), one, one, one, None, one, one, one, one, one, 256, None) == \
        T.ERR_WORKSPACE
    assert f(ctypes.byref(p), one, None, one, None, one, one, one, one, one, 1 << 30, None) == \
        T.ERR_NULL
    assert f(ctypes.byref(p), one, one, one, None, one, one, one, None, one, 1 << 30, None) == \
        T.ERR_NULL
    assert f(ctypes.byref(p), one, one, one, None, one, one, one, one, ctypes.c_void_p(260),
             1 << 30, None) == T.ERR_WORKSPACE


def test_model_options_accepted(T):
    for qm in (T.QUEUE_PER_REPLICA, T.QUEUE_SHARED, T.QUEUE_WORST_CASE):
        for pf in (T.PROFILE_5, T.PROFILE_EQ1):
            for pr in (T.PRUNE_NONE, T.PRUNE_DOMINATED, T.PRUNE_STEPS,
                       T.PRUNE_DOMINATED | T.PRUNE_STEPS):
                p = T.make_problem(64, 3, 8, [1, 2], 8, 1000, 300_000, queue_model=qm,
                                   profile_form=pf, prune=pr)
                assert T.check_problem(p) == T.OK


def test_missing_library_fails_loudly(monkeypatch):
    """No CPU fallback: without the built HIP library the binding raises."""
    from paper_2407_14843_amd import themis
    monkeypatch.setattr(themis, "_lib", None)
    monkeypatch.setattr(themis, "LIB_PATH", "/nonexistent/libthemis_hip.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        themis.lib()
    with pytest.raises(RuntimeError):
        themis.check_problem(themis.make_problem(1, 1, 1, [1], 1, 1, 1))
