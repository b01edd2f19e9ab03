"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and turns bad arguments into status codes before any
HIP call."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "cdsgd.h"), os.path.join(ROOT, "include", "cdsgd_cost_model.h")]


@pytest.fixture(scope="module")
def L():
    from paper_2106_10796_amd import binding, build
    build.ensure_built()
    return binding.lib()


def declared_functions():
    src = "\n".join(open(h).read() for h in HEADERS)
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(cdsgd_[a-z_]+)\s*\(", src)))


def test_header_declares_the_named_entry_points():
    names = declared_functions()
    for must in ("cdsgd_quantize_pack", "cdsgd_decode_sum", "cdsgd_update", "cdsgd_step_fused",
                 "cdsgd_plan_create", "cdsgd_plan_destroy", "cdsgd_packed_words", "cdsgd_status_string",
                 "cdsgd_plan_bind_full_grads", "cdsgd_step_warmup", "cdsgd_trainer_create",
                 "cdsgd_trainer_step", "cdsgd_trainer_iteration", "cdsgd_trainer_destroy",
                 "cdsgd_step_local", "cdsgd_step_global", "cdsgd_cost_iteration", "cdsgd_cost_period_mean",
                 "cdsgd_plan_create_typed", "cdsgd_plan_set_thresholds", "cdsgd_plan_set_max_workgroups",
                 "cdsgd_step_fused_static", "cdsgd_build_id", "cdsgd_sparse_encode", "cdsgd_decode_sum_sparse",
                 "cdsgd_sparse_words", "cdsgd_sparse_segments", "cdsgd_plan_set_peer_format", "cdsgd_probe_streams",
                 "cdsgd_step_fused_range", "cdsgd_step_local_range", "cdsgd_step_global_range"):
        assert must in names


def test_binding_constants_match_the_header():
    from paper_2106_10796_amd import binding
    src = "\n".join(open(h).read() for h in HEADERS)
    defines = {k: int(v) for k, v in re.findall(r"#define\s+(CDSGD_[A-Z_]+)\s+(\d+)", src)}
    assert defines["CDSGD_MAX_WORKERS"] == binding.MAX_WORKERS
    assert defines["CDSGD_STATIC_MAX_TENSORS"] == binding.STATIC_MAX_TENSORS
    assert defines["CDSGD_STATIC_MAX_CHUNKS"] == binding.STATIC_MAX_CHUNKS
    assert defines["CDSGD_STATIC_CHUNK_ELEMS"] == binding.STATIC_CHUNK_ELEMS
    enums = dict(re.findall(r"(CDSGD_[A-Z0-9_]+)\s*=\s*(\d+)", src))
    for name, val in (("CDSGD_OK", binding.OK), ("CDSGD_ERR_NULL", binding.ERR_NULL), ("CDSGD_ERR_SIZE", binding.ERR_SIZE),
                      ("CDSGD_ERR_PARAM", binding.ERR_PARAM), ("CDSGD_ERR_ALIGN", binding.ERR_ALIGN),
                      ("CDSGD_ERR_WORKERS", binding.ERR_WORKERS), ("CDSGD_ERR_DEVICE", binding.ERR_DEVICE),
                      ("CDSGD_ERR_ALIAS", binding.ERR_ALIAS), ("CDSGD_PEERS_PACKED", binding.PEERS_PACKED),
                      ("CDSGD_PEERS_SPARSE", binding.PEERS_SPARSE), ("CDSGD_PASS_WARMUP", binding.PASS_WARMUP),
                      ("CDSGD_PASS_COMPRESSED", binding.PASS_COMPRESSED), ("CDSGD_PASS_CORRECTION", binding.PASS_CORRECTION),
                      ("CDSGD_GRAD_BF16", 1), ("CDSGD_GRAD_F16", 2)):
        assert int(enums[name]) == val, name


def test_library_exports_every_declared_symbol(L):
    for name in declared_functions():
        assert hasattr(L, name), name


def test_library_matches_the_tree(L, monkeypatch):
    """The library carries the identity of the sources, headers and flags it was built from;
    ensure_built() rebuilds exactly when that differs from what the tree holds now."""
    from paper_2106_10796_amd import build
    now = build.source_id()
    assert re.fullmatch(r"[0-9a-f]{16}", now)
    assert build.built_id() == now == L.cdsgd_build_id().decode()
    assert build.source_id(("-DSOMETHING",)) != now               # flags are part of the identity
    calls = []
    monkeypatch.setattr(build, "build", lambda *a, **k: calls.append(1) or build.LIB)
    build.ensure_built()
    assert calls == []                                            # current: loaded as it is
    monkeypatch.setattr(build, "source_id", lambda extra_flags=(): "f" * 16)
    build.ensure_built()
    assert calls == [1]                                           # stale: rebuilt
    assert build.built_id(os.path.join(ROOT, "include", "cdsgd.h")) is None


def test_packed_words(L):
    for n, w in ((1, 1), (15, 1), (16, 1), (17, 2), (32, 2), (33, 3), (65536, 4096), (1 << 30, 1 << 26)):
        assert L.cdsgd_packed_words(n) == w


def test_sparse_sizes_and_argument_errors(L):
    from paper_2106_10796_amd.binding import ERR_ALIAS, ERR_ALIGN, ERR_NULL, ERR_PARAM, ERR_SIZE, ERR_WORKERS
    for n, segs in ((1, 1), (4096, 1), (4097, 2), (8192, 2), (8193, 3), (1 << 30, 1 << 18)):
        assert L.cdsgd_sparse_segments(n) == segs and L.cdsgd_sparse_words(n) == 264 * segs
    e = L.cdsgd_sparse_encode
    assert e(None, 16, A, None, None) == ERR_NULL
    assert e(A, 16, None, None, None) == ERR_NULL
    assert e(A, 0, A + 0x10000, None, None) == ERR_SIZE
    assert e(A + 2, 16, A + 0x10000, None, None) == ERR_ALIGN
    assert e(A, 16, A, None, None) == ERR_ALIAS
    assert e(A, 4096 * 4, A + 1024, None, None) == ERR_ALIAS        # sparse buffer inside the packed stream
    d = L.cdsgd_decode_sum_sparse
    two = (ctypes.c_void_p * 2)(A, A + 0x10000)
    assert d(None, 2, A + 0x20000, 16, 0.5, None) == ERR_NULL
    assert d(two, 2, None, 16, 0.5, None) == ERR_NULL
    assert d(two, 2, A + 0x20000, 0, 0.5, None) == ERR_SIZE
    assert d(two, 2, A + 0x20000, 16, 0.0, None) == ERR_PARAM
    assert d(two, 65, A + 0x20000, 16, 0.5, None) == ERR_WORKERS
    assert d(two, 2, A + 0x20004, 16, 0.5, None) == ERR_ALIGN
    assert d(two, 2, A + 64, 16, 0.5, None) == ERR_ALIAS
    assert L.cdsgd_plan_set_peer_format(None, 0) == ERR_NULL


def test_probe_streams_argument_errors(L):
    from paper_2106_10796_amd.binding import ERR_ALIAS, ERR_ALIGN, ERR_NULL, ERR_PARAM, ERR_SIZE
    f = L.cdsgd_probe_streams
    r = (ctypes.c_void_p * 3)(A, A + 0x100000, A + 0x200000)
    w = (ctypes.c_void_p * 3)(A + 0x300000, A + 0x400000, A + 0x500000)
    S = A + 0x600000
    assert f(r, 18, w, 1, 1024, S, 0, None) == ERR_PARAM
    assert f(r, 1, w, 4, 1024, S, 0, None) == ERR_PARAM
    assert f(r, 1, w, 1, 1024, S, 65537, None) == ERR_PARAM
    assert f(r, 0, w, 0, 1024, S, 0, None) == ERR_PARAM
    assert f(None, 1, w, 1, 1024, S, 0, None) == ERR_NULL
    assert f(r, 2, w, 0, 1024, None, 0, None) == ERR_NULL            # read-only needs the sink
    assert f(r, 1, w, 1, 1000, S, 0, None) == ERR_SIZE              # not a multiple of 256
    assert f(r, 1, w, 1, 0, S, 0, None) == ERR_SIZE
    odd = (ctypes.c_void_p * 1)(A + 4)
    assert f(odd, 1, w, 1, 1024, S, 0, None) == ERR_ALIGN
    assert f(r, 1, r, 1, 1024, S, 0, None) == ERR_ALIAS             # writing what is read
    assert f(r, 1, (ctypes.c_void_p * 2)(A + 0x300000, A + 0x300010), 2, 1024, S, 0, None) == ERR_ALIAS


def test_status_strings(L):
    seen = set()
    for s in range(8):
        msg = L.cdsgd_status_string(s)
        assert msg and msg not in seen
        seen.add(msg)
    assert L.cdsgd_status_string(99) == b"unknown status"


A = 0x1000  # a fake, well aligned, non-NULL device address; never dereferenced on these paths


def test_quantize_pack_argument_errors(L):
    from paper_2106_10796_amd.binding import ERR_ALIGN, ERR_NULL, ERR_PARAM, ERR_SIZE
    q = L.cdsgd_quantize_pack
    assert q(None, A, A, 16, 0.5, None) == ERR_NULL
    assert q(A, None, A, 16, 0.5, None) == ERR_NULL
    assert q(A, A, None, 16, 0.5, None) == ERR_NULL
    assert q(A, A, A, 0, 0.5, None) == ERR_SIZE
    for t in (0.0, -0.5, float("nan"), float("inf")):
        assert q(A, A, A, 16, t, None) == ERR_PARAM
    assert q(A + 4, A, A, 16, 0.5, None) == ERR_ALIGN
    assert q(A, A + 8, A, 16, 0.5, None) == ERR_ALIGN
    assert q(A, A, A + 2, 16, 0.5, None) == ERR_ALIGN


def test_decode_sum_argument_errors(L):
    from paper_2106_10796_amd.binding import ERR_ALIGN, ERR_NULL, ERR_PARAM, ERR_SIZE, ERR_WORKERS, MAX_WORKERS
    d = L.cdsgd_decode_sum
    two = (ctypes.c_void_p * 2)(A, A)
    assert d(None, 2, A, 16, 0.5, None) == ERR_NULL
    assert d(two, 2, None, 16, 0.5, None) == ERR_NULL
    assert d(two, 2, A, 0, 0.5, None) == ERR_SIZE
    assert d(two, 2, A, 16, -1.0, None) == ERR_PARAM
    assert d(two, 0, A, 16, 0.5, None) == ERR_WORKERS
    many = (ctypes.c_void_p * (MAX_WORKERS + 1))(*([A] * (MAX_WORKERS + 1)))
    assert d(many, MAX_WORKERS + 1, A, 16, 0.5, None) == ERR_WORKERS
    hole = (ctypes.c_void_p * 2)(A, None)
    assert d(hole, 2, A, 16, 0.5, None) == ERR_NULL
    assert d(two, 2, A + 4, 16, 0.5, None) == ERR_ALIGN
    odd = (ctypes.c_void_p * 2)(A, A + 1)
    assert d(odd, 2, A, 16, 0.5, None) == ERR_ALIGN


def test_update_argument_errors(L):
    from paper_2106_10796_amd.binding import ERR_ALIGN, ERR_NULL, ERR_PARAM, ERR_SIZE, ERR_WORKERS
    u = L.cdsgd_update
    assert u(None, A, A, A, 16, 0.1, 0.1, 2, None) == ERR_NULL
    assert u(A, A, None, A, 16, 0.1, 0.1, 2, None) == ERR_NULL   # local half given without gradient
    assert u(A, None, A, A, 16, 0.1, 0.1, 2, None) == ERR_NULL
    assert u(A, None, None, None, 16, 0.1, 0.1, 2, None) == ERR_NULL  # nothing to do
    assert u(A, A, A, A, 0, 0.1, 0.1, 2, None) == ERR_SIZE
    assert u(A, A, A, A, 16, float("nan"), 0.1, 2, None) == ERR_PARAM
    assert u(A, A, A, A, 16, 0.1, float("inf"), 2, None) == ERR_PARAM
    assert u(A, A, A, A, 16, 0.1, 0.1, 0, None) == ERR_WORKERS
    assert u(A, A, A, A, 16, 0.1, 0.1, 65, None) == ERR_WORKERS
    assert u(A, A + 4, A, A, 16, 0.1, 0.1, 2, None) == ERR_ALIGN


def _tensor(L, **kw):
    from paper_2106_10796_amd.binding import cdsgd_tensor
    t = cdsgd_tensor()
    # distinct fake addresses 64 KiB apart: the buffers of a tensor must not overlap
    t.w_global, t.w_local, t.residual, t.grad, t.packed_self, t.agg_full = (A + 0x10000 * i for i in range(6))
    t.n = 64
    for k, v in kw.items():
        setattr(t, k, v)
    return t


def test_plan_and_step_argument_errors(L):
    from paper_2106_10796_amd.binding import (ERR_ALIGN, ERR_NULL, ERR_PARAM, ERR_SIZE, ERR_WORKERS, OK,
                                              cdsgd_tensor)
    create = L.cdsgd_plan_create
    out = ctypes.c_void_p()
    arr = (cdsgd_tensor * 1)(_tensor(L))
    row = (ctypes.c_void_p * 1)(A)
    rows = (ctypes.POINTER(ctypes.c_void_p) * 2)(ctypes.POINTER(ctypes.c_void_p)(),
                                                 ctypes.cast(row, ctypes.POINTER(ctypes.c_void_p)))
    assert create(arr, 1, rows, 2, 0, None) == ERR_NULL
    assert create(None, 1, rows, 2, 0, ctypes.byref(out)) == ERR_NULL
    assert create(arr, 0, rows, 2, 0, ctypes.byref(out)) == ERR_SIZE
    assert create(arr, 1, rows, 0, 0, ctypes.byref(out)) == ERR_WORKERS
    assert create(arr, 1, rows, 2, 2, ctypes.byref(out)) == ERR_WORKERS
    assert create(arr, 1, rows, 2, -1, ctypes.byref(out)) == ERR_WORKERS
    assert create(arr, 1, None, 2, 0, ctypes.byref(out)) == ERR_NULL        # peers needed for N > 1
    assert create(arr, 1, rows, 2, 1, ctypes.byref(out)) == ERR_NULL        # row 0 is a peer now and is NULL
    for fld in ("w_global", "w_local", "residual", "grad", "packed_self"):
        bad = (cdsgd_tensor * 1)(_tensor(L, **{fld: None}))
        assert create(bad, 1, rows, 2, 0, ctypes.byref(out)) == ERR_NULL
    assert create((cdsgd_tensor * 1)(_tensor(L, n=0)), 1, rows, 2, 0, ctypes.byref(out)) == ERR_SIZE
    assert create((cdsgd_tensor * 1)(_tensor(L, grad=A + 4)), 1, rows, 2, 0, ctypes.byref(out)) == ERR_ALIGN
    badrow = (ctypes.c_void_p * 1)(A + 2)
    badrows = (ctypes.POINTER(ctypes.c_void_p) * 2)(ctypes.POINTER(ctypes.c_void_p)(),
                                                    ctypes.cast(badrow, ctypes.POINTER(ctypes.c_void_p)))
    assert create(arr, 1, badrows, 2, 0, ctypes.byref(out)) == ERR_ALIGN
    assert out.value is None
    step = L.cdsgd_step_fused
    assert step(None, 1, 4, 0.5, 0.1, 0.1, None) == ERR_NULL
    assert L.cdsgd_plan_set_max_workgroups(None, 4) == ERR_NULL
    assert L.cdsgd_step_fused_range(None, 0, 1, 1, 4, 0.5, 0.1, 0.1, None) == ERR_NULL
    assert L.cdsgd_step_local_range(None, 0, 1, 0.1, None) == ERR_NULL
    assert L.cdsgd_step_global_range(None, 0, 1, 1, 4, 0.5, 0.1, None) == ERR_NULL
    assert L.cdsgd_plan_destroy(None) == OK
    fake = ctypes.c_void_p(A)  # parameter checks come before the plan is looked at
    assert step(fake, 1, 0, 0.5, 0.1, 0.1, None) == ERR_PARAM
    assert step(fake, -1, 4, 0.5, 0.1, 0.1, None) == ERR_PARAM
    assert step(fake, 1, 4, 0.0, 0.1, 0.1, None) == ERR_PARAM
    assert step(fake, 1, 4, 0.5, float("nan"), 0.1, None) == ERR_PARAM


def test_step_fused_static_argument_errors(L):
    """The entry point that allocates nothing checks like plan creation plus a step, and refuses
    layer lists beyond its static tables, all on the host (fake addresses are never dereferenced)."""
    from paper_2106_10796_amd.binding import (ERR_ALIGN, ERR_NULL, ERR_PARAM, ERR_SIZE, ERR_WORKERS,
                                              STATIC_CHUNK_ELEMS, STATIC_MAX_CHUNKS, STATIC_MAX_TENSORS,
                                              cdsgd_tensor)
    f = L.cdsgd_step_fused_static
    arr = (cdsgd_tensor * 1)(_tensor(L))
    row = (ctypes.c_void_p * 1)(A + 0x70000)
    rows = (ctypes.POINTER(ctypes.c_void_p) * 2)(ctypes.POINTER(ctypes.c_void_p)(),
                                                 ctypes.cast(row, ctypes.POINTER(ctypes.c_void_p)))
    assert f(None, 1, rows, 2, 0, 0, 1, 4, 0.5, 0.1, 0.1, None) == ERR_NULL
    assert f(arr, 0, rows, 2, 0, 0, 1, 4, 0.5, 0.1, 0.1, None) == ERR_SIZE
    assert f(arr, 1, rows, 65, 0, 0, 1, 4, 0.5, 0.1, 0.1, None) == ERR_WORKERS
    assert f(arr, 1, None, 2, 0, 0, 1, 4, 0.5, 0.1, 0.1, None) == ERR_NULL
    assert f(arr, 1, rows, 2, 0, 7, 1, 4, 0.5, 0.1, 0.1, None) == ERR_PARAM       # gradient type
    assert f(arr, 1, rows, 2, 0, 0, 1, 0, 0.5, 0.1, 0.1, None) == ERR_PARAM       # k
    assert f(arr, 1, rows, 2, 0, 0, -1, 4, 0.5, 0.1, 0.1, None) == ERR_PARAM      # step
    assert f(arr, 1, rows, 2, 0, 0, 1, 4, -0.5, 0.1, 0.1, None) == ERR_PARAM      # threshold
    assert f(arr, 1, rows, 2, 0, 0, 1, 4, 0.5, float("inf"), 0.1, None) == ERR_PARAM
    assert f((cdsgd_tensor * 1)(_tensor(L, w_local=A + 0x10004)), 1, rows, 2, 0, 0, 1, 4, 0.5, 0.1, 0.1, None) == ERR_ALIGN
    assert f((cdsgd_tensor * 1)(_tensor(L, agg_full=None)), 1, rows, 2, 0, 0, 0, 4, 0.5, 0.1, 0.1, None) == ERR_NULL
    # too many tensors
    T = STATIC_MAX_TENSORS + 1
    big = (cdsgd_tensor * T)(*[_tensor(L) for _ in range(T)])
    bigrow = (ctypes.c_void_p * T)(*([A + 0x70000] * T))
    bigrows = (ctypes.POINTER(ctypes.c_void_p) * 2)(ctypes.POINTER(ctypes.c_void_p)(),
                                                    ctypes.cast(bigrow, ctypes.POINTER(ctypes.c_void_p)))
    assert f(big, T, bigrows, 2, 0, 0, 1, 4, 0.5, 0.1, 0.1, None) == ERR_SIZE
    # too many chunks: one tensor one chunk beyond the table (buffers spaced so that nothing overlaps)
    n = STATIC_MAX_CHUNKS * STATIC_CHUNK_ELEMS + 1
    t = cdsgd_tensor()
    step_b = 1 << 34
    t.w_global, t.w_local, t.residual, t.grad, t.packed_self, t.agg_full = (A + step_b * i for i in range(6))
    t.n = n
    farrow = (ctypes.c_void_p * 1)(A + step_b * 7)
    farrows = (ctypes.POINTER(ctypes.c_void_p) * 2)(ctypes.POINTER(ctypes.c_void_p)(),
                                                    ctypes.cast(farrow, ctypes.POINTER(ctypes.c_void_p)))
    assert f((cdsgd_tensor * 1)(t), 1, farrows, 2, 0, 0, 1, 4, 0.5, 0.1, 0.1, None) == ERR_SIZE


def test_aliasing_is_refused(L):
    """An output that overlaps an input (or another output) of the same tensor would make the
    result depend on the launch order; the host checks refuse it."""
    from paper_2106_10796_amd.binding import ERR_ALIAS, cdsgd_tensor
    B1, B2, B3, B4, B5, B6 = (0x100000 * i for i in range(1, 7))
    n = 1000
    assert L.cdsgd_quantize_pack(B1, B1, B3, n, 0.5, None) == ERR_ALIAS
    assert L.cdsgd_quantize_pack(B1, B1 + 4 * n - 16, B3, n, 0.5, None) == ERR_ALIAS      # partial overlap
    assert L.cdsgd_update(B1, B1, B2, B3, n, 0.1, 0.1, 2, None) == ERR_ALIAS              # w_local on w_global
    assert L.cdsgd_update(B1, B2, B2, B3, n, 0.1, 0.1, 2, None) == ERR_ALIAS              # w_local on grad
    assert L.cdsgd_update(B1, B2, B3, B1 + 16, n, 0.1, 0.1, 2, None) == ERR_ALIAS         # agg on w_global
    out = ctypes.c_void_p()
    row = (ctypes.c_void_p * 1)(B6)
    rows = (ctypes.POINTER(ctypes.c_void_p) * 2)(ctypes.POINTER(ctypes.c_void_p)(),
                                                 ctypes.cast(row, ctypes.POINTER(ctypes.c_void_p)))
    def tensor(**kw):
        t = cdsgd_tensor()
        t.w_global, t.w_local, t.residual, t.grad, t.packed_self, t.agg_full, t.n = B1, B2, B3, B4, B5, None, n
        for k, v in kw.items():
            setattr(t, k, v)
        return (cdsgd_tensor * 1)(t)
    for bad in (dict(w_local=B1), dict(residual=B4), dict(grad=B1 + 64), dict(w_local=B3), dict(agg_full=B2),
                dict(packed_self=B3 + 4 * n - 4), dict(packed_self=B1), dict(packed_self=B4 + 16),
                dict(packed_self=B6)):                      # own codes on a peer's stream
        assert L.cdsgd_plan_create(tensor(**bad), 1, rows, 2, 0, ctypes.byref(out)) == ERR_ALIAS
    row_on_w = (ctypes.c_void_p * 1)(B1 + 32)                # a peer's stream inside w_global
    rows_on_w = (ctypes.POINTER(ctypes.c_void_p) * 2)(ctypes.POINTER(ctypes.c_void_p)(),
                                                      ctypes.cast(row_on_w, ctypes.POINTER(ctypes.c_void_p)))
    assert L.cdsgd_plan_create(tensor(), 1, rows_on_w, 2, 0, ctypes.byref(out)) == ERR_ALIAS
    # the single-tensor calls: packed on grad / residual, agg on a packed stream
    assert L.cdsgd_quantize_pack(B1, B2, B1 + 8, n, 0.5, None) == ERR_ALIAS
    assert L.cdsgd_quantize_pack(B1, B2, B2 + 4 * n - 4, n, 0.5, None) == ERR_ALIAS
    two = (ctypes.c_void_p * 2)(B1, B2 + 4)
    assert L.cdsgd_decode_sum(two, 2, B2, n, 0.5, None) == ERR_ALIAS
    # a 16-bit gradient buffer is half as long: a residual right behind it is fine for bf16, not for fp32
    tight = dict(grad=B4, residual=B4 + 2 * n + 48)       # 2n bytes of bf16, next 16-byte boundary
    assert L.cdsgd_plan_create(tensor(**tight), 1, rows, 2, 0, ctypes.byref(out)) == ERR_ALIAS
    assert L.cdsgd_plan_create_typed(tensor(**dict(tight, residual=B4 + 2 * n - 16)), 1, rows, 2, 0, 1,
                                     ctypes.byref(out)) == ERR_ALIAS
    assert out.value is None


def test_warmup_and_trainer_argument_errors(L):
    from paper_2106_10796_amd.binding import ERR_NULL, ERR_PARAM, OK
    fake = ctypes.c_void_p(A)   # never dereferenced: parameter checks come first
    w = L.cdsgd_step_warmup
    assert w(None, 0, 2, 0.1, 0.1, None) == ERR_NULL
    assert w(fake, -1, 2, 0.1, 0.1, None) == ERR_PARAM
    assert w(fake, 3, 2, 0.1, 0.1, None) == ERR_PARAM
    assert w(fake, 0, -1, 0.1, 0.1, None) == ERR_PARAM
    assert w(fake, 0, 2, float("nan"), 0.1, None) == ERR_PARAM
    out = ctypes.c_void_p()
    c = L.cdsgd_trainer_create
    assert c(None, 2, 4, 0.5, 0.1, 0.1, ctypes.byref(out)) == ERR_NULL
    assert c(fake, 2, 4, 0.5, 0.1, 0.1, None) == ERR_NULL
    assert c(fake, -1, 4, 0.5, 0.1, 0.1, ctypes.byref(out)) == ERR_PARAM
    assert c(fake, 2, 0, 0.5, 0.1, 0.1, ctypes.byref(out)) == ERR_PARAM
    assert c(fake, 2, 4, -0.5, 0.1, 0.1, ctypes.byref(out)) == ERR_PARAM
    assert c(fake, 2, 4, 0.5, float("inf"), 0.1, ctypes.byref(out)) == ERR_PARAM
    assert out.value is None
    assert L.cdsgd_trainer_step(None, None, None) == ERR_NULL
    assert L.cdsgd_trainer_iteration(None) == -1
    assert L.cdsgd_trainer_destroy(None) == OK
    assert L.cdsgd_plan_bind_full_grads(None, None) == ERR_NULL
    arr = (__import__("paper_2106_10796_amd.binding", fromlist=["x"]).cdsgd_tensor * 1)(_tensor(L))
    assert L.cdsgd_plan_create_typed(arr, 1, None, 1, 0, 7, ctypes.byref(out)) == ERR_PARAM   # unknown dtype
    assert L.cdsgd_plan_set_thresholds(None, None) == ERR_NULL
    assert L.cdsgd_step_local(None, 0.1, None) == ERR_NULL
    assert L.cdsgd_step_local(fake, float("nan"), None) == ERR_PARAM
    assert L.cdsgd_step_global(None, 1, 4, 0.5, 0.1, None) == ERR_NULL
    assert L.cdsgd_step_global(fake, 1, 0, 0.5, 0.1, None) == ERR_PARAM
    assert L.cdsgd_step_global(fake, 1, 4, 0.5, float("inf"), None) == ERR_PARAM
    # a trainer is host state only: create / query / destroy work without a GPU
    assert c(fake, 2, 4, 0.5, 0.1, 0.1, ctypes.byref(out)) == OK
    assert L.cdsgd_trainer_iteration(out) == 0
    assert L.cdsgd_trainer_destroy(out) == OK


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2106_10796_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.lib()


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2106_10796_amd")
    pat = re.compile(r"^\s*(from\s+oracle|import\s+oracle|from\s+\.+\s*oracle)|liboracle|cdsgd_oracle", re.M)
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                assert not pat.search(open(os.path.join(dirpath, f)).read()), f


def test_native_client_builds_and_needs_a_gpu():
    """The C++ client of the ABI (tests/native/abi_client.cpp) compiles against the header and links the
    library with the host compiler alone; without a GPU it stops at its first HIP call, before any call
    into the library."""
    import importlib.util
    import subprocess
    spec = importlib.util.spec_from_file_location("native_client_build", os.path.join(ROOT, "tests", "native", "build.py"))
    native = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(native)
    exe = native.ensure_built()
    assert os.access(exe, os.X_OK)
    import torch
    if torch.cuda.is_available():
        return
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=60)
    assert r.returncode == 2 and "abi client ok" not in r.stdout
