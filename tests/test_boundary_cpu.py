"""CPU-only checks of the boundary: the C-ABI library loads, exports every symbol the
header declares, the binding prototypes cover them, argument validation that needs no
GPU works, and the chunking rule covers every element exactly once."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "selsync.h")


@pytest.fixture(scope="module")
def B():
    from paper_2307_07950_amd import build
    if build.needs_build():
        build.build()
    from paper_2307_07950_amd import binding
    return binding


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(selsync_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol(B):
    names = declared_functions()
    assert len(names) >= 18
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), "libselsync.so does not export %s" % n


def test_binding_prototypes_match_header(B):
    assert sorted(B.PROTOTYPES) == declared_functions()
    for n in B.PROTOTYPES:
        assert callable(getattr(B, n))


def test_struct_layouts_are_plain_c(B):
    assert ctypes.sizeof(B.selsync_tensor) == 24
    assert ctypes.sizeof(B.selsync_tensor_list) == 16
    assert ctypes.sizeof(B.selsync_config) == 24
    assert ctypes.sizeof(B.selsync_sgd) == 24
    assert ctypes.sizeof(B.selsync_stats) == 40
    assert ctypes.sizeof(B.selsync_tuning) == 16


def test_status_strings(B):
    assert B.selsync_status_string(0) == b"SELSYNC_OK"
    assert B.selsync_status_string(B.SELSYNC_ERR_DTYPE) == b"SELSYNC_ERR_DTYPE"
    assert B.selsync_status_string(B.SELSYNC_WARN_NONFINITE) == b"SELSYNC_WARN_NONFINITE"
    assert B.selsync_status_string(12345) == b"SELSYNC_UNKNOWN_STATUS"
    assert B.selsync_last_error(None) == b"context is NULL"


@pytest.mark.parametrize("cfg", [
    dict(num_workers=0, window=25, delta=0.3, alpha=-1.0),
    dict(num_workers=-3, window=25, delta=0.3, alpha=-1.0),
    dict(num_workers=4, window=-1, delta=0.3, alpha=-1.0),
    dict(num_workers=4, window=25, delta=-0.1, alpha=-1.0),
    dict(num_workers=4, window=25, delta=float("nan"), alpha=-1.0),
    dict(num_workers=4, window=25, delta=0.3, alpha=1.5),
    dict(num_workers=4, window=25, delta=0.3, alpha=float("nan")),
])
def test_create_rejects_bad_config_before_touching_the_gpu(B, cfg):
    c = B.selsync_config(**cfg)
    h = ctypes.c_void_p(1234)
    assert B.selsync_create(ctypes.byref(c), ctypes.byref(h)) == B.SELSYNC_ERR_INVALID_ARG
    assert h.value is None


def test_null_arguments_are_errors_not_crashes(B):
    h = ctypes.c_void_p()
    assert B.selsync_create(None, ctypes.byref(h)) == B.SELSYNC_ERR_INVALID_ARG
    c = B.selsync_config(4, 25, 0.3, -1.0)
    assert B.selsync_create(ctypes.byref(c), None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_destroy(None) == B.SELSYNC_OK
    assert B.selsync_plan_destroy(None) == B.SELSYNC_OK
    assert B.selsync_reset(None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_set_delta(None, 0.1, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_plan_info(None, None, None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_step(None, None, None, None, 0, None, None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_track_grad_change(None, None, 1.0, None, 0, None, None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_local_step(None, None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_aggregate_params(None, None, 0, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_get_stats(None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_read_decision(None, None, None, None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_profile_enable(None, 1, 10) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_step_bsp(None, None, None, None, 0, None, None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_step_bsp_adam(None, None, None, None, 0, None, None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_step_ga(None, None, None, None, 0, None, None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_ga_update_adam(None, None, None, 0, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_step_ga_adam(None, None, None, None, 0, None, None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    # the allocation-free entry point validates on the host before it touches the GPU
    assert B.selsync_grad_norm_sq_noalloc(None, 1, 1.0, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_status_string(B.SELSYNC_ERR_TOO_LARGE) == b"SELSYNC_ERR_TOO_LARGE"


def chunk_preview(B, numel, chunk, lead=None):
    arr = (ctypes.c_int64 * max(1, len(numel)))(*numel)
    la = None if lead is None else (ctypes.c_int32 * max(1, len(numel)))(*lead)
    n = ctypes.c_int32()
    assert B.selsync_chunk_table_preview(arr, la, len(numel), chunk, 0, None, None, None, ctypes.byref(n)) == 0
    cap = n.value
    t = (ctypes.c_int32 * max(1, cap))()
    o = (ctypes.c_int64 * max(1, cap))()
    c = (ctypes.c_int32 * max(1, cap))()
    assert B.selsync_chunk_table_preview(arr, la, len(numel), chunk, cap, t, o, c, ctypes.byref(n)) == 0
    assert n.value == cap
    return list(t)[:cap], list(o)[:cap], list(c)[:cap]


@pytest.mark.parametrize("chunk", [4096, 8192, 65536, 1 << 20])
def test_chunk_table_covers_every_element_exactly_once(B, chunk):
    from paper_2307_07950_amd import workloads as W
    for name in ("c1", "c2", "c3", "c4", "c5"):
        wl = W.get(name)
        numel = wl.numels + [0, 1, chunk, chunk + 1, chunk - 1]
        t, o, c = chunk_preview(B, numel, chunk)
        seen = {}
        for ti, oi, ci in zip(t, o, c):
            assert 0 < ci <= chunk
            assert oi % chunk == 0                         # chunk starts keep 16-byte alignment of the tensor base
            seen.setdefault(ti, []).append((oi, ci))
        for ti, n in enumerate(numel):
            pieces = sorted(seen.get(ti, []))
            pos = 0
            for oi, ci in pieces:
                assert oi == pos                           # no gap, no overlap
                pos += ci
            assert pos == n
            assert len(pieces) == -(-n // chunk)
            if n == 0:
                assert ti not in seen
        # table order is tensor-major, offsets ascending
        assert t == sorted(t)


@pytest.mark.parametrize("chunk", [256, 1024, 4096])
def test_chunk_pieces_are_cut_at_chunk_aligned_addresses(B, chunk):
    import numpy as np
    r = np.random.default_rng(chunk)
    numel = [0, 1, 3, chunk - 1, chunk, chunk + 1, 5 * chunk + 7, 100003, 2, chunk // 2]
    lead = [int(x) for x in r.integers(0, chunk, len(numel))]
    lead[4], lead[6] = 0, chunk - 1
    t, o, c = chunk_preview(B, numel, chunk, lead)
    seen = {}
    for ti, oi, ci in zip(t, o, c):
        assert 0 < ci <= chunk
        seen.setdefault(ti, []).append((oi, ci))
    for ti, n in enumerate(numel):
        pieces = sorted(seen.get(ti, []))
        pos = 0
        for idx, (oi, ci) in enumerate(pieces):
            assert oi == pos                               # no gap, no overlap
            if idx > 0:
                assert (lead[ti] + oi) % chunk == 0        # every later piece starts on an aligned address
            if idx < len(pieces) - 1:
                assert (lead[ti] + oi + ci) % chunk == 0   # and every piece but the last ends on one
            pos += ci
        assert pos == n
        assert len(pieces) == (-(-(lead[ti] + n) // chunk) if n else 0)
    assert t == sorted(t)
    # a lead outside [0, chunk) is refused
    n_out = ctypes.c_int32()
    arr = (ctypes.c_int64 * 1)(10)
    for bad in (-1, chunk):
        la = (ctypes.c_int32 * 1)(bad)
        assert B.selsync_chunk_table_preview(arr, la, 1, chunk, 0, None, None, None,
                                             ctypes.byref(n_out)) == B.SELSYNC_ERR_INVALID_ARG


def test_chunk_table_preview_rejects_bad_arguments(B):
    n = ctypes.c_int32()
    arr = (ctypes.c_int64 * 2)(10, -1)
    assert B.selsync_chunk_table_preview(arr, None, 2, 8192, 0, None, None, None, ctypes.byref(n)) == B.SELSYNC_ERR_INVALID_ARG
    arr = (ctypes.c_int64 * 2)(10, 5)
    assert B.selsync_chunk_table_preview(arr, None, 2, 1000, 0, None, None, None, ctypes.byref(n)) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_chunk_table_preview(arr, None, 2, 8192, 0, None, None, None, None) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_chunk_table_preview(None, None, 2, 8192, 0, None, None, None, ctypes.byref(n)) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_chunk_table_preview(arr, None, 2, 0, 0, None, None, None, ctypes.byref(n)) == 0 and n.value == 2


def test_product_path_has_no_cpu_fallback_and_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2307_07950_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower() or f == "workloads.py", f
    src = open(os.path.join(pkg, "workloads.py")).read()
    assert "import oracle" not in src and "from oracle" not in src
    # and the oracle does not import the product
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            assert "paper_2307_07950_amd" not in open(os.path.join(ROOT, "oracle", f)).read()


def test_workload_shapes_match_the_stated_models():
    from paper_2307_07950_amd import workloads as W
    for name in ("c1", "c2", "c3", "c4", "c5"):
        wl = W.get(name)
        assert (wl.num_tensors, wl.num_params) == W.FULL_SIZE_PARAMS[wl.name]
    # 507 MB fp32 model size quoted for VGG11 (Sec. II-A)
    assert round(W.get("c4").num_params * 4 / 2 ** 20) == 507


def test_workload_generators_are_seeded_and_order_independent():
    from paper_2307_07950_amd import workloads as W
    wl = W.get("c1")
    a = W.unit_grads(wl, 2, 3)
    _ = W.unit_grads(wl, 0, 0)
    b = W.unit_grads(wl, 2, 3)
    for x, y in zip(a, b):
        assert x.tobytes() == y.tobytes()
    assert a[0].tobytes() != W.unit_grads(wl, 1, 3)[0].tobytes()
    wl5 = W.get("c5", shrink=8)
    g = W.unit_grads(wl5, 0, 0)
    assert g[0].dtype == np.uint16
    f = W.tensor_factors(wl5)
    assert 50 < max(f) / min(f) <= 100.0 + 1e-9


@pytest.mark.parametrize("D,N", [(100, 4), (103, 4), (7, 3), (5, 8), (0, 3), (1000, 16), (17, 1), (12345, 7)])
def test_partition_order_matches_oracle_bit_for_bit(B, D, N):
    # Sec. III-D: integer work, compared exactly against the oracle's plain construction
    from oracle import selsync_oracle as O
    for n in range(N):
        assert B.partition_order(D, N, n, seldp=True) == O.seldp_order(D, N, n)
        assert B.partition_order(D, N, n, seldp=False) == O.defdp_order(D, N, n)


def test_partition_order_rejects_bad_arguments(B):
    n = ctypes.c_int64()
    bad = B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_partition_order(-1, 4, 0, 1, 0, None, ctypes.byref(n)) == bad
    assert B.selsync_partition_order(10, 0, 0, 1, 0, None, ctypes.byref(n)) == bad
    assert B.selsync_partition_order(10, 4, 4, 1, 0, None, ctypes.byref(n)) == bad
    assert B.selsync_partition_order(10, 4, -1, 1, 0, None, ctypes.byref(n)) == bad
    assert B.selsync_partition_order(10, 4, 0, 2, 0, None, ctypes.byref(n)) == bad
    assert B.selsync_partition_order(10, 4, 0, 1, 0, None, None) == bad
    # capacity smaller than the order: only `capacity` entries are written
    out = (ctypes.c_int64 * 4)(-1, -1, -1, -1)
    assert B.selsync_partition_order(10, 4, 1, 1, 3, out, ctypes.byref(n)) == 0
    assert n.value == 10 and list(out) == [3, 4, 5, -1]
