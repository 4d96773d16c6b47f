"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/lcn.h declares, and rejects bad arguments before it
touches the device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "lcn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:lcn_status|void|const char \*)\s*\**\s*(\w+)\s*\(", text)
    return sorted(set(n for n in names if n not in ("lcn_status",)))


def test_header_declares_the_expected_entry_points():
    names = _declared_functions()
    for required in ("lcn_build", "sinkhorn_run", "transport_cost", "plan_marginals", "lcn_workspace_bytes",
                     "lcn_get_scalings", "lcn_set_scalings", "lcn_get_landmarks", "lcn_get_buckets", "lcn_get_csr",
                     "lcn_get_factors", "lcn_get_info", "lcn_destroy", "lcn_status_string", "lcn_build_batched",
                     "lcn_batched_results", "lcn_batched_get", "lcn_last_run_timing", "lcn_backward",
                     "lcn_backward_scratch_bytes", "lcn_plan_rows", "lcn_deletion_costs", "lcn_head_lambdas",
                     "lcn_last_error_counts", "lcn_backward_static", "lcn_calibrate"):
        assert required in names


def test_library_loads_and_exports_every_declared_symbol():
    import paper_2107_06876_amd as lcn
    lib = lcn.load_library()
    assert os.path.basename(lcn.library_path()) == "liblcn_hip.so"
    for name in _declared_functions():
        assert hasattr(lib, name), "missing symbol %s" % name


def test_status_strings():
    import paper_2107_06876_amd as lcn
    seen = {lcn.lcn_status_string(i) for i in range(9)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert lcn.lcn_status_string(99) == "unknown status"


def test_invalid_arguments_are_rejected_before_any_device_work():
    """Every call below must return INVALID_ARG / STATE from the host-side
    checks; none may reach a HIP call (there is no GPU here)."""
    import paper_2107_06876_amd as lcn
    from paper_2107_06876_amd.binding import (ERR_INVALID_ARG, ERR_STATE, LandmarkParams, LshParams, OK)
    lib = lcn.load_library()
    vp = ctypes.c_void_p
    fake = vp(256 * 1024)           # never dereferenced: validation fails first
    out = vp()
    need = ctypes.c_size_t()
    lm = LandmarkParams(8, 10, 1, 0.0)
    ls = LshParams(0, 4, 1, 10, 1, None)

    def build(**kw):
        args = dict(X=fake, n=100, Y=fake, m=100, d=4, dtype=0, a=fake, b=fake, lam=0.5, cost=0, mode=3,
                    lm=ctypes.byref(lm), ls=ctypes.byref(ls), ws=fake, wsb=1 << 20)
        args.update(kw)
        return lib.lcn_build(args["X"], args["n"], args["Y"], args["m"], args["d"], args["dtype"], args["a"],
                             args["b"], args["lam"], args["cost"], args["mode"], args["lm"], args["ls"], args["ws"],
                             args["wsb"], None, ctypes.byref(need), ctypes.byref(out))

    assert build(X=None) == ERR_INVALID_ARG
    assert build(n=0) == ERR_INVALID_ARG
    assert build(d=0) == ERR_INVALID_ARG
    assert build(lam=0.0) == ERR_INVALID_ARG
    assert build(lam=-1.0) == ERR_INVALID_ARG
    assert build(lam=float("nan")) == ERR_INVALID_ARG
    assert build(cost=7) == ERR_INVALID_ARG
    assert build(mode=9) == ERR_INVALID_ARG
    assert build(dtype=5) == ERR_INVALID_ARG
    assert build(lm=None) == ERR_INVALID_ARG               # LCN needs landmarks
    assert build(ls=None) == ERR_INVALID_ARG               # ... and hashing
    assert build(ws=vp(12345)) == ERR_INVALID_ARG          # misaligned workspace
    assert build(n=1 << 20, m=1 << 20) == ERR_INVALID_ARG  # k-means needs n + m <= 2^20
    lm_bad = LandmarkParams(1000, 10, 1, 0.0)
    assert build(lm=ctypes.byref(lm_bad)) == ERR_INVALID_ARG
    lm_bad = LandmarkParams(8, -1, 1, 0.0)
    assert build(lm=ctypes.byref(lm_bad)) == ERR_INVALID_ARG
    lm_bad = LandmarkParams(8, 10, 1, 0.0, 3, None)         # unknown start
    assert build(lm=ctypes.byref(lm_bad)) == ERR_INVALID_ARG
    lm_bad = LandmarkParams(8, 10, 1, 0.0, 2, None)         # LCN_INIT_GIVEN without centroids
    assert build(lm=ctypes.byref(lm_bad)) == ERR_INVALID_ARG
    lm_bad = LandmarkParams(8, 10, 1, 0.0, 1, 256 * 1024)   # centroids given although the start is not GIVEN
    assert build(lm=ctypes.byref(lm_bad)) == ERR_INVALID_ARG
    lm_bad = LandmarkParams(8, 10, 1, -1.0)
    assert build(lm=ctypes.byref(lm_bad)) == ERR_INVALID_ARG
    ls_bad = LshParams(1, 5, 1, 10, 1, None)               # cross-polytope: odd bucket count, no projections
    assert build(ls=ctypes.byref(ls_bad)) == ERR_INVALID_ARG
    ls_bad = LshParams(0, 4, 9, 10, 1, None)
    assert build(ls=ctypes.byref(ls_bad)) == ERR_INVALID_ARG
    assert out.value is None

    # workspace too small: reported as ALLOC with the size that is needed, still without device work
    from paper_2107_06876_amd.binding import ERR_ALLOC
    assert build(wsb=4096) == ERR_ALLOC and need.value > 4096
    assert lcn.lcn_workspace_bytes(100, 100, 4, lcn.MODE_LCN, dict(num_landmarks=8), dict(num_buckets=4, num_rounds=1)) \
        >= need.value - 256 - 8 * 100 * 100  # same layout, plus the sparse-value guess

    # null / foreign handles
    d = ctypes.c_double()
    assert lib.sinkhorn_run(None, 5) == ERR_STATE
    assert lib.transport_cost(None, ctypes.byref(d)) == ERR_STATE
    assert lib.plan_marginals(None, None, None, None) == ERR_STATE
    assert lib.lcn_get_scalings(None, None, None) == ERR_STATE
    c = ctypes.c_int64(-7)
    assert lib.lcn_last_error_counts(None, ctypes.byref(c), None, None) == ERR_STATE and c.value == -7
    junk = (ctypes.c_uint32 * 64)()
    assert lib.sinkhorn_run(ctypes.cast(junk, vp), 5) == ERR_STATE
    assert lib.sinkhorn_run(ctypes.cast(junk, vp), -1) == ERR_INVALID_ARG
    assert lib.lcn_last_error_counts(ctypes.cast(junk, vp), None, None, None) == ERR_STATE
    assert lib.lcn_backward_static(None, None, None, None, None) == ERR_STATE
    assert lib.lcn_backward_static(ctypes.cast(junk, vp), None, None, None, None) == ERR_STATE
    lib.lcn_destroy(None)                                   # must be a no-op
    lib.lcn_destroy(ctypes.cast(junk, vp))


def test_batched_arguments():
    import paper_2107_06876_amd as lcn
    from paper_2107_06876_amd.binding import BatchDesc, ERR_INVALID_ARG, LandmarkParams, LshParams
    lib = lcn.load_library()
    vp = ctypes.c_void_p
    fake = vp(256 * 1024)
    out, need = vp(), ctypes.c_size_t()
    lm = LandmarkParams(8, 10, 1, 0.0)
    ls = LshParams(0, 4, 1, 10, 1, None)

    def call(x_off, y_off, lam, d=8):
        x_off = np.asarray(x_off, dtype=np.int64)
        y_off = np.asarray(y_off, dtype=np.int64)
        lam = np.asarray(lam, dtype=np.float32)
        desc = BatchDesc(len(lam), x_off.ctypes.data, y_off.ctypes.data, lam.ctypes.data, None, None)
        return lib.lcn_build_batched(fake, fake, d, ctypes.byref(desc), 1, 3, ctypes.byref(lm), ctypes.byref(ls), fake,
                                     1 << 20, None, ctypes.byref(need), ctypes.byref(out))

    assert call([0, 70], [0, 20], [0.1]) == ERR_INVALID_ARG       # more than 64 points on a side
    assert call([0, 20], [0, 0], [0.1]) == ERR_INVALID_ARG        # empty side
    assert call([0, 20], [0, 20], [0.0]) == ERR_INVALID_ARG       # lambda
    assert call([0, 20], [0, 20], [0.1], d=100) == ERR_INVALID_ARG
    assert call([0, 3], [0, 3], [0.1]) == ERR_INVALID_ARG         # fewer points than landmarks
    assert call([1, 20], [0, 20], [0.1]) == ERR_INVALID_ARG       # offsets must start at 0


def test_head_lambdas_host_call():
    """lcn_head_lambdas runs on the host: lambda_k = 2^(k - K/2) lambda, k = 1 .. K (Sec. 6)."""
    import oracle
    import paper_2107_06876_amd as lcn
    from paper_2107_06876_amd.binding import ERR_INVALID_ARG
    for lam, K in ((0.05, 1), (0.25, 2), (0.1, 8), (3.0, 5)):
        np.testing.assert_array_equal(lcn.lcn_head_lambdas(lam, K), oracle.head_lambdas(lam, K))
    lib = lcn.load_library()
    buf = np.zeros(64, dtype=np.float32)
    assert lib.lcn_head_lambdas(0.0, 4, buf.ctypes.data) == ERR_INVALID_ARG
    assert lib.lcn_head_lambdas(0.1, 0, buf.ctypes.data) == ERR_INVALID_ARG
    assert lib.lcn_head_lambdas(0.1, 65, buf.ctypes.data) == ERR_INVALID_ARG
    assert lib.lcn_head_lambdas(0.1, 4, None) == ERR_INVALID_ARG
    assert lib.lcn_head_lambdas(1e38, 64, buf.ctypes.data) == ERR_INVALID_ARG   # overflows fp32
    assert lib.lcn_deletion_costs(None, 4, 4, None, None, None) == ERR_INVALID_ARG
    assert lib.lcn_deletion_costs(ctypes.c_void_p(256), -1, 4, ctypes.c_void_p(256), ctypes.c_void_p(256),
                                  None) == ERR_INVALID_ARG
    assert lib.lcn_deletion_costs(ctypes.c_void_p(256), 4, 0, ctypes.c_void_p(256), ctypes.c_void_p(256),
                                  None) == ERR_INVALID_ARG


def test_gpu_entry_points_fail_loudly_without_the_library(monkeypatch, tmp_path):
    """There is no CPU fallback: a missing library is an error."""
    import paper_2107_06876_amd.binding as binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError):
        binding.load_library()


def test_calibrate_validates_its_arguments_before_it_touches_the_device():
    import ctypes
    import paper_2107_06876_amd as lcn
    from paper_2107_06876_amd.binding import ERR_INVALID_ARG
    lib = lcn.load_library()
    v = ctypes.c_double(0.0)
    assert lib.lcn_calibrate(0, None, 1 << 30, None, ctypes.byref(v)) == ERR_INVALID_ARG     # no workspace
    assert lib.lcn_calibrate(0, 4096, 1 << 20, None, ctypes.byref(v)) == ERR_INVALID_ARG     # too small
    assert lib.lcn_calibrate(0, 4097, 1 << 30, None, ctypes.byref(v)) == ERR_INVALID_ARG     # misaligned
    assert lib.lcn_calibrate(5, 4096, 1 << 30, None, ctypes.byref(v)) == ERR_INVALID_ARG     # no such figure
    assert lib.lcn_calibrate(0, 4096, 1 << 30, None, None) == ERR_INVALID_ARG                # nowhere to put it
