"""Host-side behaviour of the C ABI that needs no GPU: argument checks happen before any device is touched,
null handles are errors, and without a device the library says so instead of falling back to anything."""
import ctypes
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

import paper_1808_03843_amd as P
from paper_1808_03843_amd.binding import AlsConfig

EINVAL, EHIP = -1, -2


def _cfg(f=100, solver=None, cg_iters=6, factor_dtype=None, herm_dtype=None, device=0, chunk=0, batch_slots=0):
    return AlsConfig(f, P.SOLVER_CG if solver is None else solver, cg_iters, 0.0,
                     P.F32 if factor_dtype is None else factor_dtype, P.F32 if herm_dtype is None else herm_dtype,
                     device, None, chunk, batch_slots, 0)


def _create(cfg):
    lib = P.load_library()
    ctx = ctypes.c_void_p()
    rc = lib.als_create(ctypes.byref(ctx), ctypes.byref(cfg))
    if rc == 0:
        lib.als_destroy(ctx)
    return rc


def test_error_codes_are_the_documented_ones():
    import os
    import re
    header = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "als.h")).read()
    codes = dict(re.findall(r"#define (ALS_E[A-Z]+) \(?(-\d+)\)?", header))
    assert int(codes["ALS_EINVAL"]) == EINVAL and int(codes["ALS_EHIP"]) == EHIP


@pytest.mark.parametrize("cfg", [
    _cfg(f=17), _cfg(f=0), _cfg(f=512),                                   # unsupported widths
    _cfg(solver=7), _cfg(cg_iters=-1),
    _cfg(factor_dtype=9), _cfg(herm_dtype=P.F16),                         # fp16 cannot store A_u
    _cfg(solver=P.SOLVER_CHOLESKY, herm_dtype=P.BF16),                    # reduced storage goes with the approximate solver
    _cfg(f=256, factor_dtype=P.BF16, herm_dtype=P.BF16),
    _cfg(chunk=100), _cfg(chunk=32), _cfg(chunk=1 << 21), _cfg(chunk=-64), _cfg(batch_slots=-1),
])
def test_als_create_rejects_bad_configurations_before_touching_a_device(cfg):
    assert _create(cfg) == EINVAL


def test_als_create_null_arguments():
    lib = P.load_library()
    ctx = ctypes.c_void_p()
    assert lib.als_create(None, ctypes.byref(_cfg())) == EINVAL
    assert lib.als_create(ctypes.byref(ctx), None) == EINVAL


def test_device_that_does_not_exist_is_an_error_not_a_fallback():
    """A device ordinal beyond the last one (on a box without a GPU: any ordinal) gives ALS_EHIP and no context."""
    assert _create(_cfg(device=4096)) == EHIP
    assert _create(_cfg(device=-1)) == EHIP


def test_null_context_is_rejected_by_every_entry_point():
    lib = P.load_library()
    lib.als_destroy(None)   # allowed
    assert lib.als_last_error(None) == b"context is null"
    d = ctypes.c_double()
    n = ctypes.c_int64()
    assert lib.als_update_rows(None, None, None, 0.1, 100, None) == EINVAL
    assert lib.als_update_cols(None, None, None, 0.1, 100, None) == EINVAL
    assert lib.als_update_rows_implicit(None, None, None, 0.1, 1.0, 100, None) == EINVAL
    assert lib.als_update_cols_implicit(None, None, None, 0.1, 1.0, 100, None) == EINVAL
    assert lib.als_rmse(None, None, None, None, 100, ctypes.byref(d)) == EINVAL
    assert lib.als_implicit_loss(None, None, None, None, 0.1, 1.0, 100, ctypes.byref(d)) == EINVAL
    assert lib.als_gram(None, None, 0, 100, None) == EINVAL
    assert lib.als_hermitian(None, None, None, 0.1, 100, 0, 0, None, None) == EINVAL
    assert lib.als_bin_rows(None, None, 8, None, None) == EINVAL
    assert lib.als_csr_to_csc(None, None, None, None, None) == EINVAL
    assert lib.als_synchronize(None) == EINVAL
    assert lib.als_kernel_time(None, 0, ctypes.byref(d), ctypes.byref(n)) == EINVAL
    assert lib.als_profile_reset(None) == EINVAL
    assert lib.als_drop_plans(None) == EINVAL
    assert lib.als_check_matrix(None, None) == EINVAL
    assert lib.als_measure_peak(None, 0, ctypes.byref(d)) == EINVAL


def test_bench_traffic_figures_agree_with_the_committed_counter_summary():
    """bench.py reports roofline.traffic from a table typed in from a rocprofv3 counter run; the summary of that
    run is committed under profiles/.  The two must agree: FETCH_SIZE counts 2 KiB and WRITE_SIZE 1 KiB per unit
    on this machine (calibrated against a copy of known size, stated in the summary), summed per kernel over the
    dispatches of one sweep and divided by its launches."""
    import re
    import bench
    path = os.path.join(ROOT, bench.TRAFFIC_SOURCE)
    text = open(path).read()
    assert "1 unit = 2 KiB" in text and "1 unit = 1 KiB" in text          # the calibration the table relies on
    sums, launches = {}, {}
    for line in text.splitlines():
        m = re.match(r"(k_hermitian(?:_cg)?)<.*?(FETCH_SIZE|WRITE_SIZE)=([0-9.e+]+)", line)
        if not m or line.startswith("#"):
            continue
        kernel, counter, value = m.group(1), m.group(2), float(m.group(3))
        sums[kernel] = sums.get(kernel, 0.0) + value * (2048 if counter == "FETCH_SIZE" else 1024)
        if counter == "FETCH_SIZE":
            launches[kernel] = launches.get(kernel, 0) + 1
    table = bench.MEASURED_TRAFFIC_BYTES_PER_LAUNCH[("mid", 100, "cg", 6, "f32", 4096)]
    assert set(table) == set(sums) == {"k_hermitian", "k_hermitian_cg"}
    for kernel, per_launch in table.items():
        assert launches[kernel] == 2                                       # one launch per side and sweep
        assert per_launch == pytest.approx(sums[kernel] / launches[kernel], rel=1e-3)


def test_workspace_bytes_needs_no_device_and_grows_with_the_matrix():
    lib = P.load_library()
    cfg = _cfg()
    small = lib.als_workspace_bytes(ctypes.byref(cfg), 1000, 100_000)
    mid = lib.als_workspace_bytes(ctypes.byref(cfg), 480_189, 99_072_112)
    assert 0 < small < mid
    assert small % 256 == 0 and mid % 256 == 0
    # the slots dominate: min(batch_slots, 2 nnz / chunk + 1) partial Gram matrices of slot_floats(100) floats
    slot = 4 * (28 * 256 + 7 * 16)
    assert mid >= (2 * 99_072_112 // 4096 + 1) * slot
    # a smaller batch bounds the slot region; bf16 storage halves it (nearly)
    capped = lib.als_workspace_bytes(ctypes.byref(_cfg(batch_slots=1024)), 480_189, 99_072_112)
    assert capped < mid and capped <= 1024 * slot + 64 * 2 ** 20
    half = lib.als_workspace_bytes(ctypes.byref(_cfg(herm_dtype=P.BF16)), 480_189, 99_072_112)
    assert 0.45 * mid < half < 0.6 * mid
    # refused configurations and sizes give 0
    assert lib.als_workspace_bytes(ctypes.byref(_cfg(f=17)), 10, 10) == 0
    assert lib.als_workspace_bytes(ctypes.byref(cfg), -1, 10) == 0
    assert lib.als_workspace_bytes(None, 10, 10) == 0


def test_create_refuses_a_workspace_that_is_too_small_or_misaligned():
    lib = P.load_library()
    need = lib.als_workspace_bytes(ctypes.byref(_cfg()), 1000, 100_000)
    for ptr, size, rows, nnz in [(0x1000, need - 1, 1000, 100_000),      # too small
                                 (0x1010, need, 1000, 100_000),          # not 256-byte aligned
                                 (0x1000, need, -1, 100_000),            # negative maximum
                                 (0, need, 1000, 100_000)]:              # sizes without a workspace
        cfg = _cfg()
        cfg.workspace, cfg.workspace_bytes, cfg.workspace_max_rows, cfg.workspace_max_nnz = ptr, size, rows, nnz
        assert _create(cfg) == EINVAL     # found before any device is touched


def test_three_part_inputs_are_refused_where_they_do_not_exist():
    assert _create(_cfg(f=256, factor_dtype=P.F32X3)) == EINVAL          # the route exists for f <= 128
    assert _create(_cfg(f=256, factor_dtype=P.F32X2)) == EINVAL
    assert _create(_cfg(f=100, factor_dtype=5)) == EINVAL                # no such element type
