"""Host-side checks of the C-ABI library: it loads, exports every symbol the header declares,
validates arguments and sizes buffers.  No kernel runs here."""
import ctypes as C
import os
import re
from fractions import Fraction

import pytest

from paper_2501_02379_amd import sizing, synth, tgrad as T

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "tgrad.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tgrad_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = T.load()
    names = _declared_symbols()
    assert set(names) == set(T.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_strerror_names_every_status():
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -6):
        s = T.strerror(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 7
    assert T.strerror(-99) == "unknown status"


def test_query_sizes_counts_the_compressed_state():
    w = synth.WORKLOADS["cfg4"]
    cfg = T.make_config(w.shape, w.ranks, w.k, refresh_every=w.T)
    rc, sb, wb = T.tgrad_query_sizes(cfg)
    assert rc == T.TGRAD_OK
    core = 32 * 32 * 32 * 16
    factors = 3 * 128 * 32 + 65 * 16
    exact = core * 12 + w.k * 16 + factors * 8
    assert exact <= sb <= exact + 16 * 256           # plus alignment padding only
    dense_adam = w.numel * 12                        # complex64 M + float32 V
    assert sb / dense_adam < 0.011
    assert wb > 0


@pytest.mark.parametrize("mutate,expected", [
    (lambda c: setattr(c, "ndim", 1), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "ndim", 7), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: c.shape.__setitem__(0, 0), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: c.rank.__setitem__(1, 0), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: c.rank.__setitem__(1, 99), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "k_sparse", -1), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "k_sparse", 16 * 16 * 8 * 5 + 1), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "grad_dtype", 7), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "weight_dtype", 5), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "beta1", 1.0), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "lr", float("nan")), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "refresh_every", -1), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "hooi_sweeps", -1), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "hooi_sweeps", 65), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "warm_restart", 1), T.TGRAD_ERR_INVALID_ARG),      # needs hooi_sweeps >= 1
    (lambda c: (setattr(c, "hooi_sweeps", 1), setattr(c, "warm_restart", 2)), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "select_rule", 2), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "order", 3), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "eig_max_sweeps", -1), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "eig_max_sweeps", 31), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: setattr(c, "select_rule", -1), T.TGRAD_ERR_INVALID_ARG),
    (lambda c: c.shape.__setitem__(0, 1 << 31), T.TGRAD_ERR_UNSUPPORTED),
])
def test_bad_configs_are_rejected(mutate, expected):
    cfg = T.make_config((16, 16, 8, 5), (8, 8, 4, 3), 103)
    mutate(cfg)
    rc, _, _ = T.tgrad_query_sizes(cfg)
    assert rc == expected
    h = C.c_void_p(None)
    rc2 = T.load().tgrad_init(C.byref(h), C.byref(cfg), 256, 256, None)
    assert rc2 == expected and not h


def test_null_and_misaligned_pointers():
    lib = T.load()
    cfg = T.make_config((16, 16, 8, 5), (8, 8, 4, 3), 103)
    h = C.c_void_p(None)
    assert lib.tgrad_init(None, C.byref(cfg), 256, 256, None) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_init(C.byref(h), None, 256, 256, None) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_init(C.byref(h), C.byref(cfg), None, 256, None) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_init(C.byref(h), C.byref(cfg), 256, 264, None) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_step(None, 256, 512) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_refresh_factors(None, 256) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_destroy(None) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_query_sizes(C.byref(cfg), None, None) == T.TGRAD_ERR_INVALID_ARG


def test_calibration_probes_check_their_arguments_before_the_device():
    lib = T.load()
    fl = C.c_double(0.0)
    assert lib.tgrad_calibration_mfma(2, 16, 256, None, C.byref(fl)) == T.TGRAD_ERR_INVALID_ARG     # no such instruction
    assert lib.tgrad_calibration_mfma(0, 0, 256, None, C.byref(fl)) == T.TGRAD_ERR_INVALID_ARG      # no iterations
    assert lib.tgrad_calibration_mfma(0, 16, None, None, C.byref(fl)) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_calibration_mfma(0, 16, 258, None, C.byref(fl)) == T.TGRAD_ERR_INVALID_ARG     # sink alignment
    assert lib.tgrad_calibration_mfma(1, 16, 256, None, None) == T.TGRAD_ERR_INVALID_ARG
    n = C.c_int64(0)
    assert lib.tgrad_calibration_tile_stream(None, 1 << 20, 1024, 4, None, C.byref(n)) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_calibration_tile_stream(256, 1 << 20, 1000, 4, None, C.byref(n)) == T.TGRAD_ERR_INVALID_ARG   # not whole pieces
    assert lib.tgrad_calibration_tile_stream(256, 1 << 20, 18 * 1024, 4, None, C.byref(n)) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_calibration_tile_stream(256, 1 << 20, 1024, 0, None, C.byref(n)) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_calibration_tile_stream(256, 2048, 1024, 4, None, C.byref(n)) == T.TGRAD_ERR_INVALID_ARG      # less than a slab
    assert lib.tgrad_calibration_tile_stream(256, 1 << 20, 1024, 4, None, None) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_calibration_copy(256, 512, 24, None) == T.TGRAD_ERR_INVALID_ARG                # not a multiple of 16
    assert lib.tgrad_calibration_copy(256, 264, 16, None) == T.TGRAD_ERR_INVALID_ARG                # alignment
    assert lib.tgrad_calibration_copy(256, 512, 512, None) == T.TGRAD_ERR_INVALID_ARG               # overlap


def test_caller_side_sizes():
    for w in synth.WORKLOADS.values():
        assert sizing.sparse_count(Fraction(*w.density), w.numel) == w.k
        assert tuple(sizing.rank_from_ratio(Fraction(1, 2) if w.name == "cfg1" else Fraction(1, 4), i)
                     for i in w.shape) == w.ranks


def test_static_step_argument_checks_need_no_gpu():
    """Everything `tgrad_step_static` refuses is refused before it looks at the device."""
    lib = T.load()
    big = synth.WORKLOADS["cfg4"]
    cfg = T.make_config(big.shape, big.ranks, big.k, refresh_every=big.T)
    rc, _, wb = T.tgrad_query_sizes(cfg)
    assert rc == T.TGRAD_OK and wb > T.STATIC_WORKSPACE_BYTES
    assert lib.tgrad_step_static(C.byref(cfg), 256, 0, 512, 1024, None) == T.TGRAD_ERR_UNSUPPORTED
    small = T.make_config((16, 16, 8, 5), (8, 8, 4, 3), 103, refresh_every=5)
    assert lib.tgrad_step_static(None, 256, 0, 512, 1024, None) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_step_static(C.byref(small), None, 0, 512, 1024, None) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_step_static(C.byref(small), 256, 0, None, 1024, None) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_step_static(C.byref(small), 256, 0, 512, None, None) == T.TGRAD_ERR_INVALID_ARG
    assert lib.tgrad_step_static(C.byref(small), 264, 0, 512, 1024, None) == T.TGRAD_ERR_INVALID_ARG   # state alignment
    assert lib.tgrad_step_static(C.byref(small), 256, 0, 512, 512, None) == T.TGRAD_ERR_INVALID_ARG    # W aliases G
    assert lib.tgrad_step_static(C.byref(small), 256, -1, 512, 1024, None) == T.TGRAD_ERR_INVALID_ARG
    small.refresh_every = 0
    assert lib.tgrad_step_static(C.byref(small), 256, 0, 512, 1024, None) == T.TGRAD_ERR_INVALID_ARG


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: the benchmark says so and exits instead of pretending to scale."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_byte_model_of_the_headline_workload():
    """The algorithmic bytes per launch that the roofline fractions rest on, written out by hand for the
    128 x 128 x 128 x 65 workload (I elements of 8 bytes, k sparse entries, ranks 32, 32, 32, 16)."""
    import os
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    w = synth.WORKLOADS["cfg4"]
    I, k = 128 * 128 * 128 * 65, w.k
    mid = 128 * 128 * 32 * 16 * 8                      # the tensor between the fused end kernels and the core kernel
    m = bench.kernel_model(w, True, 8, 2)
    assert m["project_first"]["bytes"] == 8 * I + mid + 12 * k          # G in, result out, index + value per sparse entry
    assert m["update"]["bytes"] == 16 * I + mid + 36 * k                # W in and out, operand tensor in, sparse state
    assert m["core"]["bytes"] == 2 * mid + 32 * (32 * 32 * 32 * 16)     # in, out, moments in and out + core gradient out
    assert "project" not in m and "backproject" not in m
    # three separate middle kernels instead: one mode each way, the core kernel one mode
    m1 = bench.kernel_model(w, True, 8, 1)
    assert m1["project"]["launches_per_step"] == 1 and m1["backproject"]["launches_per_step"] == 1
    assert m1["update"]["bytes"] == m["update"]["bytes"]
