"""Host-only checks of the C ABI: the library loads, exports what include/torq.h
declares, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2605_19561_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "torq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([A-Za-z_0-9]+)\s*\(", text)
    return sorted({n for n in names if n.startswith("torq_") or n.startswith("mxfp4_")})


def test_header_and_library_agree():
    L = binding.lib()
    declared = _declared()
    assert declared == sorted(binding.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings():
    for s in (0, -1, -2, -3, -4, -5, -6, -7, -8, -99):
        assert isinstance(binding.status_string(s), str) and binding.status_string(s)


def test_rotation_create_rejects_bad_arguments():
    L = binding.lib()
    h = C.c_void_p()
    Ri = np.eye(128, dtype=np.float32)
    Ra = np.eye(32, dtype=np.float32)
    pi, pa = Ri.ctypes.data_as(C.c_void_p), Ra.ctypes.data_as(C.c_void_p)
    assert L.torq_rotation_create(None, 4096, 128, pi, pa) == binding.TORQ_EINVAL
    assert L.torq_rotation_create(C.byref(h), 4096, 128, None, pa) == binding.TORQ_EINVAL
    assert L.torq_rotation_create(C.byref(h), 4096, 128, pi, None) == binding.TORQ_EINVAL
    assert L.torq_rotation_create(C.byref(h), 4100, 128, pi, pa) == binding.TORQ_EINVAL    # d % 32
    assert L.torq_rotation_create(C.byref(h), 4096, 24, pi, pa) == binding.TORQ_EINVAL     # G % 16
    assert L.torq_rotation_create(C.byref(h), 4096, 48, pi, pa) == binding.TORQ_EINVAL     # G does not divide 128
    assert L.torq_rotation_create(C.byref(h), 32 * 512, 512, pi, pa) == binding.TORQ_EINVAL  # G too large
    assert L.torq_rotation_create(C.byref(h), 0, 128, pi, pa) == binding.TORQ_EINVAL
    assert not h.value
    L.torq_rotation_destroy(None)


def test_compute_calls_reject_bad_arguments_without_launching():
    L = binding.lib()
    good = C.c_void_p(0x1000)       # never dereferenced: every call below fails validation first
    odd = C.c_void_p(0x1004)
    assert L.torq_quantize_f32(good, -1, 4096, good, good, None) == binding.TORQ_EINVAL
    assert L.torq_quantize_f32(good, 4, 100, good, good, None) == binding.TORQ_EINVAL
    assert L.torq_quantize_f32(None, 4, 4096, good, good, None) == binding.TORQ_EINVAL
    assert L.torq_quantize_f32(odd, 4, 4096, good, good, None) == binding.TORQ_EALIGN
    assert L.torq_quantize_f32(good, 0, 4096, None, None, None) == binding.TORQ_OK            # empty
    assert L.mxfp4_gemm(good, good, good, good, good, 4, 4, 96, None) == binding.TORQ_EINVAL  # d % 128
    assert L.mxfp4_gemm(good, good, good, good, good, -4, 4, 128, None) == binding.TORQ_EINVAL
    assert L.mxfp4_gemm(None, good, good, good, good, 4, 4, 128, None) == binding.TORQ_EINVAL
    assert L.mxfp4_gemm(odd, good, good, good, good, 4, 4, 128, None) == binding.TORQ_EALIGN
    assert L.mxfp4_gemm(good, good, good, good, good, 0, 4, 128, None) == binding.TORQ_OK
    assert L.mxfp4_gemm(good, good, good, good, good, 4, 0, 128, None) == binding.TORQ_OK
    assert L.torq_rotate_quantize(None, good, 4, good, good, None) == binding.TORQ_EINVAL
    assert L.torq_rotate(None, good, 4, good, None) == binding.TORQ_EINVAL
    assert L.torq_linear(None, good, good, good, good, 4, 4, good, 1 << 20, None) == binding.TORQ_EINVAL
    assert L.torq_linear_static(None, good, good, good, good, 4, 4, None) == binding.TORQ_EINVAL
    assert L.torq_rotation_d(None) == binding.TORQ_EINVAL
    odd2 = C.c_void_p(0x1002)
    assert L.torq_diag_mfma_burn(7, good, 4096, 4, good, None) == binding.TORQ_EINVAL          # unknown kind
    assert L.torq_diag_mfma_burn(0, None, 4096, 4, good, None) == binding.TORQ_EINVAL
    assert L.torq_diag_mfma_burn(0, good, 64, 4, good, None) == binding.TORQ_EINVAL            # too few operand bytes
    assert L.torq_diag_mfma_burn(1, good, 4096, 0, good, None) == binding.TORQ_EINVAL
    assert L.torq_diag_mfma_burn(1, odd2, 4096, 4, good, None) == binding.TORQ_EALIGN
    assert L.torq_diag_copy(good, good, 100, None) == binding.TORQ_EINVAL                      # not a multiple of 16
    assert L.torq_diag_copy(None, good, 160, None) == binding.TORQ_EINVAL
    assert L.torq_diag_copy(odd, good, 160, None) == binding.TORQ_EALIGN
    assert L.torq_diag_gemm_ablation(good, good, good, good, good, 256, 256, 768, 0, None) == binding.TORQ_EINVAL   # d % 512
    assert L.torq_diag_gemm_ablation(good, good, good, good, good, 256, 256, 1024, 2, None) == binding.TORQ_EINVAL  # unknown skip
    assert L.torq_diag_gemm_ablation(good, odd, good, good, good, 256, 256, 1024, 0, None) == binding.TORQ_EALIGN
    assert L.torq_diag_gemm_persistent(good, good, good, good, good, 256, 256, 1536, 0, 8, None) == binding.TORQ_EINVAL   # d % 1024
    assert L.torq_diag_gemm_persistent(good, good, good, good, good, 256, 256, 1024, 2, 8, None) == binding.TORQ_EINVAL   # unknown tile
    assert L.torq_diag_gemm_persistent(good, good, good, good, good, 256, 256, 1024, 0, 0, None) == binding.TORQ_EINVAL   # no workgroups
    assert L.torq_diag_gemm_persistent(good, good, good, good, None, 256, 256, 1024, 0, 8, None) == binding.TORQ_EINVAL
    assert L.torq_diag_gemm_persistent(good, good, good, odd, good, 256, 256, 1024, 0, 8, None) == binding.TORQ_EALIGN
    # torq_diag_gemm_plan: what a form of the tiled kernel cannot take is refused before anything is launched
    plan = lambda *a: L.torq_diag_gemm_plan(*a)
    assert plan(good, good, good, good, good, 256, 256, 1024, 4, 1, 0, None, 0, None) == binding.TORQ_EINVAL    # unknown tile
    assert plan(good, good, good, good, good, 256, 256, 1024, 2, 0, 0, None, 0, None) == binding.TORQ_EINVAL    # no pieces
    assert plan(good, good, good, good, good, 256, 256, 1024, 0, 1, 1, None, 0, None) == binding.TORQ_EINVAL    # deep: small tiles only
    assert plan(good, good, good, good, good, 256, 256, 640, 3, 1, 0, None, 0, None) == binding.TORQ_EINVAL     # 128x64 needs d % 512 == 0
    assert plan(good, good, good, good, good, 256, 256, 1024, 2, 2, 0, None, 0, None) == binding.TORQ_EINVAL    # a cut needs a workspace
    assert plan(good, good, good, good, good, 256, 256, 1024, 2, 2, 0, good, 1024, None) == binding.TORQ_EINVAL  # ... large enough
    assert plan(good, good, good, good, good, 256, 256, 1536, 2, 2, 0, good, 1 << 30, None) == binding.TORQ_EINVAL  # 3 pairs / 2
    assert plan(good, good, good, good, good, 256, 252, 1024, 2, 2, 0, good, 1 << 30, None) == binding.TORQ_EINVAL  # N % 8
    assert plan(good, good, good, good, good, 256, 256, 1024, 2, 2, 0, odd, 1 << 30, None) == binding.TORQ_EALIGN
    assert plan(good, good, good, good, None, 256, 256, 1024, 2, 1, 0, None, 0, None) == binding.TORQ_EINVAL
    assert L.torq_diag_rotate_ablation(None, good, 4, good, good, 0, None) == binding.TORQ_EINVAL


def test_workspace_size():
    L = binding.lib()
    assert L.torq_linear_workspace_bytes(0, 4096) == 0
    assert L.torq_linear_workspace_bytes(4, 100) == 0
    # codes M*d/2 and scales M*d/32, each rounded up to 256 bytes
    assert L.torq_linear_workspace_bytes(64, 4096) == 64 * 2048 + 64 * 128
    assert L.torq_linear_workspace_bytes(1, 4096) == 2048 + 256
    assert L.torq_linear_workspace_bytes(3, 32) == 256 + 256


@pytest.mark.skipif(os.path.exists("/dev/kfd"), reason="a GPU is present")
def test_rotation_create_without_device_reports_it():
    L = binding.lib()
    h = C.c_void_p()
    Ri = np.eye(16, dtype=np.float32)
    Ra = np.eye(32, dtype=np.float32)
    st = L.torq_rotation_create(C.byref(h), 512, 16, Ri.ctypes.data_as(C.c_void_p), Ra.ctypes.data_as(C.c_void_p))
    assert st == binding.TORQ_ENODEVICE and not h.value


def test_gemm_workspace_entry_points_validate_and_plan_on_the_host():
    L = binding.lib()
    good, odd = C.c_void_p(0x1000), C.c_void_p(0x1004)
    assert L.mxfp4_gemm_ws(good, good, good, good, good, 4, 4, 96, good, 1 << 20, None) == binding.TORQ_EINVAL
    assert L.mxfp4_gemm_ws(good, good, good, good, None, 4, 4, 128, good, 1 << 20, None) == binding.TORQ_EINVAL
    assert L.mxfp4_gemm_ws(good, good, good, good, good, 4, 4, 128, odd, 1 << 20, None) == binding.TORQ_EALIGN
    assert L.mxfp4_gemm_ws(good, good, good, good, good, 0, 4, 128, None, 0, None) == binding.TORQ_OK
    # the plan and the workspace size are pure host functions of the shape
    assert binding.mxfp4_gemm_workspace_bytes(8192, 28672, 8192) == 0            # plenty of tiles: never cut
    assert binding.mxfp4_gemm_plan(8192, 28672, 8192) == (False, 256, 256, 1)
    assert binding.mxfp4_gemm_plan(1, 14336, 4096)[0] is True                    # a decode row streams the weights
    need = binding.mxfp4_gemm_workspace_bytes(128, 8192, 28672)
    streaming, tm, tn, pieces = binding.mxfp4_gemm_plan(128, 8192, 28672, need)
    assert not streaming and pieces > 1 and need == pieces * 128 * 8192 * 4
    assert (28672 // 512) % pieces == 0                                          # whole, even runs of iterations
    assert binding.mxfp4_gemm_plan(128, 8192, 28672, need - 1)[3] == 1           # too small: not cut
    assert binding.mxfp4_gemm_workspace_bytes(96, 512, 4100) == 0                # invalid d: nothing to size
    assert binding.mxfp4_gemm_workspace_bytes(96, 516, 4096) == 0                # N % 8 != 0: fp32 rows not 16-byte aligned
    assert binding.torq_linear_workspace_bytes_n(128, 8192, 28672) == binding.torq_linear_workspace_bytes(128, 28672) + need
    # a round and a quarter of 256 x 256 tiles: the whole round first, the remaining columns on their own
    assert binding.mxfp4_gemm_main_columns(4096, 5120, 5120) == 4096
    assert binding.mxfp4_gemm_plan(4096, 5120, 5120) == (False, 256, 256, 1)
    assert binding.mxfp4_gemm_main_columns(4096, 25600, 5120) == 24576          # six rounds and a quarter
    need = binding.mxfp4_gemm_workspace_bytes(4096, 5120, 25600)                # the remainder's k range is cut
    assert binding.mxfp4_gemm_main_columns(4096, 5120, 25600, need) == 4096
    pieces = binding.mxfp4_gemm_plan(4096, 1024, 25600, need)[3]
    assert pieces > 1 and need == pieces * 4096 * 1024 * 4
    for M, N, d in [(8192, 28672, 8192), (8192, 8192, 28672), (2048, 14336, 4096), (4096, 5124, 5120), (64, 70000, 4096)]:
        assert binding.mxfp4_gemm_main_columns(M, N, d) == N                    # whole rounds, a last round more than
    assert binding.mxfp4_gemm_main_columns(0, 4, 128) == 0                      # half full, N % 8 != 0, few rows; invalid
    v = [C.c_int() for _ in range(4)]
    assert L.mxfp4_gemm_plan(0, 4, 128, 0, *(C.byref(x) for x in v)) == binding.TORQ_EINVAL
    assert L.mxfp4_gemm_plan(4, 4, 128, 0, None, C.byref(v[1]), C.byref(v[2]), C.byref(v[3])) == binding.TORQ_EINVAL


def test_gemm_planner_invariants_over_random_shapes():
    # whatever the cost model prefers, a plan has to be one the kernels can run: pieces that divide the k range
    # into whole pairs of iterations, fp32 rows that are 16-byte aligned, a workspace that holds them, a first
    # launch of whole tile columns
    import numpy as np
    rng = np.random.default_rng(20260519)
    shapes = [(int(rng.integers(1, 5000)), int(rng.integers(1, 40000)), 128 * int(rng.integers(1, 225))) for _ in range(400)]
    shapes += [(M, N, d) for M in (1, 64, 65, 4096) for N in (8, 1000, 5120, 70000) for d in (128, 512, 5120, 28672)]
    for M, N, d in shapes:
        need = binding.mxfp4_gemm_workspace_bytes(M, N, d)
        for ws in (0, need):
            main = binding.mxfp4_gemm_main_columns(M, N, d, ws)
            assert main == N or (0 < main < N and main % 256 == 0 and d % 512 == 0 and N % 8 == 0), (M, N, d, main)
            for n in ((N,) if main == N else (N, N - main)):
                streaming, tm, tn, pieces = binding.mxfp4_gemm_plan(M, n, d, ws)
                if streaming:
                    assert M <= 64 and pieces == 1
                    continue
                assert (tm, tn) in ((256, 256), (256, 128), (128, 128), (128, 64)), (M, n, d, tm, tn)
                if (tm, tn) == (128, 64):
                    assert d % 512 == 0
                if pieces > 1:
                    assert d % 512 == 0 and (d // 512) % pieces == 0 and n % 8 == 0 and (tm, tn) != (256, 256)
                    assert ws >= pieces * M * n * 4, (M, n, d, pieces, ws)
            if main < N:
                assert binding.mxfp4_gemm_plan(M, N, d, ws)[:3] == (False, 256, 256)


def test_format_entry_points_reject_unknown_formats_and_bad_scales():
    L = binding.lib()
    good = C.c_void_p(0x1000)
    f = C.c_float
    assert L.torq_quantize_f32_fmt(good, 4, 64, 3, f(1.0), good, good, None) == binding.TORQ_EINVAL      # unknown format
    assert L.torq_quantize_f32_fmt(good, 4, 64, -1, f(1.0), good, good, None) == binding.TORQ_EINVAL
    assert L.torq_quantize_f32_fmt(good, 4, 64, 2, f(0.0), good, good, None) == binding.TORQ_EINVAL      # NVFP4 needs a positive scale
    assert L.torq_quantize_f32_fmt(good, 4, 64, 2, f(-1.0), good, good, None) == binding.TORQ_EINVAL
    assert L.torq_quantize_f32_fmt(good, 4, 64, 2, f(float("inf")), good, good, None) == binding.TORQ_EINVAL
    assert L.torq_quantize_f32_fmt(good, 4, 48, 1, f(1.0), good, good, None) == binding.TORQ_EINVAL      # d % 32
    assert L.torq_quantize_f32_fmt(good, 0, 64, 1, f(0.0), None, None, None) == binding.TORQ_OK          # empty; scale unused
    assert L.torq_quantize_f32_fmt(C.c_void_p(0x1004), 4, 64, 1, f(1.0), good, good, None) == binding.TORQ_EALIGN
    assert L.torq_rotate_quantize_fmt(None, good, 4, 1, f(1.0), good, good, None) == binding.TORQ_EINVAL


def test_host_routines_reject_non_finite_and_out_of_range_input():
    L = binding.lib()
    # Algorithm 1 helper: a NaN in Sigma must not come back as "converged, R = I"
    G = 16
    Sigma = np.diag(np.arange(1.0, G + 1.0))
    R = np.zeros((G, G), dtype=np.float32)
    steps = C.c_int(-1)
    args = lambda S: (S.ctypes.data_as(C.c_void_p), G, C.c_double(1e-12), R.ctypes.data_as(C.c_void_p), C.byref(steps))
    assert L.torq_equalize_inter(*args(Sigma)) == binding.TORQ_OK and steps.value > 0
    for bad in (np.nan, np.inf, -np.inf):
        S = Sigma.copy()
        S[3, 5] = bad
        R[:] = 7.0
        assert L.torq_equalize_inter(*args(S)) == binding.TORQ_EINVAL
        assert (R == 7.0).all()                     # nothing written
    # butterfly handle: tangents beyond the stated limit (or NaN) are refused before any device work
    Gb = 32
    Ra = np.eye(32, dtype=np.float32)
    h = C.c_void_p()
    for bad in (np.float32(binding.TORQ_BUTTERFLY_MAX_TAN) * 2, -np.float32(1e30), np.float32(np.nan), np.float32(np.inf)):
        T = np.zeros((5, Gb // 2), dtype=np.float32)
        T[2, 7] = bad
        st = L.torq_rotation_create_butterfly(C.byref(h), 32 * Gb, Gb, T.ctypes.data_as(C.c_void_p),
                                              Ra.ctypes.data_as(C.c_void_p))
        assert st == binding.TORQ_EINVAL and not h.value
    # one-launch layer: its test hook validates the wait limit; the counter calls need a handle
    good = C.c_void_p(0x1000)
    assert L.torq_linear_single_launch_probe(None, good, good, good, good, 4, 4, good, 1 << 20, 16, 1, None) == binding.TORQ_EINVAL
    assert L.torq_linear_single_launch_reset(None, None) == binding.TORQ_EINVAL
    assert L.torq_linear_single_launch_gave_up(None, None) == binding.TORQ_EINVAL


def test_bench_refuses_more_than_one_gpu():
    # the build is for one GPU: asking bench.py for more ends with a message before anything is imported
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "ONE GPU" in (p.stdout + p.stderr)
