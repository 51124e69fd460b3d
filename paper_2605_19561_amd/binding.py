"""Thin ctypes binding of libtorq.so: same names as the C ABI (include/torq.h).

Argument marshalling only: torch supplies device memory and the current HIP
stream, every step of the path runs in the library's kernels.  There is no CPU
fallback: a missing library or a failing call raises.
"""
import ctypes as C
import os

import torch  # loads the HIP runtime that libtorq.so binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtorq.so")

EXPORTS = [
    "torq_status_string", "torq_rotation_create", "torq_rotation_destroy", "torq_rotation_d",
    "torq_rotation_G", "torq_rotate_quantize", "torq_rotate", "torq_quantize_f32", "mxfp4_gemm",
    "torq_linear_workspace_bytes", "torq_linear", "mxfp4_gemm_workspace_bytes", "mxfp4_gemm_ws", "mxfp4_gemm_plan", "mxfp4_gemm_main_columns",
    "torq_rotate_quantize_fmt", "torq_quantize_f32_fmt", "torq_equalize_inter_butterfly",
    "torq_rotation_create_butterfly", "torq_linear_single_launch",
    "torq_linear_workspace_bytes_n", "torq_block_gram_workspace_bytes", "torq_block_gram", "torq_block_gram_positions",
    "torq_equalize_inter", "torq_code_histogram_workspace_bytes", "torq_code_histogram", "torq_intra_pair_scores",
    "torq_intra_best_angle", "torq_calibrate_intra", "torq_diag_mfma_burn", "torq_linear_static",
    "torq_diag_copy", "torq_diag_gemm_ablation", "torq_diag_gemm_persistent", "torq_diag_gemm_plan", "torq_diag_rotate_ablation", "torq_linear_single_launch_reset", "torq_linear_single_launch_gave_up", "torq_linear_single_launch_probe",
]

TORQ_OK, TORQ_EINVAL, TORQ_EALIGN, TORQ_EWORKSPACE, TORQ_EHIP, TORQ_ENODEVICE, TORQ_ECONVERGE = 0, -1, -2, -3, -4, -5, -6
TORQ_ETOOBIG = -7
TORQ_ENOMEM = -8
TORQ_BUTTERFLY_MAX_TAN = 256.0
TORQ_STATIC_SCRATCH_BYTES = 4 << 20

_lib = None


class TorqError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


def lib():
    """Load libtorq.so (built by paper_2605_19561_amd.build); raise if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2605_19561_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
        L.torq_status_string.restype = C.c_char_p
        L.torq_status_string.argtypes = [i32]
        L.torq_rotation_create.restype = i32
        L.torq_rotation_create.argtypes = [C.POINTER(vp), i32, i32, vp, vp]
        L.torq_rotation_destroy.restype = None
        L.torq_rotation_destroy.argtypes = [vp]
        L.torq_rotation_d.restype = i32
        L.torq_rotation_d.argtypes = [vp]
        L.torq_rotation_G.restype = i32
        L.torq_rotation_G.argtypes = [vp]
        L.torq_rotate_quantize.restype = i32
        L.torq_rotate_quantize.argtypes = [vp, vp, i64, vp, vp, vp]
        L.torq_rotate.restype = i32
        L.torq_rotate.argtypes = [vp, vp, i64, vp, vp]
        L.torq_quantize_f32.restype = i32
        L.torq_quantize_f32.argtypes = [vp, i64, i32, vp, vp, vp]
        L.mxfp4_gemm.restype = i32
        L.mxfp4_gemm.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, vp]
        L.mxfp4_gemm_workspace_bytes.restype = sz
        L.mxfp4_gemm_workspace_bytes.argtypes = [i64, i64, i32]
        L.torq_equalize_inter_butterfly.restype = i32
        L.torq_equalize_inter_butterfly.argtypes = [vp, i32, vp, vp]
        L.torq_rotation_create_butterfly.restype = i32
        L.torq_rotation_create_butterfly.argtypes = [C.POINTER(vp), i32, i32, vp, vp]
        L.torq_rotate_quantize_fmt.restype = i32
        L.torq_rotate_quantize_fmt.argtypes = [vp, vp, i64, i32, C.c_float, vp, vp, vp]
        L.torq_quantize_f32_fmt.restype = i32
        L.torq_quantize_f32_fmt.argtypes = [vp, i64, i32, i32, C.c_float, vp, vp, vp]
        L.mxfp4_gemm_plan.restype = i32
        L.mxfp4_gemm_plan.argtypes = [i64, i64, i32, sz] + [C.POINTER(i32)] * 4
        L.mxfp4_gemm_main_columns.restype = i64
        L.mxfp4_gemm_main_columns.argtypes = [i64, i64, i32, sz]
        L.mxfp4_gemm_ws.restype = i32
        L.mxfp4_gemm_ws.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, vp, sz, vp]
        L.torq_linear_workspace_bytes_n.restype = sz
        L.torq_linear_workspace_bytes_n.argtypes = [i64, i64, i32]
        L.torq_linear_workspace_bytes.restype = sz
        L.torq_linear_workspace_bytes.argtypes = [i64, i32]
        L.torq_linear.restype = i32
        L.torq_linear.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, sz, vp]
        L.torq_linear_static.restype = i32
        L.torq_linear_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp]
        L.torq_linear_single_launch.restype = i32
        L.torq_linear_single_launch.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, sz, vp]
        L.torq_linear_single_launch_probe.restype = i32
        L.torq_linear_single_launch_probe.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, sz, i32, i32, vp]
        L.torq_linear_single_launch_reset.restype = i32
        L.torq_linear_single_launch_reset.argtypes = [vp, vp]
        L.torq_linear_single_launch_gave_up.restype = i32
        L.torq_linear_single_launch_gave_up.argtypes = [vp, C.POINTER(i32)]
        L.torq_block_gram_workspace_bytes.restype = sz
        L.torq_block_gram_workspace_bytes.argtypes = [i32]
        L.torq_block_gram.restype = i32
        L.torq_block_gram.argtypes = [vp, i64, i32, i32, vp, vp, sz, vp]
        L.torq_block_gram_positions.restype = i32
        L.torq_block_gram_positions.argtypes = [vp, i64, i32, i32, vp, vp, sz, vp]
        L.torq_equalize_inter.restype = i32
        L.torq_equalize_inter.argtypes = [vp, i32, C.c_double, vp, C.POINTER(i32)]
        L.torq_code_histogram_workspace_bytes.restype = sz
        L.torq_code_histogram_workspace_bytes.argtypes = []
        L.torq_code_histogram.restype = i32
        L.torq_code_histogram.argtypes = [vp, i64, i32, vp, vp, sz, vp]
        L.torq_intra_pair_scores.restype = i32
        L.torq_intra_pair_scores.argtypes = [vp, C.c_double, vp, vp]
        L.torq_intra_best_angle.restype = i32
        L.torq_intra_best_angle.argtypes = [vp, vp, i64, vp, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                            C.POINTER(i64)]
        L.torq_calibrate_intra.restype = i32
        L.torq_calibrate_intra.argtypes = [vp, i64, i32, i32, i32, C.c_double, C.c_double, vp, vp, C.POINTER(i32)]
        L.torq_diag_mfma_burn.restype = i32
        L.torq_diag_mfma_burn.argtypes = [i32, vp, sz, i32, vp, vp]
        L.torq_diag_gemm_ablation.restype = i32
        L.torq_diag_gemm_ablation.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, vp]
        L.torq_diag_gemm_persistent.restype = i32
        L.torq_diag_gemm_persistent.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, i32, vp]
        L.torq_diag_gemm_plan.restype = i32
        L.torq_diag_gemm_plan.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, i32, i32, vp, sz, vp]
        L.torq_diag_rotate_ablation.restype = i32
        L.torq_diag_rotate_ablation.argtypes = [vp, vp, i64, vp, vp, i32, vp]
        L.torq_diag_copy.restype = i32
        L.torq_diag_copy.argtypes = [vp, vp, sz, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().torq_status_string(int(status)).decode()


def _check(status, what):
    if status != TORQ_OK:
        raise TorqError(status, what)


def _stream(stream=None):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dev(t: torch.Tensor, dtype, what):
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise ValueError(f"{what}: expected a contiguous {dtype} device tensor")
    return C.c_void_p(t.data_ptr())


class Rotation:
    """Owner of a torq_rotation_t handle (R_inter [G, G], R_intra [32, 32], fp32 host arrays)."""

    def __init__(self, d: int, G: int, R_inter, R_intra):
        import numpy as np
        Ri = np.ascontiguousarray(R_inter, dtype=np.float32)
        Ra = np.ascontiguousarray(R_intra, dtype=np.float32)
        if Ri.shape != (G, G) or Ra.shape != (32, 32):
            raise ValueError("R_inter must be [G, G] and R_intra [32, 32]")
        h = C.c_void_p()
        _check(lib().torq_rotation_create(C.byref(h), d, G, Ri.ctypes.data_as(C.c_void_p),
                                          Ra.ctypes.data_as(C.c_void_p)), "torq_rotation_create")
        self.handle, self.d, self.G = h, d, G

    def close(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.torq_rotation_destroy(self.handle)
        self.handle = None

    __del__ = close


class ButterflyRotation(Rotation):
    """Handle whose inter-block rotation is a butterfly of plane rotations (tangents [log2 G, G/2])."""

    def __init__(self, d: int, G: int, tangents, R_intra):
        import numpy as np
        T = np.ascontiguousarray(tangents, dtype=np.float32)
        Ra = np.ascontiguousarray(R_intra, dtype=np.float32)
        if T.shape != (G.bit_length() - 1, G // 2) or Ra.shape != (32, 32):
            raise ValueError("tangents must be [log2 G, G/2] and R_intra [32, 32]")
        h = C.c_void_p()
        _check(lib().torq_rotation_create_butterfly(C.byref(h), d, G, T.ctypes.data_as(C.c_void_p),
                                                    Ra.ctypes.data_as(C.c_void_p)), "torq_rotation_create_butterfly")
        self.handle, self.d, self.G = h, d, G


def torq_equalize_inter_butterfly(Sigma):
    """Butterfly equaliser on the host.  Returns (R_inter float32 [G, G], tangents float32 [log2 G, G/2])."""
    import numpy as np
    S = np.ascontiguousarray(Sigma, dtype=np.float64)
    G = S.shape[0]
    if S.shape != (G, G):
        raise ValueError("Sigma must be square")
    R = np.empty((G, G), np.float32)
    T = np.empty((max(G.bit_length() - 1, 1), max(G // 2, 1)), np.float32)
    _check(lib().torq_equalize_inter_butterfly(S.ctypes.data_as(C.c_void_p), G, R.ctypes.data_as(C.c_void_p),
                                               T.ctypes.data_as(C.c_void_p)), "torq_equalize_inter_butterfly")
    return R, T


def torq_rotate_quantize(rot: Rotation, x_bf16: torch.Tensor, codes=None, scales=None, stream=None):
    M, d = x_bf16.shape
    assert d == rot.d
    if codes is None:
        codes = torch.empty((M, d // 2), dtype=torch.uint8, device=x_bf16.device)
    if scales is None:
        scales = torch.empty((M, d // 32), dtype=torch.uint8, device=x_bf16.device)
    _check(lib().torq_rotate_quantize(rot.handle, _dev(x_bf16, torch.bfloat16, "x"), M,
                                      _dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"),
                                      _stream(stream)), "torq_rotate_quantize")
    return codes, scales


def torq_rotate(rot: Rotation, x_bf16: torch.Tensor, z=None, stream=None):
    M, d = x_bf16.shape
    assert d == rot.d
    if z is None:
        z = torch.empty((M, d), dtype=torch.float32, device=x_bf16.device)
    _check(lib().torq_rotate(rot.handle, _dev(x_bf16, torch.bfloat16, "x"), M, _dev(z, torch.float32, "z"),
                             _stream(stream)), "torq_rotate")
    return z


def torq_quantize_f32(z: torch.Tensor, codes=None, scales=None, stream=None):
    M, d = z.shape
    if codes is None:
        codes = torch.empty((M, d // 2), dtype=torch.uint8, device=z.device)
    if scales is None:
        scales = torch.empty((M, d // 32), dtype=torch.uint8, device=z.device)
    _check(lib().torq_quantize_f32(_dev(z, torch.float32, "z"), M, d, _dev(codes, torch.uint8, "codes"),
                                   _dev(scales, torch.uint8, "scales"), _stream(stream)), "torq_quantize_f32")
    return codes, scales


TORQ_FMT_MXFP4, TORQ_FMT_MXINT4, TORQ_FMT_NVFP4 = 0, 1, 2


def _scale_cols(d: int, fmt: int) -> int:
    return d // 16 if fmt == TORQ_FMT_NVFP4 else d // 32


def torq_rotate_quantize_fmt(rot: Rotation, x_bf16: torch.Tensor, fmt: int, global_scale: float = 1.0,
                             codes=None, scales=None, stream=None):
    M, d = x_bf16.shape
    assert d == rot.d
    if codes is None:
        codes = torch.empty((M, d // 2), dtype=torch.uint8, device=x_bf16.device)
    if scales is None:
        scales = torch.empty((M, _scale_cols(d, fmt)), dtype=torch.uint8, device=x_bf16.device)
    _check(lib().torq_rotate_quantize_fmt(rot.handle, _dev(x_bf16, torch.bfloat16, "x"), M, int(fmt),
                                          float(global_scale), _dev(codes, torch.uint8, "codes"),
                                          _dev(scales, torch.uint8, "scales"), _stream(stream)),
           "torq_rotate_quantize_fmt")
    return codes, scales


def torq_quantize_f32_fmt(z: torch.Tensor, fmt: int, global_scale: float = 1.0, codes=None, scales=None, stream=None):
    M, d = z.shape
    if codes is None:
        codes = torch.empty((M, d // 2), dtype=torch.uint8, device=z.device)
    if scales is None:
        scales = torch.empty((M, _scale_cols(d, fmt)), dtype=torch.uint8, device=z.device)
    _check(lib().torq_quantize_f32_fmt(_dev(z, torch.float32, "z"), M, d, int(fmt), float(global_scale),
                                       _dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"),
                                       _stream(stream)), "torq_quantize_f32_fmt")
    return codes, scales


def mxfp4_gemm(A_q, A_s, W_q, W_s, out=None, stream=None):
    M, half = A_q.shape
    N = W_q.shape[0]
    d = half * 2
    assert W_q.shape == (N, half) and A_s.shape == (M, d // 32) and W_s.shape == (N, d // 32)
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=A_q.device)
    _check(lib().mxfp4_gemm(_dev(A_q, torch.uint8, "A_q"), _dev(A_s, torch.uint8, "A_s"),
                            _dev(W_q, torch.uint8, "W_q"), _dev(W_s, torch.uint8, "W_s"),
                            _dev(out, torch.bfloat16, "out"), M, N, d, _stream(stream)), "mxfp4_gemm")
    return out


def mxfp4_gemm_workspace_bytes(M: int, N: int, d: int) -> int:
    return int(lib().mxfp4_gemm_workspace_bytes(M, N, d))


def mxfp4_gemm_plan(M: int, N: int, d: int, workspace_bytes: int = 0):
    """Returns (weight_streaming, tile_m, tile_n, k_pieces) for a product of that shape."""
    v = [C.c_int(0) for _ in range(4)]
    _check(lib().mxfp4_gemm_plan(M, N, d, workspace_bytes, *(C.byref(x) for x in v)), "mxfp4_gemm_plan")
    return bool(v[0].value), v[1].value, v[2].value, v[3].value


def mxfp4_gemm_main_columns(M: int, N: int, d: int, workspace_bytes: int = 0) -> int:
    """N, or the leading output columns that a first launch of whole rounds of tiles computes."""
    return int(lib().mxfp4_gemm_main_columns(M, N, d, workspace_bytes))


def mxfp4_gemm_ws(A_q, A_s, W_q, W_s, out=None, workspace=None, stream=None):
    """mxfp4_gemm with scratch memory for cutting the k range (allocated here if not given)."""
    M, half = A_q.shape
    N = W_q.shape[0]
    d = half * 2
    assert W_q.shape == (N, half) and A_s.shape == (M, d // 32) and W_s.shape == (N, d // 32)
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=A_q.device)
    if workspace is None:
        workspace = torch.empty((max(mxfp4_gemm_workspace_bytes(M, N, d), 16),), dtype=torch.uint8, device=A_q.device)
    _check(lib().mxfp4_gemm_ws(_dev(A_q, torch.uint8, "A_q"), _dev(A_s, torch.uint8, "A_s"),
                               _dev(W_q, torch.uint8, "W_q"), _dev(W_s, torch.uint8, "W_s"),
                               _dev(out, torch.bfloat16, "out"), M, N, d, _dev(workspace, torch.uint8, "workspace"),
                               workspace.numel(), _stream(stream)), "mxfp4_gemm_ws")
    return out


def torq_linear_workspace_bytes(M: int, d: int) -> int:
    return int(lib().torq_linear_workspace_bytes(M, d))


def torq_linear_workspace_bytes_n(M: int, N: int, d: int) -> int:
    return int(lib().torq_linear_workspace_bytes_n(M, N, d))


def torq_linear_single_launch(rot: Rotation, x_bf16, W_q, W_s, out=None, workspace=None, stream=None):
    """torq_linear for at most 64 rows, G = 128, in one kernel launch (see include/torq.h)."""
    M, d = x_bf16.shape
    N = W_q.shape[0]
    assert d == rot.d and W_q.shape == (N, d // 2) and W_s.shape == (N, d // 32)
    if workspace is None:
        workspace = torch.empty((max(torq_linear_workspace_bytes(M, d), 1),), dtype=torch.uint8, device=x_bf16.device)
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=x_bf16.device)
    _check(lib().torq_linear_single_launch(rot.handle, _dev(x_bf16, torch.bfloat16, "x"), _dev(W_q, torch.uint8, "W_q"),
                                           _dev(W_s, torch.uint8, "W_s"), _dev(out, torch.bfloat16, "out"), M, N,
                                           _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)),
           "torq_linear_single_launch")
    return out


def torq_linear_single_launch_probe(rot: Rotation, x_bf16, W_q, W_s, spin_limit, withhold_ready, out=None,
                                    workspace=None, stream=None):
    """torq_linear_single_launch with its wait limit and the hand-off switch exposed (tests of the give-up path)."""
    M, d = x_bf16.shape
    N = W_q.shape[0]
    assert d == rot.d and W_q.shape == (N, d // 2) and W_s.shape == (N, d // 32)
    if workspace is None:
        workspace = torch.empty((max(torq_linear_workspace_bytes(M, d), 1),), dtype=torch.uint8, device=x_bf16.device)
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=x_bf16.device)
    _check(lib().torq_linear_single_launch_probe(
        rot.handle, _dev(x_bf16, torch.bfloat16, "x"), _dev(W_q, torch.uint8, "W_q"), _dev(W_s, torch.uint8, "W_s"),
        _dev(out, torch.bfloat16, "out"), M, N, _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
        int(spin_limit), int(bool(withhold_ready)), _stream(stream)), "torq_linear_single_launch_probe")
    return out


def torq_linear_single_launch_reset(rot: Rotation, stream=None):
    _check(lib().torq_linear_single_launch_reset(rot.handle, _stream(stream)), "torq_linear_single_launch_reset")


def torq_linear_single_launch_gave_up(rot: Rotation) -> bool:
    flag = C.c_int(0)
    _check(lib().torq_linear_single_launch_gave_up(rot.handle, C.byref(flag)), "torq_linear_single_launch_gave_up")
    return bool(flag.value)


def torq_linear(rot: Rotation, x_bf16, W_q, W_s, out=None, workspace=None, stream=None):
    M, d = x_bf16.shape
    N = W_q.shape[0]
    assert d == rot.d and W_q.shape == (N, d // 2) and W_s.shape == (N, d // 32)
    if workspace is None:
        workspace = torch.empty((max(torq_linear_workspace_bytes_n(M, N, d), 1),), dtype=torch.uint8,
                                device=x_bf16.device)
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=x_bf16.device)
    _check(lib().torq_linear(rot.handle, _dev(x_bf16, torch.bfloat16, "x"), _dev(W_q, torch.uint8, "W_q"),
                             _dev(W_s, torch.uint8, "W_s"), _dev(out, torch.bfloat16, "out"), M, N,
                             _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)),
           "torq_linear")
    return out


def torq_linear_static(rot: Rotation, x_bf16, W_q, W_s, out, stream=None):
    """torq_linear through the library's built-in scratch: the caller passes inputs and the output only."""
    M, d = x_bf16.shape
    N = W_q.shape[0]
    assert d == rot.d and W_q.shape == (N, d // 2) and W_s.shape == (N, d // 32) and out.shape == (M, N)
    _check(lib().torq_linear_static(rot.handle, _dev(x_bf16, torch.bfloat16, "x"), _dev(W_q, torch.uint8, "W_q"),
                                    _dev(W_s, torch.uint8, "W_s"), _dev(out, torch.bfloat16, "out"), M, N,
                                    _stream(stream)), "torq_linear_static")
    return out


TORQ_DIAG_FP4, TORQ_DIAG_BF16 = 0, 1
TORQ_DIAG_SINK_FLOATS = 1024 * 256
TORQ_DIAG_FLOP_PER_ITER = {TORQ_DIAG_FP4: 1024.0 * 4 * 16 * 2 * 32 * 32 * 64,
                           TORQ_DIAG_BF16: 1024.0 * 4 * 16 * 2 * 32 * 32 * 16}


def torq_diag_mfma_burn(kind: int, operands: torch.Tensor, iters: int, sink=None, stream=None):
    """Enqueue the matrix-core burn kernel on `operands` (any contiguous device tensor); returns
    the number of floating-point operations it executes."""
    if not (operands.is_cuda and operands.is_contiguous()):
        raise ValueError("operands: expected a contiguous device tensor")
    if sink is None:
        sink = torch.empty((TORQ_DIAG_SINK_FLOATS,), dtype=torch.float32, device=operands.device)
    _check(lib().torq_diag_mfma_burn(kind, C.c_void_p(operands.data_ptr()), operands.numel() * operands.element_size(),
                                     iters, _dev(sink, torch.float32, "sink"), _stream(stream)),
           "torq_diag_mfma_burn")
    return TORQ_DIAG_FLOP_PER_ITER[kind] * iters


def torq_diag_gemm_ablation(A_q, A_s, W_q, W_s, out, skip: int, stream=None):
    """mxfp4_gemm's 256 x 256-tile kernel with parts of its k loop left out (see include/torq.h); `out` is garbage."""
    M, N, d = A_q.shape[0], W_q.shape[0], A_q.shape[1] * 2
    _check(lib().torq_diag_gemm_ablation(_dev(A_q, torch.uint8, "A_q"), _dev(A_s, torch.uint8, "A_s"),
                                         _dev(W_q, torch.uint8, "W_q"), _dev(W_s, torch.uint8, "W_s"),
                                         _dev(out, torch.bfloat16, "out"), M, N, d, int(skip), _stream(stream)),
           "torq_diag_gemm_ablation")


def torq_diag_gemm_persistent(A_q, A_s, W_q, W_s, tile: int, workgroups: int, out=None, stream=None):
    """mxfp4_gemm on the persistent form of its tiled kernel with `workgroups` workgroups (see include/torq.h)."""
    M, N, d = A_q.shape[0], W_q.shape[0], A_q.shape[1] * 2
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=A_q.device)
    _check(lib().torq_diag_gemm_persistent(_dev(A_q, torch.uint8, "A_q"), _dev(A_s, torch.uint8, "A_s"),
                                           _dev(W_q, torch.uint8, "W_q"), _dev(W_s, torch.uint8, "W_s"),
                                           _dev(out, torch.bfloat16, "out"), M, N, d, int(tile), int(workgroups),
                                           _stream(stream)), "torq_diag_gemm_persistent")
    return out


def torq_diag_gemm_plan(A_q, A_s, W_q, W_s, tile: int, k_pieces: int = 1, deep: bool = False, out=None, workspace=None,
                        stream=None):
    """mxfp4_gemm's tiled kernel on a chosen tile shape, number of k pieces and load pipeline (see include/torq.h)."""
    M, N, d = A_q.shape[0], W_q.shape[0], A_q.shape[1] * 2
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=A_q.device)
    if workspace is None and k_pieces > 1:
        workspace = torch.empty((k_pieces * M * N * 4,), dtype=torch.uint8, device=A_q.device)
    ws_ptr = _dev(workspace, torch.uint8, "workspace") if workspace is not None else None
    _check(lib().torq_diag_gemm_plan(_dev(A_q, torch.uint8, "A_q"), _dev(A_s, torch.uint8, "A_s"),
                                     _dev(W_q, torch.uint8, "W_q"), _dev(W_s, torch.uint8, "W_s"),
                                     _dev(out, torch.bfloat16, "out"), M, N, d, int(tile), int(k_pieces), int(bool(deep)),
                                     ws_ptr, workspace.numel() if workspace is not None else 0, _stream(stream)),
           "torq_diag_gemm_plan")
    return out


def torq_diag_rotate_ablation(rot, x_bf16, codes, scales, skip: int, stream=None):
    """torq_rotate_quantize's G = 128 kernel with work left out (see include/torq.h); codes / scales are garbage."""
    _check(lib().torq_diag_rotate_ablation(rot.handle, _dev(x_bf16, torch.bfloat16, "x"), x_bf16.shape[0],
                                           _dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"),
                                           int(skip), _stream(stream)), "torq_diag_rotate_ablation")


def torq_diag_copy(src: torch.Tensor, dst: torch.Tensor, stream=None):
    """dst <- src by the library's own copy kernel (known traffic: the counters' yardstick)."""
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n and src.is_cuda and dst.is_cuda
    assert src.is_contiguous() and dst.is_contiguous()
    _check(lib().torq_diag_copy(C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()), n, _stream(stream)),
           "torq_diag_copy")
    return dst


def torq_block_gram_workspace_bytes(G: int) -> int:
    return int(lib().torq_block_gram_workspace_bytes(G))


def torq_block_gram(x_bf16: torch.Tensor, G: int, Sigma=None, workspace=None, stream=None):
    """Sigma [G, G] float64 on the device: mean Gram matrix of the runs of G blocks of x's rows."""
    M, d = x_bf16.shape
    if Sigma is None:
        Sigma = torch.empty((G, G), dtype=torch.float64, device=x_bf16.device)
    if workspace is None:
        workspace = torch.empty((max(torq_block_gram_workspace_bytes(G), 16),), dtype=torch.uint8,
                                device=x_bf16.device)
    _check(lib().torq_block_gram(_dev(x_bf16, torch.bfloat16, "x"), M, d, G, _dev(Sigma, torch.float64, "Sigma"),
                                 _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)),
           "torq_block_gram")
    return Sigma


def torq_block_gram_positions(x_bf16: torch.Tensor, G: int, Sigma_pos=None, workspace=None, stream=None):
    """Sigma_pos [32, G, G] float64 on the device: the Gram matrix kept apart by the position inside a block."""
    M, d = x_bf16.shape
    if Sigma_pos is None:
        Sigma_pos = torch.empty((32, G, G), dtype=torch.float64, device=x_bf16.device)
    if workspace is None:
        workspace = torch.empty((max(torq_block_gram_workspace_bytes(G), 16),), dtype=torch.uint8,
                                device=x_bf16.device)
    _check(lib().torq_block_gram_positions(_dev(x_bf16, torch.bfloat16, "x"), M, d, G,
                                           _dev(Sigma_pos, torch.float64, "Sigma_pos"),
                                           _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                           _stream(stream)), "torq_block_gram_positions")
    return Sigma_pos


def torq_equalize_inter(Sigma, eps: float = 0.0):
    """Algorithm 1 on the host.  Sigma: [G, G] array-like (float64).  Returns (R_inter float32 [G, G], steps)."""
    import numpy as np
    S = np.ascontiguousarray(Sigma, dtype=np.float64)
    G = S.shape[0]
    if S.shape != (G, G):
        raise ValueError("Sigma must be square")
    R = np.empty((G, G), np.float32)
    steps = C.c_int(0)
    _check(lib().torq_equalize_inter(S.ctypes.data_as(C.c_void_p), G, float(eps), R.ctypes.data_as(C.c_void_p),
                                     C.byref(steps)), "torq_equalize_inter")
    return R, steps.value


def torq_code_histogram_workspace_bytes() -> int:
    return int(lib().torq_code_histogram_workspace_bytes())


def torq_code_histogram(codes: torch.Tensor, d: int, counts: torch.Tensor = None, workspace: torch.Tensor = None,
                        stream=None):
    """codes: uint8 [M, d/2] device (packed e2m1).  Returns counts int64 [32, 8] device (N_j^(k), Appendix A.5)."""
    M = codes.shape[0]
    if codes.dim() != 2 or codes.shape[1] * 2 != d:
        raise ValueError("codes must be [M, d/2]")
    if counts is None:
        counts = torch.empty((32, 8), dtype=torch.int64, device=codes.device)
    if workspace is None:
        workspace = torch.empty(torq_code_histogram_workspace_bytes(), dtype=torch.uint8, device=codes.device)
    _check(lib().torq_code_histogram(_dev(codes, torch.uint8, "codes"), M, d, _dev(counts, torch.int64, "counts"),
                                     _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)),
           "torq_code_histogram")
    return counts


def torq_intra_pair_scores(counts, lam: float):
    """counts: [32, 8] array-like of non-negative integers (host).  Returns (h [32], H [32, 32]) float64."""
    import numpy as np
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    if c.shape != (32, 8):
        raise ValueError("counts must be [32, 8]")
    h = np.empty((32,), np.float64)
    H = np.empty((32, 32), np.float64)
    _check(lib().torq_intra_pair_scores(c.ctypes.data_as(C.c_void_p), float(lam), h.ctypes.data_as(C.c_void_p),
                                        H.ctypes.data_as(C.c_void_p)), "torq_intra_pair_scores")
    return h, H


def torq_intra_best_angle(u, v, rest):
    """Appendix A.4 on the host.  Returns (theta, loss, number of distinct critical angles)."""
    import numpy as np
    u = np.ascontiguousarray(u, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    r = np.ascontiguousarray(rest, dtype=np.uint64)
    if u.ndim != 1 or u.shape != v.shape or r.shape != (8,):
        raise ValueError("u, v must be vectors of one length and rest 8 counts")
    th, lo, k = C.c_double(0.0), C.c_double(0.0), C.c_int64(0)
    _check(lib().torq_intra_best_angle(u.ctypes.data_as(C.c_void_p), v.ctypes.data_as(C.c_void_p), u.shape[0],
                                       r.ctypes.data_as(C.c_void_p), C.byref(th), C.byref(lo), C.byref(k)),
           "torq_intra_best_angle")
    return th.value, lo.value, k.value


def torq_calibrate_intra(X, max_iter: int, k_top: int, P: int, lam: float, eps: float):
    """Algorithm 2 on the host.  X: [n, 32] float32 sample blocks.  Returns (R_intra float32 [32, 32], losses)."""
    import numpy as np
    X = np.ascontiguousarray(X, dtype=np.float32)
    if X.ndim != 2 or X.shape[1] != 32:
        raise ValueError("X must be [n, 32]")
    R = np.empty((32, 32), np.float32)
    losses = np.zeros((max(int(max_iter), 0) + 1,), np.float64)
    k = C.c_int(0)
    _check(lib().torq_calibrate_intra(X.ctypes.data_as(C.c_void_p), X.shape[0], int(max_iter), int(k_top), int(P),
                                      float(lam), float(eps), R.ctypes.data_as(C.c_void_p),
                                      losses.ctypes.data_as(C.c_void_p), C.byref(k)), "torq_calibrate_intra")
    return R, losses[: k.value].copy()
