"""ctypes front end of the C oracle (oracle/torq_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg; never by the product package.  All arrays are
numpy, C-contiguous, on the host.  This module does argument marshalling only:
every number comes out of the C functions.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        # TORQ_ORACLE_LIB: the mutation test of the pins points this at a deliberately broken build
        path = os.environ.get("TORQ_ORACLE_LIB") or _build.LIB
        if path == _build.LIB and not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        i64, i32, f32, f64, vp = C.c_int64, C.c_int, C.c_float, C.c_double, C.c_void_p
        L.torq_o_bf16_to_f32.restype = f32
        L.torq_o_bf16_to_f32.argtypes = [C.c_uint16]
        L.torq_o_f32_to_bf16.restype = C.c_uint16
        L.torq_o_f32_to_bf16.argtypes = [f32]
        L.torq_o_rotate_inter.restype = None
        L.torq_o_rotate_inter.argtypes = [vp, i64, i32, i32, vp, vp]
        L.torq_o_rotate_intra.restype = None
        L.torq_o_rotate_intra.argtypes = [vp, i64, i32, vp, vp]
        L.torq_o_rotate.restype = None
        L.torq_o_rotate.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp]
        L.torq_o_rotate_inverse.restype = None
        L.torq_o_rotate_inverse.argtypes = [vp, i64, i32, i32, vp, vp, vp]
        L.torq_o_e8m0_from_amax.restype = C.c_uint8
        L.torq_o_e8m0_from_amax.argtypes = [f32]
        L.torq_o_e2m1_from_f32.restype = C.c_uint8
        L.torq_o_e2m1_from_f32.argtypes = [f32]
        L.torq_o_e2m1_value.restype = f32
        L.torq_o_e2m1_value.argtypes = [C.c_uint8]
        L.torq_o_quantize.restype = None
        L.torq_o_quantize.argtypes = [vp, i64, i32, vp, vp]
        L.torq_o_dequantize.restype = None
        L.torq_o_dequantize.argtypes = [vp, vp, i64, i32, vp]
        L.torq_o_e4m3_value.restype = f32
        L.torq_o_e4m3_value.argtypes = [C.c_uint8]
        L.torq_o_e4m3_from_f32.restype = C.c_uint8
        L.torq_o_e4m3_from_f32.argtypes = [f32]
        L.torq_o_quantize_mxint4.restype = None
        L.torq_o_quantize_mxint4.argtypes = [vp, i64, i32, vp, vp]
        L.torq_o_dequantize_mxint4.restype = None
        L.torq_o_dequantize_mxint4.argtypes = [vp, vp, i64, i32, vp]
        L.torq_o_quantize_nvfp4.restype = None
        L.torq_o_quantize_nvfp4.argtypes = [vp, i64, i32, f32, vp, vp]
        L.torq_o_dequantize_nvfp4.restype = None
        L.torq_o_dequantize_nvfp4.argtypes = [vp, vp, i64, i32, f32, vp]
        L.torq_o_rotate_quantize.restype = None
        L.torq_o_rotate_quantize.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp]
        L.torq_o_gemm.restype = None
        L.torq_o_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, vp]
        L.torq_o_gemm_sampled.restype = None
        L.torq_o_gemm_sampled.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp, vp, vp]
        L.torq_o_block_gram.restype = None
        L.torq_o_block_gram.argtypes = [vp, i64, i32, i32, vp]
        L.torq_o_block_gram_positions.restype = None
        L.torq_o_block_gram_positions.argtypes = [vp, i64, i32, i32, vp]
        L.torq_o_equalize.restype = i32
        L.torq_o_equalize.argtypes = [vp, i32, f64, vp]
        u64p = C.POINTER(C.c_uint64)
        L.torq_o_equalize_butterfly.restype = None
        L.torq_o_equalize_butterfly.argtypes = [vp, i32, vp, vp]
        L.torq_o_code_histogram.restype = None
        L.torq_o_code_histogram.argtypes = [vp, i64, i32, vp]
        L.torq_o_code_loss.restype = f64
        L.torq_o_code_loss.argtypes = [vp]
        L.torq_o_pair_scores.restype = None
        L.torq_o_pair_scores.argtypes = [vp, f64, vp, vp]
        L.torq_o_best_angle.restype = i64
        L.torq_o_best_angle.argtypes = [vp, vp, i64, vp, C.POINTER(f64), C.POINTER(f64)]
        L.torq_o_mag_code.restype = i32
        L.torq_o_mag_code.argtypes = [f64]
        L.torq_o_intra_rotation.restype = None
        L.torq_o_intra_rotation.argtypes = [vp, i64, i32, i32, i32, f64, f64, vp, vp, C.POINTER(i32)]
        L.torq_o_threads.restype = i32
        L.torq_o_threads.argtypes = []
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def bf16_to_f32(h):
    """h: uint16 array of bf16 patterns -> float32 array."""
    h = _arr(h, np.uint16)
    out = np.empty(h.shape, np.float32)
    L = lib()
    flat, o = h.reshape(-1), out.reshape(-1)
    for i in range(flat.size):
        o[i] = L.torq_o_bf16_to_f32(int(flat[i]))
    return out


def f32_to_bf16(f):
    f = _arr(f, np.float32)
    out = np.empty(f.shape, np.uint16)
    L = lib()
    flat, o = f.reshape(-1), out.reshape(-1)
    for i in range(flat.size):
        o[i] = L.torq_o_f32_to_bf16(float(flat[i]))
    return out


def e8m0_from_amax(amax: float) -> int:
    return int(lib().torq_o_e8m0_from_amax(np.float32(amax)))


def e2m1_from_f32(a: float) -> int:
    return int(lib().torq_o_e2m1_from_f32(np.float32(a)))


def e2m1_value(code: int) -> float:
    return float(lib().torq_o_e2m1_value(int(code)))


def _check_rot(d, G, R_inter, R_intra):
    assert d % 32 == 0 and (d // 32) % G == 0
    R_inter = _arr(R_inter, np.float32)
    R_intra = _arr(R_intra, np.float32)
    assert R_inter.shape == (G, G) and R_intra.shape == (32, 32)
    return R_inter, R_intra


def rotate_inter(x, G, R_inter):
    x = _arr(x, np.float64)
    M, d = x.shape
    R_inter = _arr(R_inter, np.float32)
    assert R_inter.shape == (G, G) and (d // 32) % G == 0
    y = np.empty_like(x)
    lib().torq_o_rotate_inter(_p(x), M, d, G, _p(R_inter), _p(y))
    return y


def rotate_intra(y, R_intra):
    y = _arr(y, np.float64)
    M, d = y.shape
    R_intra = _arr(R_intra, np.float32)
    assert R_intra.shape == (32, 32)
    z = np.empty_like(y)
    lib().torq_o_rotate_intra(_p(y), M, d, _p(R_intra), _p(z))
    return z


def rotate(x_bf16, G, R_inter, R_intra, want_f64=False):
    """x_bf16: uint16 [M, d].  Returns z fp32 [M, d] (and z fp64 if asked)."""
    x = _arr(x_bf16, np.uint16)
    M, d = x.shape
    R_inter, R_intra = _check_rot(d, G, R_inter, R_intra)
    z32 = np.empty((M, d), np.float32)
    z64 = np.empty((M, d), np.float64) if want_f64 else None
    lib().torq_o_rotate(_p(x), M, d, G, _p(R_inter), _p(R_intra), _p(z32), _p(z64))
    return (z32, z64) if want_f64 else z32


def rotate_inverse(z, G, R_inter, R_intra):
    z = _arr(z, np.float64)
    M, d = z.shape
    R_inter, R_intra = _check_rot(d, G, R_inter, R_intra)
    x = np.empty_like(z)
    lib().torq_o_rotate_inverse(_p(z), M, d, G, _p(R_inter), _p(R_intra), _p(x))
    return x


def quantize(z):
    """z fp32 [M, d] -> (codes uint8 [M, d/2], scales uint8 [M, d/32])."""
    z = _arr(z, np.float32)
    M, d = z.shape
    assert d % 32 == 0
    codes = np.empty((M, d // 2), np.uint8)
    scales = np.empty((M, d // 32), np.uint8)
    lib().torq_o_quantize(_p(z), M, d, _p(codes), _p(scales))
    return codes, scales


def e4m3_value(code: int) -> float:
    return float(lib().torq_o_e4m3_value(int(code)))


def e4m3_from_f32(t: float) -> int:
    return int(lib().torq_o_e4m3_from_f32(float(t)))


def quantize_mxint4(z):
    """z fp32 [M, d] -> (codes uint8 [M, d/2] two's-complement nibbles, scales uint8 [M, d/32] E8M0)."""
    z = _arr(z, np.float32)
    M, d = z.shape
    assert d % 32 == 0
    codes = np.empty((M, d // 2), np.uint8)
    scales = np.empty((M, d // 32), np.uint8)
    lib().torq_o_quantize_mxint4(_p(z), M, d, _p(codes), _p(scales))
    return codes, scales


def dequantize_mxint4(codes, scales):
    codes = _arr(codes, np.uint8)
    scales = _arr(scales, np.uint8)
    M, half = codes.shape
    out = np.empty((M, half * 2), np.float32)
    lib().torq_o_dequantize_mxint4(_p(codes), _p(scales), M, half * 2, _p(out))
    return out


def quantize_nvfp4(z, global_scale):
    """z fp32 [M, d] -> (codes uint8 [M, d/2] e2m1, scales uint8 [M, d/16] E4M3)."""
    z = _arr(z, np.float32)
    M, d = z.shape
    assert d % 16 == 0
    codes = np.empty((M, d // 2), np.uint8)
    scales = np.empty((M, d // 16), np.uint8)
    lib().torq_o_quantize_nvfp4(_p(z), M, d, float(global_scale), _p(codes), _p(scales))
    return codes, scales


def dequantize_nvfp4(codes, scales, global_scale):
    codes = _arr(codes, np.uint8)
    scales = _arr(scales, np.uint8)
    M, half = codes.shape
    out = np.empty((M, half * 2), np.float32)
    lib().torq_o_dequantize_nvfp4(_p(codes), _p(scales), M, half * 2, float(global_scale), _p(out))
    return out


def dequantize(codes, scales):
    codes = _arr(codes, np.uint8)
    scales = _arr(scales, np.uint8)
    M, half = codes.shape
    d = half * 2
    assert scales.shape == (M, d // 32)
    out = np.empty((M, d), np.float32)
    lib().torq_o_dequantize(_p(codes), _p(scales), M, d, _p(out))
    return out


def rotate_quantize(x_bf16, G, R_inter, R_intra):
    x = _arr(x_bf16, np.uint16)
    M, d = x.shape
    R_inter, R_intra = _check_rot(d, G, R_inter, R_intra)
    codes = np.empty((M, d // 2), np.uint8)
    scales = np.empty((M, d // 32), np.uint8)
    lib().torq_o_rotate_quantize(_p(x), M, d, G, _p(R_inter), _p(R_intra), _p(codes), _p(scales))
    return codes, scales


def gemm(A_q, A_s, W_q, W_s, want_f64=False):
    """Returns bf16 patterns uint16 [M, N] (and the unrounded fp64 if asked)."""
    A_q, A_s = _arr(A_q, np.uint8), _arr(A_s, np.uint8)
    W_q, W_s = _arr(W_q, np.uint8), _arr(W_s, np.uint8)
    M, half = A_q.shape
    N = W_q.shape[0]
    d = half * 2
    assert W_q.shape == (N, half) and A_s.shape == (M, d // 32) and W_s.shape == (N, d // 32)
    out = np.empty((M, N), np.uint16)
    o64 = np.empty((M, N), np.float64) if want_f64 else None
    lib().torq_o_gemm(_p(A_q), _p(A_s), _p(W_q), _p(W_s), M, N, d, _p(out), _p(o64))
    return (out, o64) if want_f64 else out


def gemm_sampled(A_q, A_s, W_q, W_s, ms, ns, want_f64=False):
    A_q, A_s = _arr(A_q, np.uint8), _arr(A_s, np.uint8)
    W_q, W_s = _arr(W_q, np.uint8), _arr(W_s, np.uint8)
    d = A_q.shape[1] * 2
    ms, ns = _arr(ms, np.int64), _arr(ns, np.int64)
    assert ms.shape == ns.shape and ms.ndim == 1
    assert ms.size == 0 or (ms.min() >= 0 and ms.max() < A_q.shape[0])
    assert ns.size == 0 or (ns.min() >= 0 and ns.max() < W_q.shape[0])
    out = np.empty(ms.shape, np.uint16)
    o64 = np.empty(ms.shape, np.float64) if want_f64 else None
    lib().torq_o_gemm_sampled(_p(A_q), _p(A_s), _p(W_q), _p(W_s), d, ms.size,
                              _p(ms), _p(ns), _p(out), _p(o64))
    return (out, o64) if want_f64 else out


def block_gram(x_bf16, G):
    """x_bf16: uint16 [M, d] -> Sigma float64 [G, G], the mean Gram matrix of the runs of G blocks."""
    x = _arr(x_bf16, np.uint16)
    M, d = x.shape
    assert d % 32 == 0 and (d // 32) % G == 0
    S = np.empty((G, G), np.float64)
    lib().torq_o_block_gram(_p(x), M, d, G, _p(S))
    return S


def block_gram_positions(x_bf16, G):
    """x_bf16: uint16 [M, d] -> float64 [32, G, G]: the Gram matrix of the runs of G blocks kept apart by
    the position inside a block (Sigma_k of Theorem 4.1); sums over axis 0 to block_gram."""
    x = _arr(x_bf16, np.uint16)
    M, d = x.shape
    assert d % 32 == 0 and (d // 32) % G == 0
    S = np.empty((32, G, G), np.float64)
    lib().torq_o_block_gram_positions(_p(x), M, d, G, _p(S))
    return S


def equalize(Sigma, eps=0.0):
    """Corrected Algorithm 1.  Returns (R, Sigma_after, steps)."""
    S = np.array(Sigma, dtype=np.float64, order="C", copy=True)
    B = S.shape[0]
    assert S.shape == (B, B)
    R = np.empty((B, B), np.float64)
    steps = lib().torq_o_equalize(_p(S), B, float(eps), _p(R))
    return R, S, steps


def equalize_butterfly(Sigma):
    """Butterfly variance equaliser.  Returns (R [B, B], R Sigma R^T, tangents [log2 B, B/2])."""
    S = _arr(Sigma, np.float64).copy()
    B = S.shape[0]
    assert S.shape == (B, B) and B >= 2 and (B & (B - 1)) == 0
    R = np.empty((B, B), np.float64)
    L = B.bit_length() - 1
    tangents = np.empty((L, B // 2), np.float64)
    lib().torq_o_equalize_butterfly(_p(S), B, _p(R), _p(tangents))
    return R, S, tangents


def code_histogram(codes, d):
    """codes: uint8 [M, d/2] -> uint64 [32, 8]: occupancy of the 8 magnitude codewords per in-block position."""
    c = _arr(codes, np.uint8)
    M = c.shape[0]
    assert c.shape == (M, d // 2)
    out = np.empty((32, 8), np.uint64)
    lib().torq_o_code_histogram(_p(c), M, d, _p(out))
    return out


def code_loss(n):
    n = _arr(n, np.uint64)
    assert n.shape == (8,)
    return float(lib().torq_o_code_loss(_p(n)))


def pair_scores(counts, lam):
    cts = _arr(counts, np.uint64)
    assert cts.shape == (32, 8)
    h = np.empty((32,), np.float64)
    H = np.empty((32, 32), np.float64)
    lib().torq_o_pair_scores(_p(cts), float(lam), _p(h), _p(H))
    return h, H


def best_angle(u, v, rest):
    """Appendix A.4 for one column pair.  Returns (theta, loss, intervals)."""
    u = _arr(u, np.float64)
    v = _arr(v, np.float64)
    rest = _arr(rest, np.uint64)
    assert u.shape == v.shape and u.ndim == 1 and rest.shape == (8,)
    th, lo = C.c_double(0.0), C.c_double(0.0)
    k = lib().torq_o_best_angle(_p(u), _p(v), u.shape[0], _p(rest), C.byref(th), C.byref(lo))
    return th.value, lo.value, int(k)


def mag_code(a: float) -> int:
    return int(lib().torq_o_mag_code(float(a)))


def intra_rotation(X, max_iter, k_top, P, lam, eps):
    """Algorithm 2 on sample blocks X [n, 32].  Returns (R_intra [32, 32], losses per evaluation)."""
    X = _arr(X, np.float64)
    n = X.shape[0]
    assert X.shape == (n, 32)
    R = np.empty((32, 32), np.float64)
    losses = np.zeros((max_iter + 1,), np.float64)
    k = C.c_int32(0)
    lib().torq_o_intra_rotation(_p(X), n, max_iter, k_top, P, float(lam), float(eps), _p(R), _p(losses), C.byref(k))
    return R, losses[: k.value].copy()


def threads() -> int:
    return int(lib().torq_o_threads())
