"""Pins for the oracle's MXINT4 and NVFP4 quantisers (Section 6, "Generalizability to Other
Formats"): the paper names the formats without defining them, so the pins are the public facts of
the encodings (OCP FP8 E4M3 bit layout, two's-complement nibbles), hand-worked roundings including
ties and saturation, a library conversion on the in-range grid, brute-force nearest search, the
half-step error bound and the scale invariances.
"""
import numpy as np
import pytest
import torch

import oracle

E2M1 = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6], np.float64)


def _unpack(codes):
    codes = np.asarray(codes, np.uint8)
    out = np.empty((codes.shape[0], codes.shape[1] * 2), np.uint8)
    out[:, 0::2] = codes & 15
    out[:, 1::2] = codes >> 4
    return out


# ------------------------------------------------------------------ E4M3 --

def test_e4m3_values_of_the_bit_layout():
    assert oracle.e4m3_value(0x00) == 0.0
    assert oracle.e4m3_value(0x01) == 2.0 ** -9             # smallest subnormal
    assert oracle.e4m3_value(0x07) == 7 * 2.0 ** -9
    assert oracle.e4m3_value(0x08) == 2.0 ** -6             # smallest normal
    assert oracle.e4m3_value(0x38) == 1.0
    assert oracle.e4m3_value(0x39) == 1.125
    assert oracle.e4m3_value(0x40) == 2.0
    assert oracle.e4m3_value(0x77) == 240.0
    assert oracle.e4m3_value(0x7E) == 448.0                 # largest: S.1111.110
    assert oracle.e4m3_value(0xB8) == -1.0
    vals = [oracle.e4m3_value(c) for c in range(0x7F)]
    assert all(b > a for a, b in zip(vals, vals[1:]))       # strictly increasing in the code


def test_e4m3_rounding_hand_worked():
    f = oracle.e4m3_from_f32
    assert f(1.0) == 0x38 and f(448.0) == 0x7E and f(0.0) == 0x00
    assert f(500.0) == 0x7E and f(1e30) == 0x7E             # saturates, no infinity
    assert f(464.0) == 0x7E                                 # past the last midpoint there is nothing to round to
    assert f(2.0 ** -10) == 0x00                            # tie 0 / 2^-9 -> even code 0
    assert f(3 * 2.0 ** -10) == 0x02                        # tie 0x01 / 0x02 -> even
    assert f(2.0 ** -10 * 1.001) == 0x01
    assert f(1.0625) == 0x38                                # tie 1.0 / 1.125 -> even mantissa
    assert f(1.1875) == 0x3A                                # tie 1.125 / 1.25 -> even mantissa
    assert f(1.0626) == 0x39
    assert f(15.5 * 2.0 ** -10) == 0x08                     # tie last subnormal 7/8 / first normal -> even (0x08)
    for c in range(0x7F):
        assert f(oracle.e4m3_value(c)) == c                 # every value is its own nearest


def test_e4m3_rounding_agrees_with_the_library_conversion_in_range():
    grid = np.concatenate([np.linspace(0, 2.0 ** -5, 4097), np.linspace(0, 448, 28673), np.geomspace(1e-4, 448, 5000)])
    grid = grid.astype(np.float32)
    lib = torch.from_numpy(grid).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = np.array([oracle.e4m3_from_f32(float(t)) for t in grid], np.uint8)
    assert np.array_equal(mine, lib)


# ------------------------------------------------------------------ MXINT4 --

def test_mxint4_hand_worked_block():
    z = np.zeros((1, 32), np.float32)
    z[0, :12] = [7.9, 2.5, 3.5, -0.5, -7.6, 0.49, -2.5, 1.5, 6.5, -6.5, 7.5, 4.0]
    codes, scales = oracle.quantize_mxint4(z)
    assert scales[0, 0] == 127                               # amax 7.9 in [4, 8): scale 1
    want = [7, 2, 4, 0, -7, 0, -2, 2, 6, -6, 7, 4]            # ties to even; 7.9, 7.5 -> 8 -> clamped to 7
    got = _unpack(codes)[0, :12].astype(np.int8)
    got = np.where(got >= 8, got - 16, got)
    assert got.tolist() == want
    assert np.all(_unpack(codes)[0, 12:] == 0)
    z2 = z * 2.0 ** -20
    c2, s2 = oracle.quantize_mxint4(z2)
    assert np.array_equal(c2, codes) and s2[0, 0] == 107     # power-of-two scaling moves only the scale


def test_mxint4_error_bound_and_nearest():
    rng = np.random.default_rng(0)
    z = (rng.standard_t(3, size=(64, 256)) * np.exp(rng.normal(size=(64, 1)) * 3)).astype(np.float32)
    codes, scales = oracle.quantize_mxint4(z)
    zh = oracle.dequantize_mxint4(codes, scales)
    step = np.exp2(scales.astype(np.float64) - 127).repeat(32, axis=1)
    a = z.astype(np.float64) / step
    err = np.abs(z - zh) / step
    inside = np.abs(a) <= 7.0
    assert np.all(err[inside] <= 0.5 + 1e-9)                 # half a step wherever nothing is clamped
    assert np.all(err[~inside] < 1.0 + 1e-9) and np.all(np.abs(a) < 8.0)
    ints = np.where(_unpack(codes) >= 8, _unpack(codes).astype(np.int16) - 16, _unpack(codes).astype(np.int16))
    assert ints.min() >= -7 and ints.max() <= 7              # -8 is never produced
    # brute force: no integer in [-7, 7] is nearer
    best = np.abs(a[..., None] - np.arange(-7, 8)[None, None, :]).min(axis=2)
    assert np.all(np.abs(a - ints) <= best + 1e-12)
    assert np.array_equal(oracle.quantize(z)[1], scales)     # the shared scale is the MXFP4 one


# ------------------------------------------------------------------ NVFP4 --

def test_nvfp4_hand_worked_blocks():
    z = np.zeros((1, 64), np.float32)
    z[0, 0:4] = [6.0, -3.0, 0.26, 1.25]            # amax 6   -> t = 1    -> 0x38, S = 1
    z[0, 16:20] = [3.0, 1.5, -0.75, 0.1]           # amax 3   -> t = 0.5  -> 0x30, S = 0.5
    z[0, 32:35] = [448.0 * 6 * 4, 5.0, -1.0]       # t = 1792 -> saturates to 448 (0x7E); a = 24 -> code 7
    codes, scales = oracle.quantize_nvfp4(z, 1.0)
    assert scales[0].tolist() == [0x38, 0x30, 0x7E, 0x00]
    u = _unpack(codes)[0]
    assert u[0:4].tolist() == [7, 8 | 5, 1, 2]      # 0.26 -> 0.5; tie 1.25 -> 1 (even code)
    assert u[16:20].tolist() == [7, 5, 8 | 3, 0]    # /0.5: 6, 3, -1.5, 0.2 -> 0
    assert u[32:35].tolist() == [7, 0, 8]           # 5/448 and -1/448 vanish; the sign survives
    assert np.all(u[48:] == 0)                      # the all-zero block: scale byte 0, codes 0
    zh = oracle.dequantize_nvfp4(codes, scales, 1.0)
    assert zh[0, 0] == 6.0 and zh[0, 16] == 3.0 and zh[0, 32] == 6 * 448.0 and zh[0, 18] == -0.75


def test_nvfp4_scale_rounding_uses_e4m3_and_the_global_scale():
    z = np.zeros((1, 16), np.float32)
    z[0, 0] = 6.0 * 1.0625                          # t = 1.0625: tie between 1.0 and 1.125 -> 1.0
    assert oracle.quantize_nvfp4(z, 1.0)[1][0, 0] == 0x38
    z[0, 0] = 6.0 * 1.07
    assert oracle.quantize_nvfp4(z, 1.0)[1][0, 0] == 0x39
    # the same data against a global scale of 1/64 needs a 64 times larger block scale
    assert oracle.quantize_nvfp4(z, 2.0 ** -6)[1][0, 0] == 0x39 + (6 << 3)
    # power-of-two invariance: data and global scale move together, codes and scale bytes stay
    rng = np.random.default_rng(3)
    zz = rng.standard_normal((8, 128)).astype(np.float32)
    c1, s1 = oracle.quantize_nvfp4(zz, 0.01)
    c2, s2 = oracle.quantize_nvfp4(zz * 1024, 0.01 * 1024)
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2)


def test_nvfp4_error_bound_and_nearest():
    rng = np.random.default_rng(1)
    z = (rng.standard_t(3, size=(32, 256)) * np.exp(rng.normal(size=(32, 1)))).astype(np.float32)
    gs = float(np.abs(z).max() / (448 * 6))        # the usual choice: the largest block scale is 448
    codes, scales = oracle.quantize_nvfp4(z, gs)
    zh = oracle.dequantize_nvfp4(codes, scales, gs)
    S = (np.array([oracle.e4m3_value(int(b)) for b in scales.reshape(-1)]).reshape(scales.shape) * np.float32(gs)).repeat(16, axis=1)
    ok = S > 0
    a = np.zeros_like(S)
    a[ok] = z[ok].astype(np.float64) / S[ok]
    # the block scale is amax / 6 rounded to 3 mantissa bits: the largest element lands within 1/16 of 6
    amax_a = np.abs(a).reshape(32, 16, 16).max(axis=2)
    nz = np.abs(z).reshape(32, 16, 16).max(axis=2) > 0
    assert np.all(amax_a[nz] <= 6.0 * (1 + 1 / 16) + 1e-6) and np.all(amax_a[nz] >= 6.0 * (1 - 1 / 16) - 1e-6)
    mags = _unpack(codes) & 7
    best = np.abs(np.abs(a)[..., None] - E2M1[None, None, :]).min(axis=2)
    assert np.all(np.abs(np.abs(a) - E2M1[mags]) <= best + 1e-6)                 # nearest codeword
    half_step = np.where(np.abs(a) <= 2, 0.25, np.where(np.abs(a) <= 4, 0.5, 1.0))
    inside = np.abs(a) <= 6
    assert np.all((np.abs(z - zh) / np.where(ok, S, 1))[inside & ok] <= half_step[inside & ok] + 1e-6)
    assert np.array_equal((_unpack(codes) >> 3).astype(bool), np.signbit(z))     # signs are copied
