"""Pins for the oracle's number formats: bf16, E8M0 scale, e2m1 rounding, packing.

Each check compares the C oracle with something that is not the oracle: values
worked by hand from the paper's definition (tests/golden), torch's own bf16
conversion, brute-force nearest-codeword search, error bounds of the codebook.
"""
import os

import numpy as np
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")
CODEBOOK_MAG = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]   # Section 4, Eq. 1


def _read_cases(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            a, b = line.split()
            rows.append((float.fromhex(a) if "0x" in a else float(a), int(b)))
    return rows


# ---------------------------------------------------------------- bf16 ------

def test_bf16_roundtrip_exhaustive(oracle):
    h = np.arange(65536, dtype=np.uint16)
    f = oracle.bf16_to_f32(h)
    # closed form: the pattern is the top half of the binary32 pattern
    isnan = np.isnan(f)      # a signalling NaN may be quietened on its way through ctypes
    assert np.array_equal(f.view(np.uint32)[~isnan], (h.astype(np.uint32) << 16)[~isnan])
    assert isnan.sum() == 2 * 127            # exponent all ones, mantissa non-zero, both signs
    back = oracle.f32_to_bf16(f)
    assert np.array_equal(back[~isnan], h[~isnan])
    assert np.all(np.isnan(oracle.bf16_to_f32(back[isnan])))


def test_bf16_narrowing_matches_torch_and_hand_cases(oracle):
    # hand cases: ties go to the even pattern
    cases = {
        1.0: 0x3F80,
        1.0 + 2.0 ** -8: 0x3F80,          # exactly half way between 0x3F80 and 0x3F81 -> even
        1.0 + 3 * 2.0 ** -8: 0x3F82,      # half way between 0x3F81 and 0x3F82 -> even
        1.0 + 2.0 ** -8 + 2.0 ** -20: 0x3F81,
        -2.5: 0xC020,
        3.3895313892515355e38: 0x7F7F,    # largest finite bf16
    }
    for v, want in cases.items():
        assert int(oracle.f32_to_bf16(np.float32(v)).reshape(-1)[0]) == want, v
    # overflow to infinity when rounding up from the largest finite fp32
    assert int(oracle.f32_to_bf16(np.float32(3.4028234e38)).reshape(-1)[0]) == 0x7F80
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32)
    f = bits.view(np.float32)
    f = f[np.isfinite(f)]
    ours = oracle.f32_to_bf16(f)
    ref = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)


# ---------------------------------------------------------------- E8M0 ------

def test_e8m0_hand_worked(oracle):
    for amax, want in _read_cases("e8m0_cases.txt"):
        assert oracle.e8m0_from_amax(amax) == want, (amax, want)


def test_e8m0_puts_normalised_max_in_4_to_8(oracle):
    # property of the rule scale = 2^(floor(log2 amax) - 2)
    rng = np.random.default_rng(3)
    amax = np.exp(rng.uniform(np.log(1e-30), np.log(1e30), size=2000)).astype(np.float32)
    for a in amax:
        byte = oracle.e8m0_from_amax(a)
        norm = float(a) / 2.0 ** (byte - 127)
        assert 4.0 <= norm < 8.0, (a, byte, norm)
        # agrees with the textbook formula floor(log2) computed by frexp
        m, e = np.frexp(np.float64(a))        # a = m 2^e, m in [0.5, 1)
        assert byte == (e - 1) - 2 + 127


# ---------------------------------------------------------------- e2m1 ------

def test_e2m1_hand_worked(oracle):
    for a, want in _read_cases("e2m1_cases.txt"):
        assert oracle.e2m1_from_f32(a) == want, (a, want)


def test_e2m1_values(oracle):
    for i, m in enumerate(CODEBOOK_MAG):
        assert oracle.e2m1_value(i) == m
        assert oracle.e2m1_value(8 | i) == -m


def test_e2m1_is_nearest_codeword_bruteforce(oracle):
    values = [s * m for m in CODEBOOK_MAG for s in (1.0, -1.0)]
    grid = np.arange(-8 * 64, 8 * 64 + 1) / 64.0            # steps of 1/64 in [-8, 8]
    rng = np.random.default_rng(11)
    extra = rng.uniform(-8, 8, size=4000)
    for a in np.concatenate([grid, extra]).astype(np.float32):
        code = oracle.e2m1_from_f32(a)
        got = oracle.e2m1_value(code)
        best = min(abs(float(a) - v) for v in values)
        assert abs(float(a) - got) == best, (a, code, got)   # either tie neighbour is nearest
        if a != 0:
            assert (code >> 3) == (1 if a < 0 else 0)


def test_e2m1_error_bounds(oracle):
    # half the local codebook step: 0.25 on [0,2], 0.5 on [2,4], 1 on [4,6]; < 2 in (6, 8)
    for a in np.linspace(0, 8, 4097, dtype=np.float32)[:-1]:
        err = abs(float(a) - oracle.e2m1_value(oracle.e2m1_from_f32(a)))
        if a <= 2:
            assert err <= 0.25
        elif a <= 4:
            assert err <= 0.5
        elif a <= 6:
            assert err <= 1.0
        else:
            assert err < 2.0


# ------------------------------------------------------- quantise / pack ----

def test_pack_roundtrip_all_bytes(oracle):
    # a block whose codes we control: values are codebook entries times 2^0 with amax 6
    # -> scale byte 127, every value is its own code.  All 256 (lo, hi) nibble pairs.
    vals = np.array([oracle.e2m1_value(c) for c in range(16)], np.float32)
    rows = []
    for byte in range(256):
        lo, hi = byte & 15, byte >> 4
        blk = np.zeros(32, np.float32)
        blk[0], blk[1] = vals[lo], vals[hi]
        blk[31] = 6.0                                   # pins amax -> byte 127
        rows.append(blk)
    z = np.stack(rows)
    codes, scales = oracle.quantize(z)
    assert np.all(scales == 127)
    assert np.array_equal(codes[:, 0], np.arange(256, dtype=np.uint8))
    assert np.all(codes[:, 15] == (7 << 4))             # element 31 -> high nibble of byte 15
    assert np.array_equal(oracle.dequantize(codes, scales), z)


def test_quantize_zero_block_and_negative_zero(oracle):
    z = np.zeros((1, 64), np.float32)
    z[0, 3] = -0.0
    z[0, 32:] = 1e-3
    z[0, 40] = -1e-5
    codes, scales = oracle.quantize(z)
    assert scales[0, 0] == 0
    # -0.0 keeps its sign bit: element 3 is the high nibble of byte 1
    assert codes[0, 1] == 0x80 and codes[0, 0] == 0
    # block 1: amax 1e-3 -> floor(log2) = -10 -> byte 115 ; 1e-3 / 2^-12 = 4.096 -> code 6
    assert scales[0, 1] == 115
    assert codes[0, 16] == 0x66
    # -1e-5 / 2^-12 = -0.04 -> -0 (code 8); element 40 is the low nibble of byte 20
    assert codes[0, 20] == 0x68


def test_quantize_saturation_and_half_ulp_bound(oracle):
    rng = np.random.default_rng(5)
    z = (rng.standard_t(3, size=(64, 1024)) * np.exp(rng.normal(size=(64, 1)) * 3)).astype(np.float32)
    codes, scales = oracle.quantize(z)
    zh = oracle.dequantize(codes, scales)
    s = np.repeat(2.0 ** (scales.astype(np.float64) - 127), 32, axis=1)
    a = np.abs(z.astype(np.float64)) / s
    assert a.max() < 8.0
    err = np.abs(z.astype(np.float64) - zh) / s
    assert np.all(err[a <= 2] <= 0.25)
    assert np.all(err[(a > 2) & (a <= 4)] <= 0.5)
    assert np.all(err[(a > 4) & (a <= 6)] <= 1.0)
    sat = a > 6
    assert sat.any() and np.all(err[sat] < 2.0)          # saturation band (6, 8) -> 6
    assert np.all(np.abs(zh[sat]) == 6.0 * s[sat])
    # every block's largest element uses one of the top two codewords (4 or 6)
    top = np.abs(zh.reshape(64, -1, 32)).max(axis=2) / 2.0 ** (scales.astype(np.float64) - 127)
    assert np.all((top == 4.0) | (top == 6.0))


def test_quantize_scale_invariance_by_powers_of_two(oracle):
    # Eq. 1: multiplying a block by 2^k moves only the shared exponent
    rng = np.random.default_rng(9)
    z = rng.standard_normal((8, 256)).astype(np.float32)
    c0, s0 = oracle.quantize(z)
    c1, s1 = oracle.quantize(z * np.float32(2.0 ** 11))
    assert np.array_equal(c0, c1) and np.array_equal(s1.astype(int), s0.astype(int) + 11)
