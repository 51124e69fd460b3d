"""Pins for the oracle's reference GEMM (Algorithm 3 "Return": y = W' vec(Zhat))
and for the whole chain rotate -> quantise -> linear layer.
"""
import numpy as np
import torch

from paper_2605_19561_amd import synth

MAG = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def _decode(codes, scales):
    """numpy decode, written independently of the oracle: [M, d] float64"""
    lo = codes & 15
    hi = codes >> 4
    c = np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1)
    v = MAG[c & 7] * np.where(c & 8, -1.0, 1.0)
    return v * np.repeat(2.0 ** (scales.astype(np.float64) - 127), 32, axis=1)


def _bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_integer_special_case_equals_integer_matmul(oracle):
    # all scale bytes 127 and codes restricted to {0, +-1, +-2, +-4}: the GEMM is an
    # integer matrix product, which numpy computes exactly in int64
    rng = np.random.default_rng(0)
    M, N, d = 7, 9, 256
    table = {0: 0, 2: 1, 4: 2, 6: 4, 10: -1, 12: -2, 14: -4}
    keys = np.array(list(table.keys()), np.uint8)
    ca = rng.choice(keys, size=(M, d))
    cw = rng.choice(keys, size=(N, d))
    A_q = (ca[:, 0::2] | (ca[:, 1::2] << 4)).astype(np.uint8)
    W_q = (cw[:, 0::2] | (cw[:, 1::2] << 4)).astype(np.uint8)
    A_s = np.full((M, d // 32), 127, np.uint8)
    W_s = np.full((N, d // 32), 127, np.uint8)
    out, o64 = oracle.gemm(A_q, A_s, W_q, W_s, want_f64=True)
    ia = np.vectorize(table.get)(ca).astype(np.int64)
    iw = np.vectorize(table.get)(cw).astype(np.int64)
    want = ia @ iw.T
    assert np.array_equal(o64, want.astype(np.float64))
    assert np.array_equal(_bf16_to_f64(out), torch.from_numpy(want.astype(np.float32)).to(torch.bfloat16)
                          .to(torch.float64).numpy())


def test_scales_shift_the_result_by_powers_of_two(oracle):
    rng = np.random.default_rng(1)
    M, N, d = 3, 5, 64
    A_q = rng.integers(0, 256, size=(M, d // 2), dtype=np.uint8)
    W_q = rng.integers(0, 256, size=(N, d // 2), dtype=np.uint8)
    A_s = np.full((M, 2), 127, np.uint8)
    W_s = np.full((N, 2), 127, np.uint8)
    base = oracle.gemm(A_q, A_s, W_q, W_s, want_f64=True)[1]
    A_s2 = A_s.copy(); A_s2[:, :] = 130
    W_s2 = W_s.copy(); W_s2[:, :] = 120
    moved = oracle.gemm(A_q, A_s2, W_q, W_s2, want_f64=True)[1]
    assert np.array_equal(moved, base * 2.0 ** (3 - 7))
    # only block 1 of A scaled: only that block's partial sum moves
    A_s3 = A_s.copy(); A_s3[:, 1] = 128
    part0 = _decode(A_q, A_s)[:, :32] @ _decode(W_q, W_s)[:, :32].T
    part1 = _decode(A_q, A_s)[:, 32:] @ _decode(W_q, W_s)[:, 32:].T
    assert np.array_equal(oracle.gemm(A_q, A_s3, W_q, W_s, want_f64=True)[1], part0 + 2 * part1)


def test_single_block_and_single_output(oracle):
    # d = 32, M = N = 1, hand-worked: a = (6, -0.5, 0, ...), w = (1.5, 4, ...) at scales 2^1 and 2^-2
    a_codes = np.zeros(32, np.uint8); w_codes = np.zeros(32, np.uint8)
    a_codes[0], a_codes[1] = 7, 9          # +6, -0.5
    w_codes[0], w_codes[1] = 3, 6          # +1.5, +4
    A_q = (a_codes[0::2] | (a_codes[1::2] << 4)).reshape(1, 16)
    W_q = (w_codes[0::2] | (w_codes[1::2] << 4)).reshape(1, 16)
    out, o64 = oracle.gemm(A_q, np.array([[128]], np.uint8), W_q, np.array([[125]], np.uint8), want_f64=True)
    # (6*2)(1.5/4) + (-0.5*2)(4/4) = 4.5 - 1 = 3.5
    assert o64[0, 0] == 3.5
    assert out[0, 0] == 0x4060              # 3.5 in bf16


def test_random_codes_match_numpy_decode_and_matmul(oracle):
    rng = np.random.default_rng(2)
    M, N, d = 11, 13, 512
    A_q = rng.integers(0, 256, size=(M, d // 2), dtype=np.uint8)
    W_q = rng.integers(0, 256, size=(N, d // 2), dtype=np.uint8)
    A_s = rng.integers(120, 134, size=(M, d // 32), dtype=np.uint8)
    W_s = rng.integers(120, 134, size=(N, d // 32), dtype=np.uint8)
    out, o64 = oracle.gemm(A_q, A_s, W_q, W_s, want_f64=True)
    a, w = _decode(A_q, A_s), _decode(W_q, W_s)
    assert np.array_equal(oracle.dequantize(A_q, A_s).astype(np.float64), a)
    # every product is a multiple of 2^-2 2^(sa+sw-254) of magnitude <= 36 2^(sa+sw-254); with the
    # scale bytes within 14 of each other a 512-term sum spans < 8 + 28 + 9 = 45 bits: the double
    # result is exact, so any summation order agrees bit for bit
    assert np.array_equal(o64, a @ w.T)
    ms = np.array([0, 10, 3, 3], np.int64); ns = np.array([12, 0, 7, 7], np.int64)
    sb, s64 = oracle.gemm_sampled(A_q, A_s, W_q, W_s, ms, ns, want_f64=True)
    assert np.array_equal(s64, o64[ms, ns]) and np.array_equal(sb, out[ms, ns])
    ref_bf16 = synth.bf16_bits(torch.from_numpy(o64.astype(np.float32)).to(torch.bfloat16))
    assert np.array_equal(out, ref_bf16)


def test_unquantised_chain_is_plain_linear_layer(oracle):
    # Section 5 / Section 5.2: with the inverse rotation folded into the weights the layer
    # output is unchanged under full precision: rot(W) rot(x) = W x
    G = 16
    d = 32 * G * 2
    Ri, Ra = synth.rotations(G, seed=3)
    x = synth.activations(5, d, seed=1)
    w = synth.weights(7, d, seed=2)
    zx = oracle.rotate(synth.bf16_bits(x), G, Ri, Ra, want_f64=True)[1]
    zw = oracle.rotate(synth.bf16_bits(w), G, Ri, Ra, want_f64=True)[1]
    plain = x.to(torch.float64).numpy() @ w.to(torch.float64).numpy().T
    assert np.abs(zx @ zw.T - plain).max() < 1e-5 * np.abs(plain).max()


def test_quantised_chain_error_is_lower_with_rotation(oracle):
    # direction of Table 2 (component ablation): on heavy-tailed inputs with outlier channels,
    # rotating before MXFP4 quantisation lowers the layer's output error.  No value to hit.
    G = 128
    d = 4096
    x = synth.workload_activations("tiny")
    w = synth.workload_weights("tiny", N=256)
    Ri, Ra = synth.rotations(G)
    xb, wb = synth.bf16_bits(x), synth.bf16_bits(w)
    plain = x.to(torch.float64).numpy() @ w.to(torch.float64).numpy().T
    eye_i, eye_a = np.eye(G, dtype=np.float32), np.eye(32, dtype=np.float32)

    def chain(Ri_, Ra_):
        aq, as_ = oracle.rotate_quantize(xb, G, Ri_, Ra_)
        wq, ws = oracle.rotate_quantize(wb, G, Ri_, Ra_)
        o = oracle.gemm(aq, as_, wq, ws, want_f64=True)[1]
        return np.linalg.norm(o - plain) / np.linalg.norm(plain), aq

    e_none, q_none = chain(eye_i, eye_a)
    e_both, q_both = chain(Ri, Ra)
    assert e_both < 0.95 * e_none
    assert e_both < 0.25
    # Section 1: without rotation most small elements are zeroed; fewer zero codes after rotation
    zeros = lambda q: np.mean(((q & 7) == 0)) / 2 + np.mean((((q >> 4) & 7) == 0)) / 2
    assert zeros(q_both) < zeros(q_none)
