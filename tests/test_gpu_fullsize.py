"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot run these shapes whole in seconds, but every output row of
rotate+quantise depends on one input row only and every GEMM output on one row
of each operand, so sampled rows / outputs are recomputed exactly by the oracle.
Inputs are seeded synthetic tensors generated on the device (same recipes as the
benchmark); the sampled rows are copied to the host and handed to the oracle.
"""
import numpy as np
import pytest
import torch

from paper_2605_19561_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def tq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_19561_amd import binding
    binding.lib()
    return binding


def _np(t):
    return t.detach().cpu().numpy()


def _bf16_bits_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _check_rows(oracle, tq, rot, x, rows, G, Ri, Ra):
    """rotate and rotate+quantise on sampled rows against the oracle"""
    d = x.shape[1]
    xs = x[rows].contiguous()
    xb = synth.bf16_bits(xs)
    z_ref = oracle.rotate(xb, G, Ri, Ra)
    want_c, want_s = oracle.quantize(z_ref)
    return xs, z_ref, want_c, want_s, d


ROT_FULL = [
    ("llama3_70b_up", None),                       # [8192, 8192], G = 128: the benchmark's step
    ("qwen3_32b", None),                           # [4096, 5120], G = 80, per-token log-normal scale
    ("llama3_70b_down", 2048),                     # d = 28672, G = 128 (rows trimmed: generation time)
    ("llama3_8b_prefill", None),                   # [2048, 4096], G = 128
    ("llama3_8b_down", None),                      # [2048, 14336], G = 112: half-empty last tile of the 32x32 kernel
    ("qwen3_32b_down", 2048),                      # d = 25600, G = 80, ten groups per row (rows trimmed)
]


@pytest.mark.parametrize("name,M", ROT_FULL)
def test_rotate_quantize_full_size_sampled_rows(tq, oracle, name, M):
    _rotate_quantize_checks(tq, oracle, synth.workload_activations(name, device=DEV, M=M))


# The three-buffer kernel takes G = 80 ... 128 from 12288 token-groups on; below that G = 128, 112 and 80 quantise
# in batches of one token-group up to 256 token-groups and from 3072 on, in batches of two between (G = 64: batches
# of one from 3072 to 16384 token-groups).  The benchmark shapes above cover the three-buffer kernel at G = 128 and
# 80, batches of one at G = 128, 112 and 80 and batches of two at G = 128 (the fp32 values they are compared with
# come from batches of two every time): here G = 112 and 96 above the three-buffer threshold, G = 128 one
# token-group above and one below it (a last batch of one token-group either way), both sides of 256 and of 3072
# token-groups at G = 128, batches of two at G = 80 and 112, and G = 64 (d = 2048) on its last size with batches
# of one and its first with batches of two again.
@pytest.mark.parametrize("M,d", [(4096, 14336), (4096, 9216), (12289, 4096), (12287, 4096), (16384, 2048), (16385, 2048),
                                 (256, 4096), (257, 4096), (3071, 4096), (3072, 4096), (1000, 5120), (300, 14336)])
def test_rotate_quantize_around_the_three_buffer_threshold(tq, oracle, M, d):
    x = synth.activations(M, d, nu=3.0, outliers=round(0.005 * d), outlier_scale=50.0, seed=4242 + d, device=DEV)
    _rotate_quantize_checks(tq, oracle, x)


def _rotate_quantize_checks(tq, oracle, x):
    M, d = x.shape
    G = synth.default_G(d)
    Ri, Ra = synth.rotations(G)
    rot = tq.Rotation(d, G, Ri, Ra)
    codes, scales = tq.torq_rotate_quantize(rot, x)
    z = tq.torq_rotate(rot, x)
    torch.cuda.synchronize()
    rng = np.random.default_rng(17)
    rows = np.unique(np.concatenate([[0, 1, M - 2, M - 1], rng.integers(0, M, size=12)]))
    rows_t = torch.from_numpy(rows).to(DEV)
    xs, z_ref, want_c, want_s, _ = _check_rows(oracle, tq, rot, x, rows_t, G, Ri, Ra)
    got_z = _np(z[rows_t]).astype(np.float64)
    zr = z_ref.astype(np.float64)
    rms = np.sqrt((zr ** 2).mean(axis=1, keepdims=True))
    assert (np.abs(got_z - zr) / rms).max() <= 1e-3
    got_c, got_s = _np(codes[rows_t]), _np(scales[rows_t])
    # the fused kernel equals the quantiser applied to its own rotated values, bit for bit, on the WHOLE
    # tensor (a fault at a tile edge or in a tail batch cannot hide between the sampled rows) ...
    c2, s2 = tq.torq_quantize_f32(z)
    torch.cuda.synchronize()
    assert torch.equal(c2, codes) and torch.equal(s2, scales)
    del c2, s2
    # ... and differs from the oracle only where the oracle's value sits on a rounding boundary
    n = len(rows)
    tol = 1e-3 * rms
    amax = np.abs(zr).reshape(n, d // 32, 32).max(axis=2)
    e = np.floor(np.log2(amax))
    pow2_dist = np.minimum(np.abs(amax - 2.0 ** e), np.abs(amax - 2.0 ** (e + 1)))
    sdiff = got_s != want_s
    assert np.all(pow2_dist[sdiff] <= tol.repeat(d // 32, axis=1)[sdiff])
    unpack = lambda c: np.stack([c & 15, c >> 4], axis=-1).reshape(n, d)
    gc, wc = unpack(got_c), unpack(want_c)
    cdiff = (gc != wc) & ~np.repeat(sdiff, 32, axis=1)
    s = np.repeat(np.ldexp(1.0, want_s.astype(np.int64) - 127), 32, axis=1)
    bounds = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    slack = np.abs((np.abs(zr) / s)[..., None] - bounds).min(axis=-1) * s
    near = (slack <= np.broadcast_to(tol, slack.shape)) | (np.abs(zr) <= np.broadcast_to(tol, zr.shape))
    assert np.all(near[cdiff])
    assert cdiff.mean() <= 0.005 and sdiff.mean() <= 0.002
    rot.close()


GEMM_FULL = [
    (8192, 28672, 8192),      # LLaMA3-70B MLP up / gate: the benchmark's step
    (8192, 8192, 28672),      # LLaMA3-70B MLP down
    (2048, 14336, 4096),      # LLaMA3-8B MLP up, prefill
    (16, 4096, 4096),         # decode-sized M
    (1, 14336, 4096),
    (4096, 5120, 25600),      # Qwen3-32B MLP down (d not a power of two)
    (2048, 4096, 4096),       # LLaMA3-8B attention projection, prefill: the 256 x 128 tile
    (1000, 8100, 1024),       # 256 x 128 tile with ragged last tiles in both directions
    (1000, 8100, 640),        # the same with a k range that is not a whole number of 512-element pieces
    (2048, 4096, 14336),      # LLaMA3-8B MLP down, prefill
    (16, 4096, 14336),        # ... and at decode size
    (2048, 1024, 4096),       # LLaMA3-8B k/v projection
    (4096, 25600, 5120),      # Qwen3-32B MLP up / gate
    (4096, 1024, 5120),       # Qwen3-32B k/v projection
    (4096, 8192, 5120),       # Qwen3-32B q projection
    (16, 28672, 8192),        # LLaMA3-70B MLP up at decode size: workgroups that keep the activations across four strip groups
    (12, 28000, 8192),        # ... with ragged rows and a ragged last group
    (8, 8192, 8192),          # ... one strip per group, two groups per workgroup
    (4096, 5120, 5120),       # Qwen3-32B attention output: a round and a quarter of tiles, run as two products
    (4000, 5000, 5120),       # ... with ragged last tiles in both
]


@pytest.mark.parametrize("M,N,d", GEMM_FULL)
def test_gemm_full_size_sampled_outputs(tq, oracle, M, N, d):
    g = torch.Generator(device=DEV)
    g.manual_seed(synth.SEED_BASE + M + N + d)
    A_q = torch.randint(0, 256, (M, d // 2), dtype=torch.uint8, device=DEV, generator=g)
    W_q = torch.randint(0, 256, (N, d // 2), dtype=torch.uint8, device=DEV, generator=g)
    A_s = torch.randint(118, 136, (M, d // 32), dtype=torch.uint8, device=DEV, generator=g)
    W_s = torch.randint(110, 126, (N, d // 32), dtype=torch.uint8, device=DEV, generator=g)
    out = tq.mxfp4_gemm(A_q, A_s, W_q, W_s)
    torch.cuda.synchronize()
    rng = np.random.default_rng(M + 3 * N)
    n_s = 4096
    ms = rng.integers(0, M, size=n_s)
    ns = rng.integers(0, N, size=n_s)
    # corners and tile edges as well
    ms[:8] = [0, 0, M - 1, M - 1, min(255, M - 1), min(256, M - 1), M // 2, M - 1]
    ns[:8] = [0, N - 1, 0, N - 1, min(255, N - 1), min(256, N - 1), N // 2, N // 2]
    um, im = np.unique(ms, return_inverse=True)
    un, inn = np.unique(ns, return_inverse=True)
    Aq_h, As_h = _np(A_q[torch.from_numpy(um).to(DEV)]), _np(A_s[torch.from_numpy(um).to(DEV)])
    Wq_h, Ws_h = _np(W_q[torch.from_numpy(un).to(DEV)]), _np(W_s[torch.from_numpy(un).to(DEV)])
    want = oracle.gemm_sampled(Aq_h, As_h, Wq_h, Ws_h, im, inn)
    got = _np(out[torch.from_numpy(ms).to(DEV), torch.from_numpy(ns).to(DEV)].view(torch.int16)).view(np.uint16)
    gw, ww = _bf16_bits_to_f64(got), _bf16_bits_to_f64(want)
    assert np.linalg.norm(gw - ww) / np.linalg.norm(ww) <= 1e-3
    # fp32 accumulation of exactly representable products: almost every output is the correctly
    # rounded bf16 value, the rest are one bf16 ulp off
    assert np.mean(got == want) > 0.98
    assert np.all(np.abs(gw - ww) <= np.abs(ww) * 2.0 ** -7 + 1e-3 * np.sqrt(np.mean(ww ** 2)))


# Products whose tile count is just above a whole number of rounds run as two: the leading columns that make
# whole rounds of 256 x 256 tiles, then the remaining columns with a plan of their own (their k range cut
# where a workspace allows).  GEMM_FULL above checks four such shapes against the oracle; here every output
# of the two launches is compared with the same columns computed as products of their own, bit for bit, and
# with the whole product on another tile shape.
@pytest.mark.parametrize("M,N,d", [(4096, 5120, 5120), (4000, 5000, 5120), (4096, 25600, 5120), (4096, 5120, 25600),
                                   (8192, 5120, 8192)])
def test_gemm_whole_rounds_first_then_the_remaining_columns(tq, M, N, d):
    g = torch.Generator(device=DEV)
    g.manual_seed(synth.SEED_BASE + 7 * M + N + d)
    A_q = torch.randint(0, 256, (M, d // 2), dtype=torch.uint8, device=DEV, generator=g)
    W_q = torch.randint(0, 256, (N, d // 2), dtype=torch.uint8, device=DEV, generator=g)
    A_s = torch.randint(118, 136, (M, d // 32), dtype=torch.uint8, device=DEV, generator=g)
    W_s = torch.randint(110, 126, (N, d // 32), dtype=torch.uint8, device=DEV, generator=g)
    main = tq.mxfp4_gemm_main_columns(M, N, d, 0)
    assert 0 < main < N and main % 256 == 0, "this shape is meant to run as two products"
    assert tq.mxfp4_gemm_plan(M, N, d, 0) == (False, 256, 256, 1)
    # one row more than the product has, so that a store past the last row would show
    guard = torch.full((M + 1, N), 0x7FC1, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    out = guard[:M]
    tq.mxfp4_gemm(A_q, A_s, W_q, W_s, out=out)
    left = tq.mxfp4_gemm(A_q, A_s, W_q[:main], W_s[:main])
    right = tq.mxfp4_gemm(A_q, A_s, W_q[main:], W_s[main:])
    torch.cuda.synchronize()
    assert torch.equal(out[:, :main].view(torch.int16), left.view(torch.int16))
    assert torch.equal(out[:, main:].view(torch.int16), right.view(torch.int16))
    assert bool((guard[M].view(torch.int16) == 0x7FC1).all())
    # the whole product on 256 x 128 tiles (the persistent form takes any shape with d a multiple of 1024)
    other = tq.torq_diag_gemm_persistent(A_q, A_s, W_q, W_s, tile=1, workgroups=256)
    torch.cuda.synchronize()
    assert torch.equal(other.view(torch.int16), out.view(torch.int16))
    del other
    # with a workspace the remainder's k range may be cut: its columns are then those of mxfp4_gemm_ws on the
    # remainder alone (bit for bit: same pieces, same order), and equal to the uncut ones up to the order of fp32 sums
    need = tq.mxfp4_gemm_workspace_bytes(M, N, d)
    ws = torch.empty((max(need, 16),), dtype=torch.uint8, device=DEV)
    assert tq.mxfp4_gemm_main_columns(M, N, d, need) == main
    guard2 = torch.full((M + 1, N), 0x7FC1, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    out2 = guard2[:M]
    tq.mxfp4_gemm_ws(A_q, A_s, W_q, W_s, out=out2, workspace=ws)
    right2 = tq.mxfp4_gemm_ws(A_q, A_s, W_q[main:], W_s[main:], workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(out2[:, :main].view(torch.int16), left.view(torch.int16))
    assert torch.equal(out2[:, main:].view(torch.int16), right2.view(torch.int16))
    assert bool((guard2[M].view(torch.int16) == 0x7FC1).all())
    a, b = out2[:, main:].double(), right.double()
    assert float((a - b).norm() / b.norm()) <= 1e-3
    if tq.mxfp4_gemm_plan(M, N - main, d, need)[3] == 1:
        assert torch.equal(out2.view(torch.int16), out.view(torch.int16))


# (the two Qwen3-32B layers run their product as whole rounds of tiles plus the remaining columns, the second
# with the remainder's k range cut in the workspace that torq_linear is given)
@pytest.mark.parametrize("name,N", [("llama3_70b_up", 4096), ("qwen3_32b", 5120), ("qwen3_32b_down", 5120)])
def test_linear_full_size_is_its_two_halves_and_matches_oracle_on_samples(tq, oracle, name, N):
    wl = synth.WORKLOADS[name]
    M, d = wl["M"], wl["d"]                     # N trimmed: the weights are generated and prepared here
    G = synth.default_G(d)
    x = synth.workload_activations(name, device=DEV)
    w = synth.workload_weights(name, device=DEV, N=N)
    Ri, Ra = synth.rotations(G)
    rot = tq.Rotation(d, G, Ri, Ra)
    W_q, W_s = tq.torq_rotate_quantize(rot, w)
    out = tq.torq_linear(rot, x, W_q, W_s)
    A_q, A_s = tq.torq_rotate_quantize(rot, x)
    out2 = tq.mxfp4_gemm_ws(A_q, A_s, W_q, W_s)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    if name != "llama3_70b_up":
        assert tq.mxfp4_gemm_main_columns(M, N, d, tq.mxfp4_gemm_workspace_bytes(M, N, d)) < N
    rng = np.random.default_rng(5)
    rm = np.unique(rng.integers(0, M, size=12))
    rn = np.unique(rng.integers(0, N, size=48))
    rm_t, rn_t = torch.from_numpy(rm).to(DEV), torch.from_numpy(rn).to(DEV)
    oA = oracle.rotate_quantize(synth.bf16_bits(x[rm_t]), G, Ri, Ra)
    oW = oracle.rotate_quantize(synth.bf16_bits(w[rn_t]), G, Ri, Ra)
    want = _bf16_bits_to_f64(oracle.gemm(oA[0], oA[1], oW[0], oW[1]))
    got = _np(out[rm_t][:, rn_t].to(torch.float64))
    # whole chain against the oracle's whole chain: a few boundary values may round differently
    # on the two sides (see test_rotate_quantize_full_size_sampled_rows), hence 5e-3 instead of 1e-3
    assert np.linalg.norm(got - want) / np.linalg.norm(want) <= 5e-3
    rot.close()


# ------------------------------------------------- sizes past 2^31 / 2^32 ----
# Element counts and byte offsets that do not fit 32 bits: every kernel indexes rows with 64-bit
# arithmetic and only tile-relative offsets with 32 bits.

def test_rotate_quantize_more_than_2_31_elements(tq, oracle):
    M, d, G = 70000, 32768, 128                  # 2.29e9 elements, 4.6 GB of input
    g = torch.Generator(device=DEV)
    g.manual_seed(synth.SEED_BASE + 31)
    x = torch.empty((M, d), dtype=torch.bfloat16, device=DEV)
    for r0 in range(0, M, 10000):                # generated in slices: fp32 temporaries stay small
        r1 = min(M, r0 + 10000)
        x[r0:r1] = (torch.randn((r1 - r0, d), device=DEV, generator=g) *
                    torch.exp(torch.randn((r1 - r0, 1), device=DEV, generator=g))).to(torch.bfloat16)
    Ri, Ra = synth.rotations(G)
    rot = tq.Rotation(d, G, Ri, Ra)
    codes, scales = tq.torq_rotate_quantize(rot, x)
    torch.cuda.synchronize()
    rows = np.array([0, 65535, 65536, 65537, M - 1])      # element index of row 65536 is exactly 2^31
    rows_t = torch.from_numpy(rows).to(DEV)
    xs = x[rows_t].contiguous()
    z_ref = oracle.rotate(synth.bf16_bits(xs), G, Ri, Ra)
    want_c, want_s = oracle.quantize(z_ref)
    got_c, got_s = _np(codes[rows_t]), _np(scales[rows_t])
    # the kernel's own result on the gathered rows (small problem, same arithmetic) must be identical
    c2, s2 = tq.torq_rotate_quantize(rot, xs)
    assert np.array_equal(_np(c2), got_c) and np.array_equal(_np(s2), got_s)
    # and close to the oracle: only boundary values may differ
    assert (got_s != want_s).mean() <= 0.002
    unpack = lambda c: np.stack([c & 15, c >> 4], axis=-1).reshape(len(rows), d)
    assert (unpack(got_c) != unpack(want_c)).mean() <= 0.006
    rot.close()


@pytest.mark.parametrize("M,N,d", [(40000, 60000, 128),      # 2.4e9 outputs (tiled kernel)
                                   (16, 300000, 32768)])     # 4.9 GB of weight codes (weight-streaming kernel)
def test_gemm_more_than_2_31_outputs_or_weight_bytes(tq, oracle, M, N, d):
    g = torch.Generator(device=DEV)
    g.manual_seed(synth.SEED_BASE + M + N)
    A_q = torch.randint(0, 256, (M, d // 2), dtype=torch.uint8, device=DEV, generator=g)
    W_q = torch.randint(0, 256, (N, d // 2), dtype=torch.uint8, device=DEV, generator=g)
    A_s = torch.randint(118, 136, (M, d // 32), dtype=torch.uint8, device=DEV, generator=g)
    W_s = torch.randint(110, 126, (N, d // 32), dtype=torch.uint8, device=DEV, generator=g)
    out = tq.mxfp4_gemm(A_q, A_s, W_q, W_s)
    torch.cuda.synchronize()
    rng = np.random.default_rng(N)
    n_s = 2048
    ms = rng.integers(0, M, size=n_s)
    ns = rng.integers(0, N, size=n_s)
    ms[:4] = [0, M - 1, M - 1, M // 2]
    ns[:4] = [0, N - 1, 0, N - 1]
    um, im = np.unique(ms, return_inverse=True)
    un, inn = np.unique(ns, return_inverse=True)
    um_t, un_t = torch.from_numpy(um).to(DEV), torch.from_numpy(un).to(DEV)
    want = oracle.gemm_sampled(_np(A_q[um_t]), _np(A_s[um_t]), _np(W_q[un_t]), _np(W_s[un_t]), im, inn)
    got = _np(out[torch.from_numpy(ms).to(DEV), torch.from_numpy(ns).to(DEV)].view(torch.int16)).view(np.uint16)
    gw, ww = _bf16_bits_to_f64(got), _bf16_bits_to_f64(want)
    assert np.linalg.norm(gw - ww) / np.linalg.norm(ww) <= 1e-3
    assert np.all(np.abs(gw - ww) <= np.abs(ww) * 2.0 ** -7 + 1e-3 * np.sqrt(np.mean(ww ** 2)))


def test_block_gram_many_token_groups_per_workgroup(tq, oracle):
    # 2048 token-groups: every workgroup accumulates several in fp32 before the double reduction
    M, d, G = 1024, 8192, 128
    x = synth.workload_activations("llama3_70b_up", device=DEV, M=M)
    want = oracle.block_gram(synth.bf16_bits(x), G)
    got = _np(tq.torq_block_gram(x, G))
    torch.cuda.synchronize()
    assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max()
    # the full benchmark input: symmetric, and its trace is the mean energy of a token-group
    xf = synth.workload_activations("llama3_70b_up", device=DEV)
    Sf = _np(tq.torq_block_gram(xf, G))
    assert np.array_equal(Sf, Sf.T)
    energy = float((xf.double() ** 2).sum().item()) / (xf.shape[0] * (xf.shape[1] // 32 // G))
    assert abs(np.trace(Sf) - energy) <= 1e-5 * energy


def test_code_histogram_more_than_255_blocks_per_lane(tq, oracle):
    # 35.8 M blocks: every lane counts more blocks than a byte counter holds, so the workgroup sum
    # through LDS runs more than once; the last span is ragged
    M, d = 39999, 28672
    g = torch.Generator(device=DEV).manual_seed(6100)
    codes = torch.randint(0, 256, (M, d // 2), dtype=torch.uint8, device=DEV, generator=g)
    codes.view(M, d // 32, 16)[:, :, 0] &= 0xF8     # position 0 of every block carries codeword 0 (or -0)
    got = _np(tq.torq_code_histogram(codes, d)).astype(np.uint64)
    torch.cuda.synchronize()
    want = oracle.code_histogram(_np(codes), d)
    assert np.array_equal(got, want)
    assert got[0, 0] == M * (d // 32) and got.sum() == M * d


def test_code_histogram_of_the_benchmark_step(tq, oracle):
    # the packed codes of the benchmark's rotate + quantise: exact against the oracle's count
    x = synth.workload_activations("llama3_70b_up", device=DEV)
    M, d = x.shape
    G = synth.default_G(d)
    Ri, Ra = synth.rotations(G)
    rot = tq.Rotation(d, G, Ri, Ra)
    codes, _ = tq.torq_rotate_quantize(rot, x)
    got = _np(tq.torq_code_histogram(codes, d)).astype(np.uint64)
    assert np.array_equal(got, oracle.code_histogram(_np(codes), d))
    rot.close()


@pytest.mark.parametrize("name,G", [("llama3_70b_up", 128), ("llama3_70b_up", 256), ("llama3_8b_prefill", 64)])
def test_butterfly_rotate_quantize_full_size_sampled_rows(tq, oracle, name, G):
    # the butterfly handle at the benchmark's sizes: tangents from the host equaliser on the Gram of the
    # activations themselves (GPU), rows sampled for the oracle, which rotates with the dense matrix
    x = synth.workload_activations(name, device=DEV)
    M, d = x.shape
    Sigma = _np(tq.torq_block_gram(x, G))
    R, T = tq.torq_equalize_inter_butterfly(Sigma)
    _, Ra = synth.rotations(G)
    rot = tq.ButterflyRotation(d, G, T, Ra)
    codes, scales = tq.torq_rotate_quantize(rot, x)
    z = tq.torq_rotate(rot, x)
    torch.cuda.synchronize()
    rng = np.random.default_rng(19)
    rows = np.unique(np.concatenate([[0, 1, M - 2, M - 1], rng.integers(0, M, size=12)]))
    rows_t = torch.from_numpy(rows).to(DEV)
    xs, z_ref, want_c, want_s, _ = _check_rows(oracle, tq, rot, x, rows_t, G, R, Ra)
    zr = z_ref.astype(np.float64)
    rms = np.sqrt((zr ** 2).mean(axis=1, keepdims=True))
    assert (np.abs(_np(z[rows_t]).astype(np.float64) - zr) / rms).max() <= 1e-3
    c2, s2 = tq.torq_quantize_f32(z[rows_t].contiguous())
    assert torch.equal(c2, codes[rows_t]) and torch.equal(s2, scales[rows_t])
    oc, os_ = oracle.quantize(_np(z[rows_t]))
    assert np.array_equal(_np(c2), oc) and np.array_equal(_np(s2), os_)
    # the whole sample's block energies are equal after the rotation (output condition of Section 5.1)
    nt = M * d // (32 * G)
    energies = (z.double().reshape(nt, G, 32) ** 2).sum(dim=2).mean(dim=0).cpu().numpy()
    c = np.trace(Sigma) / G
    assert np.diag(Sigma).max() / np.diag(Sigma).min() > 5.0
    assert np.abs(energies - c).max() <= 2e-3 * c
    rot.close()
