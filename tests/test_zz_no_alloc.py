"""torq_linear_static, the entry point for callers that cannot allocate: its output against torq_linear's,
bit for bit, through the C ABI, on two calls in a row (the second on a smaller input, so that what the
first call left in the library's scratch array must not leak into it)."""
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


def _case(tq, rot, W_q, W_s, M, d, N, seed):
    x = synth.activations(M, d, nu=3.0, outliers=8, outlier_scale=50.0, seed=seed).to(DEV)
    want = tq.torq_linear(rot, x, W_q, W_s, workspace=torch.empty((tq.torq_linear_workspace_bytes(M, d),),
                                                                   dtype=torch.uint8, device=DEV))
    got = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    tq.torq_linear_static(rot, x, W_q, W_s, got)
    torch.cuda.synchronize()
    return got, want


def test_static_scratch_entry_point_matches_torq_linear(tq):
    d, G, N = 4096, 128, 1024
    Ri, Ra = synth.rotations(G)
    rot = tq.Rotation(d, G, Ri, Ra)
    W_q, W_s = tq.torq_rotate_quantize(rot, synth.weights(N, d, seed=21).to(DEV))
    # first call: several GEMM tiles and a ragged last one; second call: fewer rows (the weight-streaming GEMM)
    got1, want1 = _case(tq, rot, W_q, W_s, 300, d, N, seed=31)
    got2, want2 = _case(tq, rot, W_q, W_s, 5, d, N, seed=32)
    assert torch.equal(got1.view(torch.int16), want1.view(torch.int16))
    assert torch.equal(got2.view(torch.int16), want2.view(torch.int16))
    assert torch.isfinite(got1.float()).all() and torch.isfinite(got2.float()).all()
    # a third, between the two in size, on the largest row count the scratch holds at this d, and one beyond
    m_max = tq.TORQ_STATIC_SCRATCH_BYTES // (d // 2 + d // 32)
    while tq.torq_linear_workspace_bytes(m_max, d) > tq.TORQ_STATIC_SCRATCH_BYTES:
        m_max -= 1
    got3, want3 = _case(tq, rot, W_q, W_s, m_max, d, N, seed=33)
    assert torch.equal(got3.view(torch.int16), want3.view(torch.int16))
    # two rows of a decode step: both entry points take ONE launch there (every workgroup rotates the rows itself);
    # checked against torq_linear and against the two separate calls
    got4, want4 = _case(tq, rot, W_q, W_s, 2, d, N, seed=34)
    assert torch.equal(got4.view(torch.int16), want4.view(torch.int16))
    x4 = synth.activations(2, d, nu=3.0, outliers=8, outlier_scale=50.0, seed=34).to(DEV)
    chain = tq.mxfp4_gemm(*tq.torq_rotate_quantize(rot, x4), W_q, W_s)
    assert torch.equal(got4.view(torch.int16), chain.view(torch.int16))
    x = torch.zeros((m_max + 1, d), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((m_max + 1, N), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(tq.TorqError) as err:
        tq.torq_linear_static(rot, x, W_q, W_s, out)
    assert err.value.status == tq.TORQ_ETOOBIG
    torch.cuda.synchronize()
    assert not out.any()                      # nothing was launched
    rot.close()


def test_static_scratch_entry_point_empty_input(tq):
    d, G, N = 4096, 128, 256
    Ri, Ra = synth.rotations(G)
    rot = tq.Rotation(d, G, Ri, Ra)
    W_q = torch.zeros((N, d // 2), dtype=torch.uint8, device=DEV)
    W_s = torch.zeros((N, d // 32), dtype=torch.uint8, device=DEV)
    x = torch.empty((0, d), dtype=torch.bfloat16, device=DEV)
    out = torch.empty((0, N), dtype=torch.bfloat16, device=DEV)
    tq.torq_linear_static(rot, x, W_q, W_s, out)
    rot.close()
