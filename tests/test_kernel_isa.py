"""Build test for the one hand-scheduled loop whose correctness rests on instruction counts.

rotate_ring_kernel32 (rotate_quant.hip) waits for "the batch requested two iterations ago" with
s_waitcnt vmcnt(N), N = the number of vector-memory instructions a wave issues after that request.
That is only right if the compiled loop holds exactly the loads and stores the source counts with, and
no wait of the compiler's own that would serialise it.  This test compiles the file to assembly (no GPU
needed) and checks that for every instantiation."""
import os
import re
import tempfile

import pytest

from paper_2605_19561_amd import build


@pytest.fixture(scope="module")
def ring_kernels():
    with tempfile.TemporaryDirectory() as tmp:
        path = build.device_asm("rotate_quant.hip", os.path.join(tmp, "rotate_quant.s"))
        text = open(path).read()
    kernels, cur = {}, None
    for line in text.splitlines():
        m = re.match(r"^(_ZN4torq20rotate_ring_kernel32\w+):", line)
        if m:
            cur = m.group(1)
            kernels[cur] = []
            continue
        if cur is None:
            continue
        code = line.split(";")[0].strip()
        if code.startswith(".Lfunc_end"):
            cur = None
        elif code and not code.startswith("."):
            kernels[cur].append(code)
    meta = {}
    for m in re.finditer(r"\.name:\s+(_ZN4torq20rotate_ring_kernel32\w+)\n(?:.*\n)*?\s+\.private_segment_fixed_size:\s+(\d+)", text):
        meta[m.group(1)] = int(m.group(2))
    return kernels, meta


def test_every_ring_instantiation_is_there(ring_kernels):
    kernels, _ = ring_kernels
    # G = 80, 96, 112, 128 x three formats (+ the diagnostic builds of G = 128 / MXFP4)
    for ks16 in (5, 6, 7, 8):
        for fmt in (0, 1, 2):
            assert any(f"ILi{ks16}ELi{fmt}ELi0E" in k for k in kernels), (ks16, fmt)


def test_ring_loop_holds_exactly_the_counted_memory_instructions(ring_kernels):
    kernels, meta = ring_kernels
    vmem = re.compile(r"^(buffer_|global_|flat_|scratch_)")
    for name, code in kernels.items():
        assert meta.get(name, 0) == 0, f"{name}: spills to scratch memory would add vector-memory instructions"
        assert sum(c.startswith("s_barrier") for c in code) == 3, name      # the loop is unrolled over the three buffers
        ops = [(i, c) for i, c in enumerate(code) if vmem.match(c)]
        lds_loads = [i for i, c in ops if c.startswith("buffer_load_dwordx4") and c.endswith("lds")]
        stores = [i for i, c in ops if c.startswith("buffer_store_")]
        others = [(i, c) for i, c in ops if i not in lds_loads and i not in stores]
        # two batches requested ahead of the loop + one per unrolled iteration, four instructions each;
        # two token-groups x (codes, scale byte) stored per unrolled iteration
        assert len(lds_loads) == 8 + 3 * 4, (name, len(lds_loads))
        assert len(stores) == 3 * 4, (name, len(stores))
        # everything else is the load of the resident operands, ahead of the first request
        assert all(c.startswith("global_load_dwordx4") and i < lds_loads[0] for i, c in others), (name, others[:3])
        # waits on the vector-memory counter behind the two requests ahead of the loop: the one for the
        # resident operands, then the hand-written ones of the three unrolled iterations (4 or 12
        # operations may stay in flight; 8 or 12; 12) and the drain at the end -- none of the compiler's
        # own, which would serialise the ring
        waits = [int(re.search(r"vmcnt\((\d+)\)", c).group(1)) for i, c in enumerate(code)
                 if "vmcnt(" in c and i > lds_loads[7]]
        assert waits[0] == 0 and sorted(waits[1:]) == [0, 4, 8, 12, 12, 12], (name, waits)


# ---- torq_linear_local_kernel (mxfp4_gemm_skinny.hip): not correctness but the point of the kernel.  The
# rotation's reads are issued ahead of the workgroup's weight reads and its LDS stores must wait for them
# alone -- s_waitcnt vmcnt(N) with N >= the number of weight loads behind them.  A load that the compiler
# moves under a condition, or a predicate on the weight loads, turns that into vmcnt(0): the rotation then
# waits for the whole weight stream.  Checked on the full-trip (EXACT) instantiations.

@pytest.fixture(scope="module")
def local_kernels():
    with tempfile.TemporaryDirectory() as tmp:
        path = build.device_asm("mxfp4_gemm_skinny.hip", os.path.join(tmp, "skinny.s"))
        text = open(path).read()
    kernels, cur = {}, None
    for line in text.splitlines():
        m = re.match(r"^(_ZN4torq24torq_linear_local_kernel\w+):", line)
        if m:
            cur = m.group(1)
            kernels[cur] = []
            continue
        if cur is None:
            continue
        code = line.split(";")[0].strip()
        if code.startswith(".Lfunc_end"):
            cur = None
        elif code and not code.startswith("."):
            kernels[cur].append(code)
    meta = {}
    for m in re.finditer(r"\.name:\s+(_ZN4torq24torq_linear_local_kernel\w+)\n(?:.*\n)*?\s+\.private_segment_fixed_size:\s+(\d+)", text):
        meta[m.group(1)] = int(m.group(2))
    return kernels, meta


def test_local_kernel_rotation_waits_for_its_own_reads_only(local_kernels):
    kernels, meta = local_kernels
    seen = 0
    for name, code in kernels.items():
        assert meta.get(name, 0) == 0, f"{name}: spills to scratch memory"
        m = re.search(r"ILi(\d+)ELi(\d+)ELb(\d)E", name)
        ns, pt, exact = int(m.group(1)), int(m.group(2)), int(m.group(3))
        if not exact:
            continue
        seen += 1
        weight_loads = 2 * pt * ns
        first_barrier = next(i for i, c in enumerate(code) if c.startswith("s_barrier"))
        second_barrier = next(i for i, c in enumerate(code) if c.startswith("s_barrier") and i > first_barrier)
        # between the waves' rendezvous and the barrier behind the LDS stores: the weight loads, all of them,
        # in straight-line code, then the four stores of the token-groups, each behind a wait that leaves
        # the weight loads in flight
        span = code[first_barrier + 1:second_barrier]
        assert not any(c.startswith("s_cbranch") for c in span), name
        assert sum(c.startswith("buffer_load_dwordx4") for c in span) == weight_loads, name
        stores = [i for i, c in enumerate(span) if c.startswith("ds_write_b128")]
        assert len(stores) == 4, (name, len(stores))
        waits = [int(re.search(r"vmcnt\((\d+)\)", c).group(1)) for c in span[:stores[-1]] if "vmcnt(" in c]
        assert waits and min(waits) >= weight_loads, (name, waits, weight_loads)
        # and ahead of the rendezvous: every read of the rotation (16 + 4 operand loads, 4 token-group loads)
        head = code[:first_barrier]
        assert sum(c.startswith("global_load_dwordx4") for c in head) == 20, name
        assert sum(c.startswith("buffer_load_dwordx4") for c in head) == 4, name
        assert not any("vmcnt(" in c for c in head[next(i for i, c in enumerate(head) if c.startswith("global_load_dwordx4")):]), name
    assert seen >= 10
