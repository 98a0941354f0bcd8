"""GPU parity on the inputs that are meant to break a kernel: non-finite bit patterns in every
byte the update must NOT read (behind each selected expert's slice, behind the banks, in the
padding columns of W), and gate values far outside what a softmax produces (sub-normal, tiny,
negative, one fp32 step apart).  All reads stay inside the tensors' own allocations by design;
the poison only shows whether a value that should not matter reached the arithmetic
(0 x NaN = NaN in a matrix-core product)."""
import numpy as np
import pytest
import torch

import adafuse_workloads as wlmod
import paper_2603_11873_amd as af
from gpu_util import Tally, compare, compare_inplace

pytestmark = pytest.mark.gpu

ULP_TOL = 1
NAN_BITS, INF_BITS = 0x7FC1, 0x7F80
KERNELS = [af.KERNEL_VALU, af.KERNEL_MFMA, af.KERNEL_GEMM]


def _sync():
    torch.cuda.synchronize()


def _poison(t):
    """Fill a bf16 tensor with alternating NaN / +Inf bit patterns."""
    flat = t.view(torch.int16).view(-1)
    flat[0::2] = NAN_BITS
    flat[1::2] = INF_BITS


def _guarded(t, guard=8192):
    """A copy of `t` at the start of a larger allocation whose remaining elements are poison:
    returns (view with t's shape, the whole allocation)."""
    big = torch.empty(t.numel() + guard, dtype=torch.bfloat16, device="cuda:0")
    _poison(big)
    view = big[: t.numel()].view(t.shape)
    view.copy_(t)
    return view, big


def _poisoned_model(g, out, in_, ldw, E, r, selected):
    """One matrix whose banks hold finite values for the `selected` experts only; every other
    expert's slices, the tails of all four allocations and W's padding columns are poison."""
    base = (0.02 * torch.randn((out, ldw), generator=g)).to(torch.bfloat16)
    a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16)
    b = (0.05 * torch.randn((E, out, r), generator=g)).to(torch.bfloat16)
    base_d, base_big = _guarded(base.cuda())
    a_d, a_big = _guarded(a.cuda())
    b_d, b_big = _guarded(b.cuda())
    if ldw > in_:
        _poison_cols = base_d[:, in_:]
        _poison_cols.view(torch.int16)[:] = NAN_BITS
    for e in range(E):
        if e not in selected:
            _poison(a_d[e])
            _poison(b_d[e])
    return base_d, a_d, b_d, (base_big, a_big, b_big)


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("r", [4, 8, 16])
@pytest.mark.parametrize("sel", [[3], [3, 0], [1, 3]])
def test_nothing_outside_the_selected_slices_reaches_the_update(oracle, kernel, r, sel):
    """Out of place, ranks 4 and 8 (zero-padded to one k-step of 16) and 16, last expert of the
    bank selected: the rank indices beyond a padded rank must read as zero, not as the next
    expert's rows or as what follows the bank."""
    g = torch.Generator().manual_seed(100 * r + len(sel))
    out, in_, ldw, E = 130, 200, 208, 4
    base, a, b, keep = _poisoned_model(g, out, in_, ldw, E, r, sel)
    work_full = torch.empty((out, ldw), dtype=torch.bfloat16, device="cuda:0")
    work_full.view(torch.int16).fill_(NAN_BITS)
    wb, ww = base[:, :in_], work_full[:, :in_]
    ctx = af.Context([(wb, ww, a, b)], len(sel))
    ctx.set_kernel(kernel)
    idx = torch.tensor(sel, dtype=torch.int32, device="cuda:0")
    gates = torch.softmax(torch.randn(len(sel), generator=g), 0)
    ctx.fused_switch(None, None, idx, gates.cuda(), len(sel), 2.0, af.MERGE)
    _sync()
    got = wlmod.bits(ww)
    assert np.isfinite(wlmod.from_bits(got).float().numpy()).all(), "poison reached the update"
    tally = Tally()
    tally.add(compare(oracle, wlmod.bits(wb), wlmod.bits(a), wlmod.bits(b), got, sel, gates.numpy(), 2.0), ULP_TOL)
    tally.finish(1e-4)
    assert bool((work_full[:, in_:].view(torch.int16) == NAN_BITS).all())   # padding columns never written
    ctx.close()


@pytest.mark.parametrize("r", [4, 8, 16])
@pytest.mark.parametrize("form,name", [(4, "switch_gemm_strip_kernel"), (0, "switch_gemm_overlap_kernel")])
def test_padded_ranks_in_the_eight_term_form(oracle, r, form, name):
    """In place with top-4: a SWAP carries eight terms, which the default kernel runs in its
    one-tile overlapped form and, on request, in its chained form (both fetch the operands 16 bytes
    per lane, with the rank padding through the descriptor).  Previous and next token share the
    bank's last expert; three experts in between are poison."""
    g = torch.Generator().manual_seed(7 + r)
    out, in_, E = 190, 264, 10
    prev = (np.array([0, 2, 4, 9], np.int32), np.array([0.4, 0.3, 0.2, 0.1], np.float32))
    nxt = (np.array([9, 1, 3, 7], np.int32), np.array([0.35, 0.3, 0.2, 0.15], np.float32))
    base, a, b, keep = _poisoned_model(g, out, in_, in_, E, r, {0, 1, 2, 3, 4, 7, 9})
    before = oracle.merge(wlmod.bits(base), wlmod.bits(a), wlmod.bits(b), prev[0], prev[1], 2.0)
    w, w_big = _guarded(wlmod.from_bits(before, "cuda:0"))
    ctx = af.Context([(w, w, a, b)], 4)
    ctx.set_option(af.OPT_GEMM_FORM, form)
    assert ctx.switch_kernel_name(4, af.SWAP) == name
    dev = lambda x: torch.as_tensor(x, device="cuda:0")
    ctx.fused_switch(dev(prev[0]), dev(prev[1]), dev(nxt[0]), dev(nxt[1]), 4, 2.0, af.SWAP)
    _sync()
    got = wlmod.bits(w)
    assert np.isfinite(wlmod.from_bits(got).float().numpy()).all(), "poison reached the update"
    tally = Tally()
    tally.add(compare_inplace(oracle, before, wlmod.bits(a), wlmod.bits(b), got, prev, nxt, 2.0), ULP_TOL)
    tally.finish(1e-4)
    ctx.close()


GATES = [
    ([1.0, 1e-40], "ordinary then sub-normal"),
    ([1e-40, 1.0], "sub-normal then ordinary"),
    ([1e-30, 1e-30], "both tiny"),
    ([1e-30, 1.0], "30 orders of magnitude apart"),
    ([0.7, -0.3], "a negative gate"),
    ([-1e-38, 0.5], "negative near the smallest normal"),
    ([0.0, 1.0], "an exact zero beside a one"),
]


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("r", [16, 64])
@pytest.mark.parametrize("inplace", [False, True])
def test_gates_far_outside_a_softmax(oracle, kernel, r, inplace):
    """The API takes any fp32 gates.  A gate that is sub-normal or many orders of magnitude
    below its neighbour must simply contribute (next to) nothing: never an infinity or a NaN
    from a ratio of coefficients.  Rank 16 runs the unrolled form of the default kernel, rank 64
    its overlapped form."""
    g = torch.Generator().manual_seed(31 * r + inplace)
    E, k = 4, 2
    mats, host = [], []
    for out, in_ in ((190, 264), (64, 128)):
        wb = (0.02 * torch.randn((out, in_), generator=g)).to(torch.bfloat16).cuda()
        a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16).cuda()
        b = (0.05 * torch.randn((E, out, r), generator=g)).to(torch.bfloat16).cuda()
        ww = wb.clone() if inplace else torch.empty_like(wb)
        mats.append((ww if inplace else wb, ww, a, b))
        host.append((wlmod.bits(wb), wlmod.bits(a), wlmod.bits(b)))
    ctx = af.Context(mats, k)
    try:
        ctx.set_kernel(kernel)
    except af.AdafuseError:
        pytest.skip("this kernel is not built for this (r, k)")
    if kernel == af.KERNEL_VALU and k * r * 768 > 65536:
        ctx.close()
        pytest.skip("more than the baseline kernel can stage in LDS (it refuses the launch)")
    idx = np.array([2, 1], np.int32)
    d_idx = torch.as_tensor(idx, device="cuda:0")
    tally = Tally()
    for gates, what in GATES:
        gates = np.array(gates, np.float32)
        for m, (w, a, b) in zip(mats, host):
            (m[1].copy_(wlmod.from_bits(w)) if inplace else m[1].view(torch.int16).fill_(NAN_BITS))
        ctx.fused_switch(None, None, d_idx, torch.as_tensor(gates, device="cuda:0"), k, 2.0, af.MERGE)
        _sync()
        for m, (w, a, b) in zip(mats, host):
            got = wlmod.bits(m[1])
            assert np.isfinite(wlmod.from_bits(got).float().numpy()).all(), what
            tally.add(compare(oracle, w, a, b, got, idx, gates, 2.0), ULP_TOL, what)
    tally.finish(1e-4)
    ctx.close()


@pytest.mark.parametrize("r", [16, 64])
def test_inplace_swap_with_a_shared_expert_one_step_apart(oracle, r):
    """In place, an expert selected by both tokens enters with the DIFFERENCE of its two
    coefficients.  Gates one fp32 step apart make that difference about 1e-7 of the other terms."""
    g = torch.Generator().manual_seed(5 * r)
    E, out, in_ = 4, 190, 264
    wb = (0.02 * torch.randn((out, in_), generator=g)).to(torch.bfloat16)
    a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16).cuda()
    b = (0.05 * torch.randn((E, out, r), generator=g)).to(torch.bfloat16).cuda()
    g0 = np.float32(0.6)
    prev = (np.array([0, 1], np.int32), np.array([g0, 0.4], np.float32))
    nxt = (np.array([0, 2], np.int32), np.array([np.nextafter(g0, np.float32(1)), 0.4], np.float32))
    before = oracle.merge(wlmod.bits(wb), wlmod.bits(a), wlmod.bits(b), prev[0], prev[1], 2.0)
    w = wlmod.from_bits(before, "cuda:0")
    ctx = af.Context([(w, w, a, b)], 2)
    dev = lambda x: torch.as_tensor(x, device="cuda:0")
    ctx.fused_switch(dev(prev[0]), dev(prev[1]), dev(nxt[0]), dev(nxt[1]), 2, 2.0, af.SWAP)
    _sync()
    got = wlmod.bits(w)
    assert np.isfinite(wlmod.from_bits(got).float().numpy()).all()
    tally = Tally()
    tally.add(compare_inplace(oracle, before, wlmod.bits(a), wlmod.bits(b), got, prev, nxt, 2.0), ULP_TOL)
    tally.finish(1e-4)
    ctx.close()


@pytest.mark.parametrize("kernel", KERNELS)
def test_one_direction_probes_touch_exactly_their_side(kernel):
    """adafuse_hbm_probe: the read pass changes nothing; the write pass zeroes every element of
    W_work inside the matrix and nothing outside it (padding columns, the allocation's tail), and
    is refused where W_work is the only copy of the weights."""
    g = torch.Generator().manual_seed(77)
    out, in_, ldw, E, r = 190, 264, 272, 3, 8
    base = (0.02 * torch.randn((out, ldw), generator=g)).to(torch.bfloat16).cuda()
    a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16).cuda()
    b = (0.05 * torch.randn((E, out, r), generator=g)).to(torch.bfloat16).cuda()
    work_full, work_big = _guarded(torch.ones((out, ldw), dtype=torch.bfloat16))
    work_full.view(torch.int16).fill_(NAN_BITS)
    before_base = base.clone()
    ctx = af.Context([(base[:, :in_], work_full[:, :in_], a, b)], 2)
    ctx.set_kernel(kernel)
    ctx.hbm_probe(af.PROBE_READ_BASE)
    _sync()
    assert torch.equal(base.view(torch.int16), before_base.view(torch.int16))
    assert bool((work_full.view(torch.int16) == NAN_BITS).all())
    ctx.hbm_probe(af.PROBE_ZERO_WORK)
    _sync()
    assert bool((work_full[:, :in_].view(torch.int16) == 0).all())
    assert bool((work_full[:, in_:].view(torch.int16) == NAN_BITS).all())
    tail = work_big[out * ldw:].view(torch.int16)
    assert bool(((tail == NAN_BITS) | (tail == INF_BITS)).all())
    assert torch.equal(base.view(torch.int16), before_base.view(torch.int16))
    with pytest.raises(af.AdafuseError):
        ctx.hbm_probe(2)
    ctx.close()
    w = base[:, :in_]
    inplace = af.Context([(w, w, a, b)], 2)
    inplace.hbm_probe(af.PROBE_READ_BASE)
    with pytest.raises(af.AdafuseError):
        inplace.hbm_probe(af.PROBE_ZERO_WORK)
    _sync()
    assert torch.equal(base.view(torch.int16), before_base.view(torch.int16))
    inplace.close()
