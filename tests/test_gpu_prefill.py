"""GPU parity of adafuse_prefill (many tokens, per-token routing decisions, adapters un-merged)
against the fp64 oracle's token-by-token Eq.2.

Tolerance.  The device forms every output element as an fp32 sum of exact bf16 x bf16 products
(the inner dimension in four parts added in a fixed order), and carries the scaled
down-projection s g (A x) as a pair of bf16 values (relative remainder below 2^-17).  With
mag = sum_i |W||x| + sum_j |s g_j| sum_rho |B_j| (sum_i |A_j||x|) the worst case is
(in / 4 + r + 8) 2^-24 mag + 2^-17 mag_adapter (the second term of mag); the fp32 roundings are
independent and add like a random walk, so what is asserted is 2e-6 mag + 2^-17 mag_adapter
(measured: 3e-8 mag on the 7B shapes, 1.4e-7 on the toy; the pair's remainder only shows where
the input width is a handful of elements and the adapters are most of the result).
"""
import numpy as np
import pytest
import torch

import adafuse_workloads as wlmod
import paper_2603_11873_amd as af
from gpu_util import oracle_decisions

pytestmark = pytest.mark.gpu

RTOL_MAG = 2e-6
NAN_BITS = 0x7FC1


def _magnitude(w, a, b, idx_t, gates_t, scale, x_t):
    """(mag, mag_adapter) per output row: sums of absolute values of everything that enters it."""
    f = lambda v: np.abs(wlmod.from_bits(v).double().numpy())
    base = f(w) @ np.abs(x_t)
    ad = np.zeros_like(base)
    for e, g in zip(idx_t, gates_t):
        ad = ad + abs(float(scale) * float(g)) * (f(b[e]) @ (f(a[e]) @ np.abs(x_t)))
    return base + ad, ad


def _check(oracle, mat, x, idx, gates, scale, y, tokens):
    """Rows `tokens` of y against the oracle; returns the largest error in units of mag."""
    wb, _, a, b = mat
    w_h, a_h, b_h, x_h = wlmod.bits(wb), wlmod.bits(a), wlmod.bits(b), wlmod.bits(x)
    want = oracle.prefill(w_h, a_h, b_h, idx, gates, scale, x_h, tokens=tokens)
    got = y.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    xs = x.double().cpu().numpy()
    worst = 0.0
    for row, t in zip(want, tokens):
        mag, mag_ad = _magnitude(w_h, a_h, b_h, idx[t], gates[t], scale, xs[t])
        err = np.abs(got[t] - row)
        assert np.all(err <= RTOL_MAG * mag + 2.0 ** -17 * mag_ad), (t, float(np.max(err / mag)))
        worst = max(worst, float(np.max(err / mag)))
    return worst


def test_toy_every_token_every_matrix(oracle):
    wl = wlmod.WORKLOADS["toy"]
    dev = torch.device("cuda:0")
    mats = []
    for layer in range(wl.layers):
        for mi in range(len(wl.mats)):
            wb = wlmod.gen_w(wl, layer, mi).to(dev)
            mats.append((wb, torch.empty_like(wb), wlmod.gen_a_bank(wl, layer, mi).to(dev), wlmod.gen_b_bank(wl, layer, mi).to(dev)))
    hidden, router = wlmod.gen_hidden(wl).to(dev), wlmod.gen_router(wl).to(dev)
    ctx = af.Context(mats, wl.k)
    hidx, hg, _, _ = oracle_decisions(oracle, hidden, router, wl.k)
    idx, gates, _ = af.pregate(hidden, router, wl.k)          # the device pipeline: router output feeds the prefill
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), hidx)
    worst = 0.0
    for mi, mat in enumerate(mats):
        y = ctx.prefill(mi, hidden, idx, gates, wl.scale)
        torch.cuda.synchronize()
        worst = max(worst, _check(oracle, mat, hidden, hidx, gates.cpu().numpy(), wl.scale, y, range(wl.T)))
    print(f"\n[toy prefill] largest error {worst:.2e} of the operand magnitude")
    ctx.close()


RAGGED = [  # out, in, E, r, k, T
    (130, 200, 4, 4, 2, 33),
    (70, 264, 5, 8, 3, 1),
    (257, 136, 8, 16, 4, 70),
    (66, 120, 3, 64, 2, 100),
    (129, 136, 4, 128, 2, 45),
    (301, 200, 9, 32, 1, 129),
    (31, 8, 2, 4, 1, 65),
]


@pytest.mark.parametrize("out,in_,E,r,k,T", RAGGED)
def test_ragged_shapes_duplicates_and_unused_experts(oracle, out, in_, E, r, k, T):
    """Token counts, widths and heights that end inside a block (in a multiple of 8 but not of 16
    included), every rank, one expert per bank that no token selects and that is filled with NaN
    patterns, a leading dimension larger than the width with NaN in the padding, and some tokens
    that list the same expert twice."""
    dev = torch.device("cuda:0")
    g = torch.Generator().manual_seed(out * 13 + T)
    ldw = in_ + 8
    base = (0.02 * torch.randn((out, ldw), generator=g)).to(torch.bfloat16).to(dev)
    base[:, in_:].view(torch.int16)[:] = NAN_BITS
    a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16).to(dev)
    b = (0.05 * torch.randn((E, out, r), generator=g)).to(torch.bfloat16).to(dev)
    unused = E - 1
    a[unused].view(torch.int16)[:] = NAN_BITS
    b[unused].view(torch.int16)[:] = NAN_BITS
    x = torch.randn((T, in_), generator=g).to(torch.bfloat16).to(dev)
    idx = torch.stack([torch.randperm(E - 1, generator=g)[:k] if E - 1 >= k else torch.zeros(k, dtype=torch.long)
                       for _ in range(T)]).to(torch.int32)
    if k >= 2:
        idx[::5, 1] = idx[::5, 0]          # every fifth token lists its first expert twice
    gates = torch.softmax(torch.randn((T, k), generator=g), 1)
    wb = base[:, :in_]
    ctx = af.Context([(wb, torch.empty_like(base)[:, :in_], a, b)], k)
    y = torch.full((T, out), float("nan"), dtype=torch.float32, device=dev)
    ctx.prefill(0, x, idx.to(dev), gates.to(dev), 2.0, y=y)
    torch.cuda.synchronize()
    _check(oracle, (wb, None, a, b), x, idx.numpy(), gates.numpy(), 2.0, y, range(T))
    ctx.close()


def test_one_7b_layer_at_the_papers_prefill_length(oracle):
    """All seven matrices of one Llama-2-7B-shaped layer, 100 tokens (the prompt length of the
    paper's latency breakdown), decisions from the router; tokens on both sides of every block
    boundary checked on all their outputs."""
    wl = wlmod.scaled_down(wlmod.WORKLOADS["llama2_7b_all"], 1)
    dev = torch.device("cuda:0")
    T = 100
    mats = [(wlmod.gen_w(wl, 0, mi, "cuda"), None, wlmod.gen_a_bank(wl, 0, mi, "cuda"), wlmod.gen_b_bank(wl, 0, mi, "cuda"))
            for mi in range(len(wl.mats))]
    ctx = af.Context([(m[0], torch.empty_like(m[0]), m[2], m[3]) for m in mats], wl.k)
    hidden, router = wlmod.gen_hidden(wl, "cuda")[:T].contiguous(), wlmod.gen_router(wl, "cuda")
    hidx, hg, idx, gates = oracle_decisions(oracle, hidden, router, wl.k)
    g = torch.Generator(device="cuda").manual_seed(11)
    worst = 0.0
    for mi, mat in enumerate(mats):
        in_ = mat[0].shape[1]
        x = hidden if in_ == wl.d else torch.randn((T, in_), generator=g, device=dev).to(torch.bfloat16)
        y = ctx.prefill(mi, x, idx, gates, wl.scale)
        torch.cuda.synchronize()
        worst = max(worst, _check(oracle, mat, x, hidx, hg, wl.scale, y, [0, 31, 32, 63, 64, 99]))
    print(f"\n[7B layer, 100 tokens] largest error {worst:.2e} of the operand magnitude")
    ctx.close()


def test_many_tokens_take_the_128_token_tiles(oracle):
    """1100 tokens on a 4096-row matrix: enough workgroups for the 128-token form of the second kernel."""
    dev = torch.device("cuda:0")
    g = torch.Generator().manual_seed(5)
    out, in_, E, r, k, T = 4096, 264, 6, 16, 2, 1100
    wb = (0.02 * torch.randn((out, in_), generator=g)).to(torch.bfloat16).to(dev)
    a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16).to(dev)
    b = (0.05 * torch.randn((E, out, r), generator=g)).to(torch.bfloat16).to(dev)
    x = torch.randn((T, in_), generator=g).to(torch.bfloat16).to(dev)
    idx = torch.stack([torch.randperm(E, generator=g)[:k] for _ in range(T)]).to(torch.int32)
    gates = torch.softmax(torch.randn((T, k), generator=g), 1)
    ctx = af.Context([(wb, torch.empty_like(wb), a, b)], k)
    y = ctx.prefill(0, x, idx.to(dev), gates.to(dev), 2.0)
    torch.cuda.synchronize()
    tokens = [0, 1, 127, 128, 129, 500, 1023, 1024, 1087, 1088, 1099]
    _check(oracle, (wb, None, a, b), x, idx.numpy(), gates.numpy(), 2.0, y, tokens)
    # same inputs, same bits: no atomics, fixed order of every sum
    y2 = ctx.prefill(0, x, idx.to(dev), gates.to(dev), 2.0)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int32), y2.view(torch.int32))
    ctx.close()


@pytest.mark.parametrize("T", [1, 100, 129, 512, 600])
def test_group_of_matrices_that_share_an_input(oracle, T):
    """Three matrices of different heights (one ragged) over one input, as the q, k and v projections of a
    GQA layer: one call for the group, every output against the oracle; token counts on both sides of the
    few-token / many-token switch (512) and of a tile boundary."""
    dev = torch.device("cuda:0")
    g = torch.Generator().manual_seed(900 + T)
    in_, E, r, k = 320, 5, 8, 2
    outs = [512, 130, 64]
    mats = []
    for out in outs:
        wb = (0.02 * torch.randn((out, in_), generator=g)).to(torch.bfloat16).to(dev)
        a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16).to(dev)
        b = (0.05 * torch.randn((E, out, r), generator=g)).to(torch.bfloat16).to(dev)
        mats.append((wb, torch.empty_like(wb), a, b))
    x = torch.randn((T, in_), generator=g).to(torch.bfloat16).to(dev)
    idx = torch.stack([torch.randperm(E, generator=g)[:k] for _ in range(T)]).to(torch.int32)
    idx[::7, 1] = idx[::7, 0]
    gates = torch.softmax(torch.randn((T, k), generator=g), 1)
    ctx = af.Context(mats, k)
    ys = [torch.full((T, out), float("nan"), dtype=torch.float32, device=dev) for out in outs]
    ctx.prefill_group([0, 1, 2], x, idx.to(dev), gates.to(dev), 2.0, ys=ys)
    torch.cuda.synchronize()
    tokens = sorted(set([0, T // 2, T - 1] + [t for t in (127, 128, 255, 256, 511, 512) if t < T]))
    for mat, y in zip(mats, ys):
        _check(oracle, (mat[0], None, mat[2], mat[3]), x, idx.numpy(), gates.numpy(), 2.0, y, tokens)
    # the group in another order writes the same bits: the cut does not depend on the order
    ys2 = ctx.prefill_group([2, 0, 1], x, idx.to(dev), gates.to(dev), 2.0)
    torch.cuda.synchronize()
    for a, b in zip(ys, [ys2[1], ys2[2], ys2[0]]):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    ctx.close()


def test_group_refuses_what_it_cannot_do():
    dev = torch.device("cuda:0")
    mk = lambda o, i: (torch.zeros((o, i), dtype=torch.bfloat16, device=dev), torch.zeros((o, i), dtype=torch.bfloat16, device=dev),
                       torch.zeros((4, 8, i), dtype=torch.bfloat16, device=dev), torch.zeros((4, o, 8), dtype=torch.bfloat16, device=dev))
    ctx = af.Context([mk(64, 64), mk(128, 64), mk(64, 128), mk(32, 64), mk(16, 64), mk(8, 64)], 2)
    x = torch.zeros((5, 64), dtype=torch.bfloat16, device=dev)
    idx = torch.zeros((5, 2), dtype=torch.int32, device=dev)
    gates = torch.zeros((5, 2), dtype=torch.float32, device=dev)
    with pytest.raises(af.AdafuseError):
        ctx.prefill_group([0, 2], x, idx, gates, 2.0)            # different input widths
    with pytest.raises(af.AdafuseError):
        ctx.prefill_group([0, 0], x, idx, gates, 2.0)            # the same matrix twice
    with pytest.raises(af.AdafuseError):
        ctx.prefill_group([0, 1, 3, 4, 5], x, idx, gates, 2.0)   # more than four
    with pytest.raises(af.AdafuseError):
        ctx.prefill_group([], x, idx, gates, 2.0)
    with pytest.raises(af.AdafuseError):
        ctx.prefill_group([0, 9], x, idx, gates, 2.0)            # no such matrix
    ys = ctx.prefill_group([0, 1, 3, 4], x, idx, gates, 2.0)     # four is fine
    torch.cuda.synchronize()
    assert [tuple(y.shape) for y in ys] == [(5, 64), (5, 128), (5, 32), (5, 16)] and all(bool((y == 0).all()) for y in ys)
    ctx.close()


def test_prefill_refuses_what_it_cannot_do():
    dev = torch.device("cuda:0")
    w = torch.zeros((64, 64), dtype=torch.bfloat16, device=dev)
    a = torch.zeros((4, 8, 64), dtype=torch.bfloat16, device=dev)
    b = torch.zeros((4, 64, 8), dtype=torch.bfloat16, device=dev)
    x = torch.zeros((5, 64), dtype=torch.bfloat16, device=dev)
    idx = torch.zeros((5, 2), dtype=torch.int32, device=dev)
    gates = torch.zeros((5, 2), dtype=torch.float32, device=dev)
    ctx = af.Context([(w, torch.empty_like(w), a, b)], 2)
    with pytest.raises(af.AdafuseError):
        ctx.prefill(1, x, idx, gates, 2.0)                                   # no such matrix
    with pytest.raises(af.AdafuseError):
        ctx.prefill(0, x, idx, gates, 2.0, workspace=torch.empty(16, dtype=torch.uint8, device=dev))   # workspace too small
    with pytest.raises(af.AdafuseError):
        ctx.prefill(0, x, torch.zeros((5, 3), dtype=torch.int32, device=dev),
                    torch.zeros((5, 3), dtype=torch.float32, device=dev), 2.0)   # k beyond k_max
    y = ctx.prefill(0, x[:0], idx[:0], gates[:0], 2.0)                        # no tokens: nothing to do
    assert y.shape == (0, 64)
    ctx.close()
    inplace = af.Context([(w, w, a, b)], 2)
    with pytest.raises(af.AdafuseError):
        inplace.prefill(0, x, idx, gates, 2.0)                               # the base weights are gone in place
    inplace.close()
