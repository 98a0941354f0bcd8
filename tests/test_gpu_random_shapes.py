"""GPU parity on seeded random models: several matrices of unrelated, ragged shapes in ONE context
(so one launch walks a tile table with edge tiles of every kind, dealt over the XCDs), random bank
size, rank and top-k, padded leading dimensions, every kernel and both forms of the default one; out
of place (MERGE, SWAP, UNMERGE) and in place (SWAP).  Every element is compared with the oracle."""
import numpy as np
import pytest
import torch

import adafuse_workloads as wlmod
import paper_2603_11873_amd as af
from gpu_util import Tally, compare, compare_inplace

pytestmark = pytest.mark.gpu

ULP_TOL = 1
NAN_BITS = 0x7FC1
RANKS = [4, 8, 16, 32, 64, 128]


def _draw_model(seed):
    rng = np.random.default_rng(seed)
    r = int(rng.choice(RANKS))
    E = int(rng.integers(1, 10))
    k = int(rng.integers(1, min(E, 4) + 1))
    n_mats = int(rng.integers(2, 5))
    shapes = []
    for _ in range(n_mats):
        out = int(rng.integers(1, 330))
        in_ = 8 * int(rng.integers(1, 90))
        ldw = in_ + 8 * int(rng.integers(0, 3))
        shapes.append((out, in_, ldw))
    return rng, r, E, k, shapes


def _tensors(g, shapes, E, r):
    mats = []
    for out, in_, ldw in shapes:
        base = (0.02 * torch.randn((out, ldw), generator=g)).to(torch.bfloat16).cuda()
        if ldw > in_:
            base[:, in_:].view(torch.int16)[:] = NAN_BITS   # padding columns: never read, never written
        a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16).cuda()
        b = (0.05 * torch.randn((E, out, r), generator=g)).to(torch.bfloat16).cuda()
        mats.append((base, a, b))
    return mats


def _decision(rng, E, k):
    idx = rng.permutation(E)[:k].astype(np.int32)
    z = rng.standard_normal(k)
    gates = (np.exp(z) / np.exp(z).sum()).astype(np.float32)
    return idx, gates


@pytest.mark.parametrize("seed", range(24))
@pytest.mark.parametrize("kernel,form", [(af.KERNEL_GEMM, 0), (af.KERNEL_GEMM, 4), (af.KERNEL_GEMM, 3), (af.KERNEL_MFMA, 0), (af.KERNEL_VALU, 0)])
def test_random_model_out_of_place(oracle, seed, kernel, form):
    rng, r, E, k, shapes = _draw_model(1000 + seed)
    g = torch.Generator().manual_seed(seed)
    mats = _tensors(g, shapes, E, r)
    works = [torch.empty_like(m[0]) for m in mats]
    ctx = af.Context([(m[0][:, :s[1]], w[:, :s[1]], m[1], m[2]) for m, w, s in zip(mats, works, shapes)], k)
    try:
        ctx.set_kernel(kernel)
        if form:
            ctx.set_option(af.OPT_GEMM_FORM, form)
    except af.AdafuseError:
        ctx.close()
        pytest.skip("this kernel or form is not built for this (r, k)")
    if kernel == af.KERNEL_VALU and k * r * 768 > 65536:
        ctx.close()
        pytest.skip("more than the baseline kernel can stage in LDS")
    dev = lambda x: torch.as_tensor(x, device="cuda:0")
    prev, nxt = _decision(rng, E, k), _decision(rng, E, k)
    tally = Tally()
    for mode, dec in ((af.MERGE, prev), (af.SWAP, nxt)):
        for w in works:
            w.view(torch.int16).fill_(NAN_BITS)
        # a previous decision bit-identical to the next one is the documented early-out (W_work is taken to hold
        # the result already): with a one-expert bank the two draws coincide, and the scribble above would stay
        same = mode == af.SWAP and np.array_equal(prev[0], dec[0]) and np.array_equal(prev[1], dec[1])
        p_idx, p_gates = (None, None) if same else (dev(prev[0]), dev(prev[1]))
        try:
            ctx.fused_switch(p_idx, p_gates, dev(dec[0]), dev(dec[1]), k, 2.0, mode)
        except af.AdafuseError:      # refused before any launch: a form that is not built for this (rank, terms)
            assert form != 0
            ctx.close()
            pytest.skip("this form is not built for this (r, k)")
        torch.cuda.synchronize()
        for (base, a, b), w, (out, in_, ldw) in zip(mats, works, shapes):
            tally.add(compare(oracle, wlmod.bits(base[:, :in_]), wlmod.bits(a), wlmod.bits(b), wlmod.bits(w[:, :in_]),
                              dec[0], dec[1], 2.0), ULP_TOL, (seed, mode, out, in_))
            if ldw > in_:
                assert bool((w[:, in_:].view(torch.int16) == NAN_BITS).all())
    tally.finish(1e-4)
    ctx.fused_switch(None, None, None, None, k, 2.0, af.UNMERGE)
    torch.cuda.synchronize()
    for (base, a, b), w, (out, in_, ldw) in zip(mats, works, shapes):
        assert torch.equal(w[:, :in_].contiguous().view(torch.int16), base[:, :in_].contiguous().view(torch.int16))
    ctx.close()


@pytest.mark.parametrize("seed", range(24))
@pytest.mark.parametrize("kernel,form", [(af.KERNEL_GEMM, 0), (af.KERNEL_GEMM, 4), (af.KERNEL_MFMA, 0), (af.KERNEL_VALU, 0)])
def test_random_model_in_place(oracle, seed, kernel, form):
    """w_work == w_base: a SWAP removes the previous token's experts and adds the next one's in one pass
    (up to 2k terms; the two decisions share experts by chance)."""
    rng, r, E, k, shapes = _draw_model(2000 + seed)
    g = torch.Generator().manual_seed(100 + seed)
    mats = _tensors(g, shapes, E, r)
    prev, nxt = _decision(rng, E, k), _decision(rng, E, k)
    befores, ws = [], []
    for (base, a, b), (out, in_, ldw) in zip(mats, shapes):
        before = oracle.merge(wlmod.bits(base[:, :in_]), wlmod.bits(a), wlmod.bits(b), prev[0], prev[1], 2.0)
        befores.append(before)
        w = base.clone()
        w[:, :in_] = wlmod.from_bits(before, "cuda:0")
        ws.append(w)
    ctx = af.Context([(w[:, :s[1]], w[:, :s[1]], m[1], m[2]) for m, w, s in zip(mats, ws, shapes)], k)
    try:
        ctx.set_kernel(kernel)
        if form:
            ctx.set_option(af.OPT_GEMM_FORM, form)
    except af.AdafuseError:
        ctx.close()
        pytest.skip("this kernel or form is not built for this (r, k) in place")
    if kernel == af.KERNEL_VALU and 2 * k * r * 768 > 65536:
        ctx.close()
        pytest.skip("more than the baseline kernel can stage in LDS")
    dev = lambda x: torch.as_tensor(x, device="cuda:0")
    try:
        ctx.fused_switch(dev(prev[0]), dev(prev[1]), dev(nxt[0]), dev(nxt[1]), k, 2.0, af.SWAP)
    except af.AdafuseError:
        assert form != 0
        ctx.close()
        pytest.skip("this form is not built for this (r, k)")
    torch.cuda.synchronize()
    tally = Tally()
    for (base, a, b), w, before, (out, in_, ldw) in zip(mats, ws, befores, shapes):
        tally.add(compare_inplace(oracle, before, wlmod.bits(a), wlmod.bits(b), wlmod.bits(w[:, :in_]), prev, nxt, 2.0),
                  ULP_TOL, (seed, out, in_))
        if ldw > in_:
            assert bool((w[:, in_:].view(torch.int16) == NAN_BITS).all())
    tally.finish(1e-4)
    ctx.close()


@pytest.mark.parametrize("seed", range(16))
def test_random_prefill_groups(oracle, seed):
    """adafuse_prefill_group on random groups (one to four matrices of random heights over one random input
    width), random token counts on both sides of the few-token / many-token switch, random rank and top-k;
    sampled tokens against the oracle's token-by-token Eq.2, every output of those tokens."""
    from test_gpu_prefill import _check
    rng = np.random.default_rng(3000 + seed)
    r = int(rng.choice(RANKS))
    E = int(rng.integers(1, 9))
    k = int(rng.integers(1, min(E, 4) + 1))
    in_ = 8 * int(rng.integers(1, 70))
    T = int(rng.choice([1, 7, 64, 100, 128, 129, 257, 512, 513, 640]))
    outs = [int(rng.integers(1, 600)) for _ in range(int(rng.integers(1, 5)))]
    g = torch.Generator().manual_seed(500 + seed)
    dev = torch.device("cuda:0")
    mats = []
    for out in outs:
        wb = (0.02 * torch.randn((out, in_), generator=g)).to(torch.bfloat16).to(dev)
        a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16).to(dev)
        b = (0.05 * torch.randn((E, out, r), generator=g)).to(torch.bfloat16).to(dev)
        mats.append((wb, torch.empty_like(wb), a, b))
    x = torch.randn((T, in_), generator=g).to(torch.bfloat16).to(dev)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    z = rng.standard_normal((T, k))
    gates = (np.exp(z) / np.exp(z).sum(1, keepdims=True)).astype(np.float32)
    ctx = af.Context(mats, k)
    ys = [torch.full((T, out), float("nan"), dtype=torch.float32, device=dev) for out in outs]
    ctx.prefill_group(list(range(len(outs))), x, torch.from_numpy(idx).to(dev), torch.from_numpy(gates).to(dev), 2.0, ys=ys)
    torch.cuda.synchronize()
    tokens = sorted({0, T // 3, T - 1} | {t for t in (127, 128, 511, 512) if t < T})
    for mat, y in zip(mats, ys):
        _check(oracle, (mat[0], None, mat[2], mat[3]), x, idx, gates, 2.0, y, tokens)
    ctx.close()
