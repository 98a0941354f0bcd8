"""The decode step (router + fused switch) captured in a HIP graph and replayed.

Both entry points only enqueue kernels (no allocation, no synchronisation, no memset),
so a serving loop can capture them once; the toy workload is launch-bound and gains
from it.  Every replay is checked, with eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

import adafuse_workloads as wlmod
import paper_2603_11873_amd as af
from gpu_util import DeviceModel, Tally, check_full, oracle_decisions

pytestmark = pytest.mark.gpu

ULP_TOL = 1
MAX_DIFF_FRACTION = 0.01


@pytest.mark.parametrize("kernel,rank", [(af.KERNEL_GEMM, 4), (af.KERNEL_MFMA, 4), (af.KERNEL_VALU, 4), (af.KERNEL_GEMM, 64)])
def test_captured_decode_step_replays_correctly(oracle, kernel, rank):
    """rank 4: the toy workload; rank 64: the same matrices with experts of the paper-typical rank, which the
    default kernel runs in its overlapped form (W tile transferred straight into LDS)."""
    toy = wlmod.WORKLOADS["toy"]
    wl = toy if rank == toy.r else wlmod.Workload("toy_r64", toy.layers, toy.d, toy.mats, toy.E, rank, toy.k, toy.T, 9,
                                                  toy.scale, toy.repeat_prob)
    m = DeviceModel(wl)
    m.ctx.set_kernel(kernel)
    if rank == 64:
        assert m.ctx.switch_kernel_name(wl.k, af.SWAP) == "switch_gemm_overlap_kernel"
    dev = m.hidden.device
    hidx, hg, _, _ = oracle_decisions(oracle, m.hidden, m.router, wl.k)

    # fixed-address buffers the graph reads and writes
    tok = torch.empty((1, wl.d), dtype=torch.bfloat16, device=dev)
    idx_prev = torch.zeros((1, wl.k), dtype=torch.int32, device=dev)
    gates_prev = torch.zeros((1, wl.k), dtype=torch.float32, device=dev)
    idx_next = torch.zeros((1, wl.k), dtype=torch.int32, device=dev)
    gates_next = torch.zeros((1, wl.k), dtype=torch.float32, device=dev)

    def step():
        s = torch.cuda.current_stream()
        af.pregate(tok, m.router, wl.k, out=(idx_next, gates_next, None), stream=s)
        m.ctx.fused_switch(idx_prev[0], gates_prev[0], idx_next[0], gates_next[0], wl.k, wl.scale, af.SWAP, stream=s)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        tok.copy_(m.hidden[0:1])
        step()                      # eager warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()

    tally = Tally()
    for t in (3, 4, 9, 4, 15):
        # eager work between the replays: new inputs, and a scribble over W_work so a replay that did nothing shows
        tok.copy_(m.hidden[t:t + 1])
        idx_prev.copy_(idx_next)
        gates_prev.copy_(gates_next)
        for _, ww, _, _ in m.mats:
            ww.view(torch.int16).fill_(0x7FC1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(idx_next.cpu().numpy()[0], hidx[t])
        assert np.allclose(gates_next.cpu().numpy()[0], hg[t], rtol=1e-6, atol=0)
        for mat in m.mats:
            tally.add(check_full(oracle, mat, hidx[t], hg[t], wl.scale), ULP_TOL, (kernel, t))
    tally.finish(MAX_DIFF_FRACTION)

    # the eager result of the same step is bit-identical to the replayed one
    replayed = [ww.clone() for _, ww, _, _ in m.mats]
    for _, ww, _, _ in m.mats:
        ww.view(torch.int16).fill_(0x7FC1)
    idx_prev.zero_()                # any decision other than token 15's: the step must do its work again
    gates_prev.zero_()
    step()
    torch.cuda.synchronize()
    for (_, ww, _, _), rep in zip(m.mats, replayed):
        assert torch.equal(ww.view(torch.int16), rep.view(torch.int16))
    m.close()


@pytest.mark.parametrize("T", [100, 600])
def test_captured_prefill_replays_correctly(T):
    """adafuse_pregate + adafuse_prefill_group (three matrices over one input) captured once and replayed on
    new inputs, in the few-token form (two launches) and in the many-token form; every replay equals the
    eager call on the same inputs bit for bit (fixed order of every sum), with eager work in between."""
    dev = torch.device("cuda:0")
    g = torch.Generator().manual_seed(40 + T)
    in_, E, r, k = 320, 6, 8, 2
    outs = [512, 130, 64]
    mats = []
    for out in outs:
        wb = (0.02 * torch.randn((out, in_), generator=g)).to(torch.bfloat16).to(dev)
        a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16).to(dev)
        b = (0.05 * torch.randn((E, out, r), generator=g)).to(torch.bfloat16).to(dev)
        mats.append((wb, torch.empty_like(wb), a, b))
    router = (0.02 * torch.randn((E, in_), generator=g)).to(torch.bfloat16).to(dev)
    ctx = af.Context(mats, k)
    xs = [torch.randn((T, in_), generator=g).to(torch.bfloat16).to(dev) for _ in range(3)]
    x = torch.empty_like(xs[0])
    idx = torch.zeros((T, k), dtype=torch.int32, device=dev)
    gates = torch.zeros((T, k), dtype=torch.float32, device=dev)
    ys = [torch.empty((T, out), dtype=torch.float32, device=dev) for out in outs]
    ws = torch.empty(ctx.prefill_group_workspace_bytes([0, 1, 2], T, k), dtype=torch.uint8, device=dev)

    def step():
        s = torch.cuda.current_stream()
        af.pregate(x, router, k, out=(idx, gates, None), stream=s)
        ctx.prefill_group([0, 1, 2], x, idx, gates, 2.0, ys=ys, workspace=ws, stream=s)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        x.copy_(xs[0])
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for which in (1, 2, 1, 0):
        x.copy_(xs[which])
        for y in ys:
            y.fill_(float("nan"))
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        replayed = [y.clone() for y in ys]
        assert all(bool(torch.isfinite(y).all()) for y in replayed)
        for y in ys:
            y.fill_(float("nan"))
        step()
        torch.cuda.synchronize()
        for a, b in zip(ys, replayed):
            assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    ctx.close()
