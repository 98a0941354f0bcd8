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
