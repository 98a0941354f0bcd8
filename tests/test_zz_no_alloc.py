"""The entry point that allocates nothing: adafuse_forward_dynamic_static against
adafuse_forward_dynamic (same launches, z in the library's built-in scratch instead of a caller
workspace), through the C ABI, two calls in a row, the second on a smaller model."""
import pytest
import torch

import adafuse_workloads as wlmod
import paper_2603_11873_amd as af

pytestmark = pytest.mark.gpu


def _model(wl, gen_device):
    dev = torch.device("cuda:0")
    mats = []
    for layer in range(wl.layers):
        for mi in range(len(wl.mats)):
            wb = wlmod.gen_w(wl, layer, mi, gen_device).to(dev)
            mats.append((wb, torch.empty_like(wb), wlmod.gen_a_bank(wl, layer, mi, gen_device).to(dev),
                         wlmod.gen_b_bank(wl, layer, mi, gen_device).to(dev)))
    return mats


def _both_ways(ctx, mats, idx, gates, scale, r, seed):
    dev = mats[0][0].device
    g = torch.Generator().manual_seed(seed)
    x = torch.cat([torch.randn(wb.shape[1], generator=g) for wb, _, _, _ in mats]).to(torch.bfloat16).to(dev)
    n_out = sum(wb.shape[0] for wb, _, _, _ in mats)
    y_ws = torch.full((n_out,), float("nan"), dtype=torch.float32, device=dev)
    y_st = torch.full((n_out,), float("nan"), dtype=torch.float32, device=dev)
    z = torch.zeros(len(idx) * r, dtype=torch.float32, device=dev)
    ctx.forward_dynamic(idx, gates, scale, x, y_ws, z)
    before = torch.cuda.memory_allocated()
    ctx.forward_dynamic_static(idx, gates, scale, x, y_st)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert torch.isfinite(y_ws).all()
    # same kernels, same order of operations: the outputs agree to the bit
    assert torch.equal(y_st.view(torch.int32), y_ws.view(torch.int32))


def test_static_scratch_entry_point_matches_the_workspace_one():
    big = wlmod.scaled_down(wlmod.WORKLOADS["llama3_8b_gqa_all"], 1)     # k r = 64 floats of scratch
    small = wlmod.WORKLOADS["toy"]                                       # k r = 8
    m_big, m_small = _model(big, "cuda"), _model(small, "cpu")
    c_big, c_small = af.Context(m_big, big.k), af.Context(m_small, small.k)
    _both_ways(c_big, m_big, [5, 0, 11, 2], [0.4, 0.3, 0.2, 0.1], big.scale, big.r, 1)
    _both_ways(c_small, m_small, [3, 1], [0.75, 0.25], small.scale, small.r, 2)    # smaller input, stale scratch behind it
    _both_ways(c_big, m_big, [1], [1.0], big.scale, big.r, 3)
    c_big.close()
    c_small.close()


def test_static_scratch_entry_point_rejects_what_the_other_rejects():
    small = wlmod.WORKLOADS["toy"]
    mats = _model(small, "cpu")
    ctx = af.Context(mats, small.k)
    x = torch.zeros(sum(m[0].shape[1] for m in mats), dtype=torch.bfloat16, device="cuda:0")
    y = torch.zeros(sum(m[0].shape[0] for m in mats), dtype=torch.float32, device="cuda:0")
    with pytest.raises(af.AdafuseError):
        ctx.forward_dynamic_static([0, 1, 2], [0.3, 0.3, 0.4], 2.0, x, y)     # k beyond the context's k_max
    with pytest.raises(af.AdafuseError):
        ctx.forward_dynamic_static([0, 4], [0.5, 0.5], 2.0, x, y)             # expert index out of range
    ctx.close()
