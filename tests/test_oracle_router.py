"""Pins for the router oracle (Eq.1's Softmax(TopK(W_g x)) applied once per token)."""
import os

import numpy as np
import pytest
import torch
from scipy.special import softmax

import adafuse_workloads as wlmod

GOLD = os.path.join(os.path.dirname(__file__), "golden", "router_worked_example.txt")


def _bf16_bits(x):
    return wlmod.bits(torch.tensor(np.asarray(x, np.float32)).to(torch.bfloat16))


def _rand(T, d, E, seed):
    g = torch.Generator().manual_seed(seed)
    h = torch.randn((T, d), generator=g).to(torch.bfloat16)
    w = (0.02 * torch.randn((E, d), generator=g)).to(torch.bfloat16)
    return h, w


def test_worked_example_from_golden_file(oracle):
    gold = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        gold[key] = [float(v) for v in vals]
    h = _bf16_bits([[1.0, 2.0]])
    w = _bf16_bits([[1, 0], [0, 1], [0.5, 0.5], [-1, 0.25]])
    r0 = oracle.pregate(h, w, 2, 0)
    assert r0["logits"][0].tolist() == gold["logits"]
    assert r0["idx"][0].tolist() == [int(v) for v in gold["idx"]]
    assert np.allclose(r0["gates"][0], gold["gates_softmax_over_topk"], rtol=0, atol=1e-15)
    r1 = oracle.pregate(h, w, 2, 1)
    assert r1["idx"][0].tolist() == [1, 2]
    assert np.allclose(r1["gates"][0], gold["gates_topk_of_softmax"], rtol=0, atol=1e-11)


def test_logits_match_library_matmul(oracle):
    h, w = _rand(16, 256, 4, 0)
    res = oracle.pregate(wlmod.bits(h), wlmod.bits(w), 2)
    ref = h.double().numpy() @ w.double().numpy().T
    assert np.allclose(res["logits"], ref, rtol=1e-13, atol=1e-14)
    assert np.array_equal(res["logits32"], res["logits"].astype(np.float32))


@pytest.mark.parametrize("E,k", [(4, 2), (8, 2), (16, 4), (8, 8), (5, 1)])
def test_topk_is_stable_argsort_and_gates_are_softmax(oracle, E, k):
    h, w = _rand(64, 128, E, E * 10 + k)
    res = oracle.pregate(wlmod.bits(h), wlmod.bits(w), k, 0)
    l32 = res["logits32"].astype(np.float64)
    order = np.argsort(-l32, axis=1, kind="stable")[:, :k]
    assert np.array_equal(res["idx"], order)
    for t in range(l32.shape[0]):
        assert len(set(res["idx"][t].tolist())) == k
        kept = l32[t, order[t]]
        assert np.allclose(res["gates"][t], softmax(kept), rtol=1e-14)
    assert np.allclose(res["gates"].sum(1), 1.0, rtol=1e-14)
    assert np.array_equal(res["gates32"], res["gates"].astype(np.float32))
    # the other reading: softmax over all E, then keep k; same idx, renormalising gives mode 0
    res1 = oracle.pregate(wlmod.bits(h), wlmod.bits(w), k, 1)
    assert np.array_equal(res1["idx"], res["idx"])
    full = softmax(l32, axis=1)
    assert np.allclose(res1["gates"], np.take_along_axis(full, order, 1), rtol=1e-14)
    assert np.allclose(res1["gates"] / res1["gates"].sum(1, keepdims=True), res["gates"], rtol=1e-13)
    if k == E:
        assert np.allclose(res["gates"], res1["gates"], rtol=1e-14)


def test_two_experts_reduce_to_sigmoid(oracle):
    h, w = _rand(32, 64, 2, 7)
    res = oracle.pregate(wlmod.bits(h), wlmod.bits(w), 2, 0)
    l = res["logits32"].astype(np.float64)
    hi = l.max(1)
    lo = l.min(1)
    assert np.allclose(res["gates"][:, 0], 1.0 / (1.0 + np.exp(lo - hi)), rtol=1e-14)


def test_constant_shift_leaves_selection_and_gates(oracle):
    # an extra input feature fixed at 1 with the same router weight c for every
    # expert shifts every logit by c
    h, w = _rand(32, 64, 8, 11)
    base = oracle.pregate(wlmod.bits(h), wlmod.bits(w), 3, 0)
    h2 = torch.cat([h, torch.ones(32, 1, dtype=torch.bfloat16)], 1)
    w2 = torch.cat([w, torch.full((8, 1), 4.0, dtype=torch.bfloat16)], 1)
    sh = oracle.pregate(wlmod.bits(h2), wlmod.bits(w2), 3, 0)
    assert np.allclose(sh["logits"], base["logits"] + 4.0, rtol=0, atol=1e-13)
    assert np.array_equal(sh["idx"], base["idx"])
    assert np.allclose(sh["gates"], base["gates"], rtol=0, atol=1e-6)   # fp32 logit rounding moves


def test_exact_tie_takes_lower_index(oracle):
    h, w = _rand(8, 64, 6, 5)
    w[1] = w[4]                      # identical rows -> identical logits
    w[3] = w[4]
    res = oracle.pregate(wlmod.bits(h), wlmod.bits(w), 6, 0)
    for t in range(8):
        order = res["idx"][t].tolist()
        p = [order.index(e) for e in (1, 3, 4)]
        assert p == sorted(p) and p[1] == p[0] + 1 and p[2] == p[1] + 1
        assert res["logits32"][t, 1] == res["logits32"][t, 3] == res["logits32"][t, 4]


def test_argument_errors(oracle):
    h, w = _rand(2, 8, 4, 1)
    with pytest.raises(ValueError):
        oracle.pregate(wlmod.bits(h), wlmod.bits(w), 5)
    with pytest.raises(ValueError):
        oracle.pregate(wlmod.bits(h), wlmod.bits(w), 0)
    with pytest.raises(ValueError):
        oracle.pregate(wlmod.bits(h), wlmod.bits(w), 2, 7)
