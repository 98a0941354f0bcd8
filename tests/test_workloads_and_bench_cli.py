"""Host-side checks that need no GPU: the workload table against the sizes the
configurations imply, the input generators' determinism, and bench.py's refusal of
more than one GPU."""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

import adafuse_workloads as wlmod

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _by_hand(layers, shapes, k, r):
    elements = layers * sum(o * i for o, i in shapes)
    slices = layers * sum(2 * k * r * (o + i) for o, i in shapes)
    return elements, 4 * elements + slices


@pytest.mark.parametrize("name,layers,shapes,E,r,k,T", [
    ("toy", 2, [(256, 256)] * 4, 4, 4, 2, 16),
    ("llama2_7b_attn", 32, [(4096, 4096)] * 4, 8, 8, 2, 64),
    ("llama2_7b_all", 32, [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)], 8, 8, 2, 256),
    ("llama3_8b_gqa_all", 32, [(4096, 4096), (1024, 4096), (1024, 4096), (4096, 4096)] + [(14336, 4096)] * 2 + [(4096, 14336)],
     16, 16, 4, 256),
    ("llama2_13b_all", 40, [(5120, 5120)] * 4 + [(13824, 5120)] * 2 + [(5120, 13824)], 8, 16, 2, 512),
])
def test_workload_table_matches_the_configurations(name, layers, shapes, E, r, k, T):
    wl = wlmod.WORKLOADS[name]
    assert (wl.layers, wl.E, wl.r, wl.k, wl.T) == (layers, E, r, k, T)
    assert [(o, i) for _, o, i in wl.mats] == shapes
    elements, alg = _by_hand(layers, shapes, k, r)
    assert wl.elements == elements and wl.algorithmic_bytes == alg
    assert wl.n_mats == layers * len(shapes)
    assert wl.flops == 2 * k * r * elements
    assert wl.scale == 2.0


def test_sizes_the_roofline_is_quoted_on():
    # bytes one switch must move: W read once and written once, each selected slice read once
    assert wlmod.WORKLOADS["llama2_7b_attn"].algorithmic_bytes == 8_623_489_024
    assert wlmod.WORKLOADS["llama2_7b_all"].algorithmic_bytes == 25_983_975_424
    assert wlmod.WORKLOADS["llama2_7b_all"].elements == 6_476_005_376
    assert wlmod.WORKLOADS["llama2_13b_all"].elements == 12_687_769_600
    assert wlmod.ORDER == ["toy", "llama2_7b_attn", "llama2_7b_all", "llama3_8b_gqa_all", "llama2_13b_all"]


def test_generators_are_deterministic_and_independent_per_tensor():
    wl = wlmod.WORKLOADS["toy"]
    a = wlmod.gen_w(wl, 1, 2)
    assert torch.equal(a.view(torch.int16), wlmod.gen_w(wl, 1, 2).view(torch.int16))
    assert not torch.equal(a.view(torch.int16), wlmod.gen_w(wl, 1, 3).view(torch.int16))
    assert not torch.equal(a.view(torch.int16), wlmod.gen_w(wl, 0, 2).view(torch.int16))
    assert wlmod.gen_a_bank(wl, 0, 0).shape == (wl.E, wl.r, 256)
    assert wlmod.gen_b_bank(wl, 0, 0).shape == (wl.E, 256, wl.r)
    assert wlmod.gen_router(wl).shape == (wl.E, wl.d) and wlmod.gen_hidden(wl).shape == (wl.T, wl.d)
    # the recipe's scales, loosely (bf16 rounding and 64 K samples)
    assert abs(float(a.float().std()) - 0.02) < 0.002
    assert abs(float(wlmod.gen_a_bank(wl, 0, 0).float().std()) - 256 ** -0.5) < 0.005
    assert abs(float(wlmod.gen_b_bank(wl, 0, 0).float().std()) - 0.01) < 0.001


def test_bits_round_trip():
    x = torch.tensor([0.0, -0.0, 1.0, -2.5, 3.0e-39, float("inf")], dtype=torch.float32).to(torch.bfloat16)
    b = wlmod.bits(x)
    assert b.dtype == np.uint16 and b[1] == 0x8000 and b[2] == 0x3F80
    assert torch.equal(wlmod.from_bits(b).view(torch.int16), x.view(torch.int16))


def test_repeating_hidden_states_follow_the_recipe():
    wl = wlmod.WORKLOADS["llama2_13b_all"]
    small = wlmod.Workload("small", 1, 64, wl.mats, wl.E, wl.r, wl.k, 200, wl.seed, wl.scale, wl.repeat_prob)
    h = wlmod.gen_hidden(small).float()
    # a repeated token is its predecessor plus a small perturbation: cosine close to 1
    cos = torch.nn.functional.cosine_similarity(h[1:], h[:-1], dim=1)
    frac = float((cos > 0.9).float().mean())
    assert 0.15 < frac < 0.45   # about 30 % of the tokens


@pytest.mark.parametrize("flag", ["2", "8"])
def test_bench_refuses_more_than_one_gpu(flag):
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", flag],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode == 2
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_bench_refuses_a_multi_rank_launch():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0")
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert res.returncode == 2 and "ONE GPU" in res.stderr
