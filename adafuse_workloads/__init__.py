"""Seeded synthetic workloads for the AdaFuse fused-switch path.

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: it only names the five workload shapes and
draws random tensors (fp32 normal draws, rounded once to bf16).  The one thing it
looks at is whether a drawn hidden state makes a clear-cut routing decision (a
library fp64 matmul and a sort: gen_hidden redraws near-tie tokens), which is a
property of the inputs, not a step of the path.  The paper's
own workload (Llama2-7B fine-tuned experts, ShareGPT prompts; section
"Experiment Setup") is not available offline and is not needed: the cost and
the correctness of the switch depend on shapes and value ranges only.

Recipe (all tensors drawn in fp32, rounded to bf16 with round-to-nearest-even):
  W ~ N(0, 0.02^2)      A_e ~ N(0, 1/in)      B_e ~ N(0, 0.01^2)
  W_router ~ N(0, 0.02^2)      hidden ~ N(0, 1)
One torch.Generator per (config seed, tensor kind, layer, matrix), so any tensor
can be regenerated alone.  Draws made on "cpu" and on "cuda" use different
streams (torch's generators differ per device); each test states which it uses.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np
import torch

KIND_W, KIND_A, KIND_B, KIND_ROUTER, KIND_HIDDEN, KIND_REPEAT = range(6)


@dataclass(frozen=True)
class Workload:
    name: str
    layers: int
    d: int                                   # router input width
    mats: Tuple[Tuple[str, int, int], ...]   # per layer: (module, out, in)
    E: int
    r: int
    k: int
    T: int                                   # tokens in the switch sequence
    seed: int
    scale: float = 2.0
    repeat_prob: float = 0.0                 # P(token t is a small perturbation of t-1)

    def matrix_list(self) -> List[Tuple[int, str, int, int]]:
        return [(l, n, o, i) for l in range(self.layers) for (n, o, i) in self.mats]

    @property
    def n_mats(self) -> int:
        return self.layers * len(self.mats)

    @property
    def elements(self) -> int:
        return self.layers * sum(o * i for _, o, i in self.mats)

    @property
    def algorithmic_bytes(self) -> int:
        """HBM bytes one switch must move: W read once + written once (bf16)
        plus each selected A/B slice read once."""
        per_layer = sum(4 * o * i + 2 * self.k * self.r * (o + i) for _, o, i in self.mats)
        return self.layers * per_layer

    @property
    def flops(self) -> int:
        return 2 * self.k * self.r * self.elements


def _attn(d, kv=None):
    kv = d if kv is None else kv
    return (("q", d, d), ("k", kv, d), ("v", kv, d), ("o", d, d))


def _mlp(d, f):
    return (("gate", f, d), ("up", f, d), ("down", d, f))


WORKLOADS = {
    "toy": Workload("toy", 2, 256, _attn(256), E=4, r=4, k=2, T=16, seed=0),
    "llama2_7b_attn": Workload("llama2_7b_attn", 32, 4096, _attn(4096), E=8, r=8, k=2, T=64, seed=2),
    "llama2_7b_all": Workload("llama2_7b_all", 32, 4096, _attn(4096) + _mlp(4096, 11008),
                              E=8, r=8, k=2, T=256, seed=3),
    "llama3_8b_gqa_all": Workload("llama3_8b_gqa_all", 32, 4096, _attn(4096, 1024) + _mlp(4096, 14336),
                                  E=16, r=16, k=4, T=256, seed=4),
    "llama2_13b_all": Workload("llama2_13b_all", 40, 5120, _attn(5120) + _mlp(5120, 13824),
                               E=8, r=16, k=2, T=512, seed=5, repeat_prob=0.3),
}
# beyond the five graded configurations: the ranks the paper calls typical (64 or 128, top-2),
# and rank 32 between them and the graded ones
WORKLOADS["llama2_7b_all_r32"] = Workload("llama2_7b_all_r32", 32, 4096, _attn(4096) + _mlp(4096, 11008),
                                          E=8, r=32, k=2, T=64, seed=8)
WORKLOADS["llama2_7b_all_r64"] = Workload("llama2_7b_all_r64", 32, 4096, _attn(4096) + _mlp(4096, 11008),
                                          E=8, r=64, k=2, T=64, seed=6)
WORKLOADS["llama2_7b_all_r128"] = Workload("llama2_7b_all_r128", 32, 4096, _attn(4096) + _mlp(4096, 11008),
                                           E=4, r=128, k=2, T=64, seed=7)
ORDER = ["toy", "llama2_7b_attn", "llama2_7b_all", "llama3_8b_gqa_all", "llama2_13b_all"]


def scaled_down(wl: Workload, layers: int, name: str = None) -> Workload:
    """Same per-layer shapes with fewer layers (for tests that cannot hold the full model)."""
    return Workload(name or f"{wl.name}_L{layers}", layers, wl.d, wl.mats, wl.E, wl.r, wl.k,
                    wl.T, wl.seed, wl.scale, wl.repeat_prob)


def _gen(seed: int, kind: int, layer: int, mat: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(((seed * 7 + kind) * 4099 + layer) * 17 + mat + 0x5AD0)
    return g


def _normal_bf16(shape, std, gen, device) -> torch.Tensor:
    x = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    return (x * std).to(torch.bfloat16)


def gen_w(wl: Workload, layer: int, mat: int, device="cpu") -> torch.Tensor:
    _, o, i = wl.mats[mat]
    return _normal_bf16((o, i), 0.02, _gen(wl.seed, KIND_W, layer, mat, device), device)


def gen_a_bank(wl: Workload, layer: int, mat: int, device="cpu") -> torch.Tensor:
    """[E][r][in], std 1/sqrt(in)."""
    _, o, i = wl.mats[mat]
    return _normal_bf16((wl.E, wl.r, i), float(i) ** -0.5, _gen(wl.seed, KIND_A, layer, mat, device), device)


def gen_b_bank(wl: Workload, layer: int, mat: int, device="cpu") -> torch.Tensor:
    """[E][out][r], std 0.01."""
    _, o, i = wl.mats[mat]
    return _normal_bf16((wl.E, o, wl.r), 0.01, _gen(wl.seed, KIND_B, layer, mat, device), device)


def gen_router(wl: Workload, device="cpu") -> torch.Tensor:
    """[E][d], std 0.02."""
    return _normal_bf16((wl.E, wl.d), 0.02, _gen(wl.seed, KIND_ROUTER, 0, 0, device), device)


TIE_MARGIN = 1e-3   # smallest gap between neighbouring logits near the selection boundary, x the token's largest |logit|


def _logits64(h: torch.Tensor, router: torch.Tensor) -> torch.Tensor:
    """Library fp64 matmul of bf16-rounded hidden states with the router rows: [T][E]."""
    return h.to(torch.bfloat16).double() @ router.double().T


def _decisive(logits: torch.Tensor, k: int) -> torch.Tensor:
    """Per token: are the k + 1 largest logits pairwise at least TIE_MARGIN x max|logit| apart?
    Then no arithmetic that is accurate to 1e-5 can order them differently, and "the k largest,
    in descending order" is one well-defined answer."""
    top = torch.sort(logits, dim=1, descending=True).values[:, : k + 1]
    if top.shape[1] < 2:
        return torch.ones(logits.shape[0], dtype=torch.bool, device=logits.device)
    gaps = (top[:, :-1] - top[:, 1:]).min(dim=1).values
    return gaps >= TIE_MARGIN * logits.abs().max(dim=1).values


def _top_set(logits_row: torch.Tensor, k: int):
    return sorted(torch.topk(logits_row, k).indices.tolist())


def gen_hidden(wl: Workload, device="cpu") -> torch.Tensor:
    """[T][d] N(0,1), rounded to bf16.

    Near-tie tokens are redrawn: a token whose k + 1 largest router logits (library fp64
    matmul against gen_router's rows) are not TIE_MARGIN apart is replaced by a fresh draw,
    so the routing decision of every token is unambiguous at any reasonable precision.
    With repeat_prob > 0, token t is h_{t-1} + 0.05*N(0,1) with that probability, redrawn
    (up to 64 times) until it keeps the expert set of token t-1; the others are fresh draws.
    """
    g = _gen(wl.seed, KIND_HIDDEN, 0, 0, device)
    h = torch.randn((wl.T, wl.d), generator=g, device=device, dtype=torch.float32)
    router = gen_router(wl, device)
    draw = lambda n: torch.randn((n, wl.d), generator=g, device=device, dtype=torch.float32)
    if wl.repeat_prob <= 0:
        for _ in range(1000):
            bad = ~_decisive(_logits64(h, router), wl.k)
            n_bad = int(bad.sum())
            if n_bad == 0:
                break
            h[bad] = draw(n_bad)
        return h.to(torch.bfloat16)
    gr = _gen(wl.seed, KIND_REPEAT, 0, 0, "cpu")
    rep = (torch.rand((wl.T,), generator=gr) < wl.repeat_prob).tolist()
    prev_set = None
    for t in range(wl.T):
        noise = h[t].clone()
        for attempt in range(1000):
            cand = h[t - 1] + 0.05 * noise if (t > 0 and rep[t]) else noise
            lg = _logits64(cand[None, :], router)
            ok = bool(_decisive(lg, wl.k)[0])
            if ok and t > 0 and rep[t] and attempt < 64:
                ok = _top_set(lg[0], wl.k) == prev_set   # after 64 tries a decisive token with a new set is accepted
            if ok:
                break
            noise = draw(1)[0]
        h[t] = cand
        prev_set = _top_set(lg[0], wl.k)
    return h.to(torch.bfloat16)


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> numpy uint16 bit patterns (host)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def from_bits(a: np.ndarray, device="cpu") -> torch.Tensor:
    """numpy uint16 bit patterns -> bf16 tensor."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)
