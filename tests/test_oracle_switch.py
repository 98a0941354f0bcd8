"""Pins for the switch oracle: exact-rational brute force, special cases that
reduce to a library GEMM, and the identities of Eq.2-8."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import adafuse_workloads as wlmod
from exact import bf16_to_fraction, fraction_to_bf16

TOY = wlmod.WORKLOADS["toy"]


def _rand_case(out, in_, E, r, seed, wstd=0.02, bstd=0.01):
    g = torch.Generator().manual_seed(seed)
    w = (wstd * torch.randn((out, in_), generator=g)).to(torch.bfloat16)
    a = (in_ ** -0.5 * torch.randn((E, r, in_), generator=g)).to(torch.bfloat16)
    b = (bstd * torch.randn((E, out, r), generator=g)).to(torch.bfloat16)
    return wlmod.bits(w), wlmod.bits(a), wlmod.bits(b)


def _f64(bits_arr):
    return wlmod.from_bits(bits_arr).double().numpy()


def _exact_merge(w, a, b, idx, gates, scale, rows, cols, w_signed_terms=None):
    """Exact rational W + sum_j (s*g_j) * sum_rho B A, rounded once to bf16."""
    res = {}
    s = Fraction(float(np.float32(scale)))
    for o in rows:
        for i in cols:
            v = bf16_to_fraction(int(w[o, i]))
            for sign, (ids, gs) in w_signed_terms or [(1, (idx, gates))]:
                for e, g in zip(ids, gs):
                    p = Fraction(0)
                    for rho in range(a.shape[1]):
                        p += bf16_to_fraction(int(b[e, o, rho])) * bf16_to_fraction(int(a[e, rho, i]))
                    v += sign * s * Fraction(float(np.float32(g))) * p
            res[(o, i)] = fraction_to_bf16(v)
    return res


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_exact_rational_tiny(oracle, seed):
    # Delta comparable to W's spacing so that roundings really move
    w, a, b = _rand_case(5, 8, 3, 2, seed, wstd=0.02, bstd=0.3)
    idx, gates = [2, 0], [0.7, 0.3]
    got = oracle.merge(w, a, b, idx, gates, 2.0)
    want = _exact_merge(w, a, b, idx, gates, 2.0, range(5), range(8))
    for (o, i), v in want.items():
        assert got[o, i] == v, (o, i)
    assert not np.array_equal(got, w)


def test_brute_force_exact_rational_on_toy_rows(oracle):
    # the Toy workload's own tensors, router-chosen experts, a band of rows
    w = wlmod.bits(wlmod.gen_w(TOY, 1, 2))
    a = wlmod.bits(wlmod.gen_a_bank(TOY, 1, 2))
    b = wlmod.bits(wlmod.gen_b_bank(TOY, 1, 2))
    pg = oracle.pregate(wlmod.bits(wlmod.gen_hidden(TOY)), wlmod.bits(wlmod.gen_router(TOY)), TOY.k)
    for t in (0, 7, 15):
        idx, gates = pg["idx"][t], pg["gates32"][t]
        rows = (100, 103)
        got = oracle.merge(w, a, b, idx, gates, TOY.scale, rows=rows)
        want = _exact_merge(w, a, b, idx.tolist(), gates.tolist(), TOY.scale, range(*rows), range(0, 256, 5))
        for (o, i), v in want.items():
            assert got[o - rows[0], i] == v, (t, o, i)


def test_zero_gates_and_empty_selection_leave_w_bit_identical(oracle):
    w, a, b = _rand_case(16, 24, 4, 4, 3)
    assert np.array_equal(oracle.merge(w, a, b, [1, 3], [0.0, 0.0], 2.0), w)
    assert np.array_equal(oracle.merge(w, a, b, [], [], 2.0), w)          # un-merge: back to base


def test_single_expert_gate_one_is_library_gemm(oracle):
    w, a, b = _rand_case(24, 40, 4, 4, 4, bstd=0.2)
    for e in range(4):
        ref = _f64(w) + 2.0 * (_f64(b[e]) @ _f64(a[e]))
        got = oracle.merge(w, a, b, [e], [1.0], 2.0, rounded=False)
        assert np.allclose(got, ref, rtol=1e-13, atol=1e-16)
        # the rounded form is the (separately pinned) single rounding of those values
        assert np.array_equal(oracle.merge(w, a, b, [e], [1.0], 2.0), oracle.f64_to_bf16(got))


def test_merged_gemv_equals_dynamic_adapter_output(oracle):
    # Eq.2 (adapter applied at run time) versus Eq.3 (merged backbone)
    w, a, b = _rand_case(48, 64, 8, 8, 5, bstd=0.2)
    idx, gates = [6, 1, 3], np.array([0.5, 0.3, 0.2], np.float32)
    x = np.random.default_rng(0).standard_normal(64)
    y_dyn = oracle.dynamic_adapter_forward(w, a, b, idx, gates, 2.0, x)
    merged = oracle.merge(w, a, b, idx, gates, 2.0, rounded=False)
    assert np.allclose(merged @ x, y_dyn, rtol=1e-12, atol=1e-14)
    # library statement of the same thing
    ref = _f64(w) @ x + 2.0 * sum(g * (_f64(b[e]) @ (_f64(a[e]) @ x)) for e, g in zip(idx, gates.astype(np.float64)))
    assert np.allclose(y_dyn, ref, rtol=1e-12, atol=1e-14)
    # after the single bf16 rounding the GEMV differs by at most half a spacing per weight
    wr = oracle.merge(w, a, b, idx, gates, 2.0)
    y_m = oracle.gemv_bf16(wr, x)
    assert np.allclose(y_m, _f64(wr) @ x, rtol=1e-13, atol=1e-15)
    vals = np.abs(_f64(wr))
    spacing = 2.0 ** (np.floor(np.log2(np.maximum(vals, 2.0 ** -126))) - 7)
    bound = 0.5 * (2 * spacing) @ np.abs(x)      # 2x: spacing of the un-rounded value's binade
    assert np.all(np.abs(y_m - y_dyn) <= bound)
    assert np.max(np.abs(y_m - y_dyn)) > 0


def test_prefill_is_the_per_token_merged_backbone(oracle):
    # Many tokens, each with its own decision: row t must equal the mat-vec of the weights merged
    # with token t's experts (Eq.2 <=> Eq.3 token by token), and a library statement of the sum.
    w, a, b = _rand_case(40, 56, 6, 4, 11, bstd=0.2)
    rng = np.random.default_rng(3)
    T, k = 9, 2
    x = (rng.standard_normal((T, 56))).astype(np.float32)
    xb = oracle.f64_to_bf16(x.astype(np.float64))
    xs = _f64(xb)
    idx = np.array([rng.permutation(6)[:k] for _ in range(T)], np.int32)
    gates = rng.random((T, k)).astype(np.float32)
    y = oracle.prefill(w, a, b, idx, gates, 2.0, xb)
    assert y.shape == (T, 40)
    for t in range(T):
        merged = oracle.merge(w, a, b, idx[t], gates[t], 2.0, rounded=False)
        assert np.allclose(y[t], merged @ xs[t], rtol=1e-12, atol=1e-14)
        ref = _f64(w) @ xs[t] + 2.0 * sum(float(g) * (_f64(b[e]) @ (_f64(a[e]) @ xs[t])) for e, g in zip(idx[t], gates[t]))
        assert np.allclose(y[t], ref, rtol=1e-12, atol=1e-14)
        # pairing a token with its neighbour's decision is a different result
        other = oracle.merge(w, a, b, idx[(t + 1) % T], gates[(t + 1) % T], 2.0, rounded=False)
        assert not np.allclose(y[t], other @ xs[t], rtol=1e-6, atol=1e-9)
    # a subset of rows, and an expert listed twice counts twice
    assert np.array_equal(oracle.prefill(w, a, b, idx, gates, 2.0, xb, tokens=[7, 2]), y[[7, 2]])
    twice = oracle.prefill(w, a, b, [[3, 3]], [[0.25, 0.5]], 2.0, xb[:1])
    once = oracle.prefill(w, a, b, [[3]], [[0.75]], 2.0, xb[:1])
    assert np.allclose(twice, once, rtol=1e-13, atol=1e-15)


def test_permutation_of_selection_is_irrelevant(oracle):
    w, a, b = _rand_case(16, 32, 8, 4, 6, bstd=0.2)
    idx, gates = [5, 2, 7], [0.2, 0.5, 0.3]
    base = oracle.merge(w, a, b, idx, gates, 2.0, rounded=False)
    for perm in ([1, 0, 2], [2, 1, 0], [1, 2, 0]):
        p = oracle.merge(w, a, b, [idx[q] for q in perm], [gates[q] for q in perm], 2.0, rounded=False)
        assert np.allclose(p, base, rtol=1e-14, atol=1e-18)
    assert np.array_equal(oracle.merge(w, a, b, [7, 5, 2], [0.3, 0.2, 0.5], 2.0),
                          oracle.merge(w, a, b, idx, gates, 2.0))


def test_concatenated_form_equals_sum_form(oracle):
    # Eq.4-6: DOWN = concat_j[g_j * DOWN_j], UP = concat_j[UP_j], one product
    w, a, b = _rand_case(20, 48, 6, 4, 7, bstd=0.2)
    idx, gates = [4, 0], np.array([0.6, 0.4], np.float32)
    down = np.concatenate([float(g) * _f64(a[e]) for e, g in zip(idx, gates)], 0)     # [(k r)][in]
    up = np.concatenate([_f64(b[e]) for e in idx], 1)                                 # [out][(k r)]
    ref = _f64(w) + 2.0 * (up @ down)
    got = oracle.merge(w, a, b, idx, gates, 2.0, rounded=False)
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-17)


def test_wrong_formulas_are_told_apart(oracle):
    # plausible mistakes (dropped scale, gate ignored, experts swapped, A/B
    # roles exchanged) all differ from the oracle on this case
    w, a, b = _rand_case(32, 32, 4, 4, 8, bstd=0.2)
    idx, gates = [3, 1], np.array([0.75, 0.25], np.float32)
    good = oracle.merge(w, a, b, idx, gates, 2.0, rounded=False)
    W, A, B = _f64(w), _f64(a), _f64(b)
    wrong = [
        W + sum(g * (B[e] @ A[e]) for e, g in zip(idx, gates)),                # no scale
        W + 2.0 * sum(B[e] @ A[e] for e in idx),                                # no gate
        W + 2.0 * sum(g * (B[e] @ A[e]) for e, g in zip(idx[::-1], gates)),    # gates crossed
        W + 2.0 * sum(g * (B[e] @ A[e]).T for e, g in zip(idx, gates)),        # transposed update
        W - 2.0 * sum(g * (B[e] @ A[e]) for e, g in zip(idx, gates)),          # sign
    ]
    for bad in wrong:
        assert not np.allclose(good, bad, rtol=1e-6, atol=1e-9)


def test_row_ranges_are_slices_of_the_full_result(oracle):
    w, a, b = _rand_case(40, 16, 4, 4, 9, bstd=0.2)
    full = oracle.merge(w, a, b, [0, 2], [0.4, 0.6], 2.0)
    assert np.array_equal(oracle.merge(w, a, b, [0, 2], [0.4, 0.6], 2.0, rows=(7, 19)), full[7:19])
    assert oracle.merge(w, a, b, [0, 2], [0.4, 0.6], 2.0, rows=(5, 5)).shape == (0, 16)
    with pytest.raises(ValueError):
        oracle.merge(w, a, b, [0, 4], [0.4, 0.6], 2.0)        # expert index out of range
    with pytest.raises(ValueError):
        oracle.merge(w, a, b, [0, 1], [0.4, 0.6], 2.0, rows=(0, 41))


# ---- the paper-literal in-place step of Eq.7-8 -------------------------------

def test_telescoping_identity(oracle):
    # W_{t-1} - dW_{t-1} + dW_t = W_base + dW_t, in fp64 before any rounding
    w, a, b = _rand_case(16, 32, 8, 4, 10, bstd=0.2)
    prev, nxt = ([1, 6], [0.3, 0.7]), ([6, 2], [0.55, 0.45])
    base = _f64(w)
    w_prev = oracle.merge(w, a, b, *prev, 2.0, rounded=False)
    d_prev = w_prev - base
    d_next = oracle.merge(w, a, b, *nxt, 2.0, rounded=False) - base
    assert np.allclose(w_prev - d_prev + d_next, base + d_next, rtol=1e-14, atol=1e-18)


def test_inplace_step_exact_rational(oracle):
    w, a, b = _rand_case(4, 8, 4, 2, 11, bstd=0.3)
    prev, nxt = ([1, 3], [0.25, 0.75]), ([3, 0], [0.6, 0.4])
    cur = oracle.merge(w, a, b, *prev, 2.0)
    got = oracle.inplace_swap(cur, a, b, *prev, *nxt, 2.0)
    want = _exact_merge(cur, a, b, None, None, 2.0, range(4), range(8),
                        w_signed_terms=[(-1, prev), (1, nxt)])
    for (o, i), v in want.items():
        assert got[o, i] == v, (o, i)


def test_inplace_step_special_cases(oracle):
    w, a, b = _rand_case(8, 16, 4, 4, 12, bstd=0.2)
    sel = ([2, 0], [0.5, 0.5])
    # nothing merged before: the in-place step is a plain merge
    assert np.array_equal(oracle.inplace_swap(w, a, b, [], [], *sel, 2.0), oracle.merge(w, a, b, *sel, 2.0))
    # same decision twice: the update is exactly zero
    cur = oracle.merge(w, a, b, *sel, 2.0)
    assert np.array_equal(oracle.inplace_swap(cur, a, b, *sel, *sel, 2.0), cur)
    # un-merging what was merged returns W_base up to the two roundings on the way:
    # half a spacing of the merged value plus half a spacing of the result
    back = oracle.inplace_swap(cur, a, b, *sel, [], [], 2.0)

    def spacing(v):
        return 2.0 ** (np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -126))) - 7)

    err = np.abs(_f64(back) - _f64(w))
    assert np.all(err <= 0.5 * spacing(_f64(cur)) + 0.5 * spacing(_f64(back)) + 1e-30)
    assert err.max() > 0          # the in-place form does drift; the out-of-place form cannot
