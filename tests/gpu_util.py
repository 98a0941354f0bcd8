"""Helpers for the GPU parity tests: put a synthetic model on the device and
compare the HIP path's weights with the CPU oracle's."""
import numpy as np
import torch

import adafuse_workloads as wlmod
import paper_2603_11873_amd as af


class DeviceModel:
    """All adapted matrices of a workload on cuda:0 (W_base, W_work, A bank, B bank)."""

    def __init__(self, wl, gen_device="cpu", k_max=None, sentinel=True):
        self.wl = wl
        dev = torch.device("cuda:0")
        self.mats = []
        for layer in range(wl.layers):
            for mi in range(len(wl.mats)):
                wb = wlmod.gen_w(wl, layer, mi, gen_device).to(dev)
                a = wlmod.gen_a_bank(wl, layer, mi, gen_device).to(dev)
                b = wlmod.gen_b_bank(wl, layer, mi, gen_device).to(dev)
                ww = torch.empty_like(wb)
                if sentinel:
                    ww.view(torch.int16).fill_(0x7FC1)       # NaN pattern: any element left unwritten shows
                self.mats.append((wb, ww, a, b))
        self.router = wlmod.gen_router(wl, gen_device).to(dev)
        self.hidden = wlmod.gen_hidden(wl, gen_device).to(dev)
        self.ctx = af.Context(self.mats, k_max or wl.k)

    def close(self):
        self.ctx.close()


def oracle_decisions(oracle, hidden, router, k, device="cuda:0", gate_norm=0):
    """The ORACLE's routing decisions for a token sequence, on the host and uploaded.

    Switch tests feed these to both sides, so no oracle input ever comes from a HIP kernel.
    Returns (idx np [T][k], gates32 np [T][k], idx device tensor, gates device tensor).
    """
    ref = oracle.pregate(wlmod.bits(hidden), wlmod.bits(router), k, gate_norm)
    return (ref["idx"], ref["gates32"], torch.from_numpy(ref["idx"]).to(device),
            torch.from_numpy(ref["gates32"]).to(device))


def _line(bits_arr):
    """bf16 bit patterns on the monotone integer line (-0 and +0 coincide)."""
    b = bits_arr.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


def _spacing(v):
    return 2.0 ** (np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -126))) - 7)


# Ceiling on the error of a cancellation case, in fp32 roundings (2^-24) of the operand magnitude
# |W| + sum |c||B||A|.  The derived bound is r + k + 2 (one rounding per accumulated product, per
# rescale of the chain, and for the final fused multiply-add); errors of independent roundings
# add like a random walk, so what a correct kernel shows is a few units.  A kernel that, say,
# rounded an operand to bf16 (2^-9) would show tens of thousands.
CANCEL_UNITS_CEILING = 4.0


class Verdict(tuple):
    """(max_ulp, n_diff, n, n_cancel) plus what the cancellation cases looked like:
    .cancel_ulp   largest bf16-ULP distance among them (0 if none)
    .cancel_units largest |got - exact| among them, in units of 2^-24 x (|W| + sum |c||B||A|),
                  i.e. in fp32 roundings of the operand magnitude; the derived bound is r + k + 2
    """
    cancel_ulp = 0
    cancel_units = 0.0


def judge(got, want, exact_and_mag, n_roundings):
    """Element-wise verdict on bf16 bit arrays `got` (HIP path) against `want` (oracle, single rounding).

    Bar: every element within 1 bf16 ULP.  Where the sum cancels to far below its operands, one
    spacing of the tiny result is smaller than the fp32 rounding of the sum itself; such an
    element passes if it is the correct rounding of a value within the fp32 accumulation bound
    of the exact one,
        |got - exact| <= spacing(want)/2 + n_roundings * 2^-24 * mag,
    mag = |W| + sum_j |c_j| |B_j| |A_j|, and the exact result really is tiny next to its operands
    (|exact| < 2^-8 mag).  exact_and_mag() -> (exact, mag) as fp64 arrays; called only if needed.
    """
    d = np.abs(_line(got) - _line(want))
    n_diff = int(np.count_nonzero(d))
    bad = np.argwhere(d > 1)
    n_cancel, cancel_ulp, cancel_units = 0, 0, 0.0
    if len(bad):
        exact, mag = exact_and_mag()
        to_f = lambda x: wlmod.from_bits(x).double().numpy()
        gv, wv = to_f(got), to_f(want)
        for o, i in bad:
            assert np.isfinite(gv[o, i]), (int(o), int(i), "not finite")
            err = abs(gv[o, i] - exact[o, i])
            assert err <= 0.5 * _spacing(wv[o, i]) + n_roundings * 2.0 ** -24 * mag[o, i], \
                (int(o), int(i), float(gv[o, i]), float(exact[o, i]), int(d[o, i]))
            assert abs(exact[o, i]) < 2.0 ** -8 * mag[o, i], (int(o), int(i), "more than 1 ULP off without a cancellation")
            cancel_ulp = max(cancel_ulp, int(d[o, i]))
            cancel_units = max(cancel_units, float(err / (2.0 ** -24 * mag[o, i])))
            d[o, i] = 0
            n_cancel += 1
    v = Verdict((int(d.max(initial=0)), n_diff, want.size, n_cancel))
    v.cancel_ulp, v.cancel_units = cancel_ulp, cancel_units
    return v


def compare(oracle, w, a, b, got, idx, gates, scale):
    """Verdict for one out-of-place merge (host bit arrays; b already restricted to w's rows):
    `got` against the oracle's W' = rn(W + s sum_j g_j B_j A_j); n_roundings = r + k + 2."""
    idx = np.asarray(idx, np.int32)
    gates = np.asarray(gates, np.float32)
    want = oracle.merge(w, a, b, idx, gates, scale)

    def exact_and_mag():
        to_f = lambda x: wlmod.from_bits(x).double().numpy()
        mag = np.abs(to_f(w))
        for e, g in zip(idx, gates):
            mag = mag + abs(float(scale) * float(g)) * (np.abs(to_f(b[e])) @ np.abs(to_f(a[e])))
        return oracle.merge(w, a, b, idx, gates, scale, rounded=False), mag

    return judge(got, want, exact_and_mag, a.shape[1] + len(idx) + 2)


def compare_inplace(oracle, before, a, b, got, prev, nxt, scale):
    """Verdict for one in-place call (Eq.8 as printed): `got` against the oracle's single-rounded
    rn(W_before - dW(prev) + dW(next)) from the same bits; prev / nxt = (idx, gates) host arrays.
    The exact value and the operand magnitude of a cancellation case come from library fp64 matmuls."""
    want = oracle.inplace_swap(before, a, b, prev[0], prev[1], nxt[0], nxt[1], scale)

    def exact_and_mag():
        to_f = lambda x: wlmod.from_bits(x).double().numpy()
        A, B = to_f(a), to_f(b)
        exact = to_f(before)
        mag = np.abs(exact)
        for sign, (ids, gs) in ((-1.0, prev), (1.0, nxt)):
            for e, g in zip(ids, gs):
                c = float(np.float32(scale)) * float(np.float32(g))
                exact = exact + sign * c * (B[e] @ A[e])
                mag = mag + abs(c) * (np.abs(B[e]) @ np.abs(A[e]))
        return exact, mag

    return judge(got, want, exact_and_mag, a.shape[1] + len(prev[0]) + len(nxt[0]) + 2)


def check_rows(oracle, mat, idx, gates, scale, rows):
    """Compare W_work[rows] of one matrix with the oracle; returns (max_ulp, n_diff, n, n_cancel)."""
    wb, ww, a, b = mat
    ridx = torch.as_tensor(rows, device=wb.device, dtype=torch.long)
    return compare(oracle, wlmod.bits(wb.index_select(0, ridx)), wlmod.bits(a), wlmod.bits(b.index_select(1, ridx)),
                   wlmod.bits(ww.index_select(0, ridx)), idx, gates, scale)


def check_full(oracle, mat, idx, gates, scale):
    wb, ww, a, b = mat
    return compare(oracle, wlmod.bits(wb), wlmod.bits(a), wlmod.bits(b), wlmod.bits(ww), idx, gates, scale)


class Tally:
    """Accumulates verdicts over many matrices and asserts the aggregate bars."""

    def __init__(self):
        self.n = self.diff = self.cancel = self.cancel_ulp = 0
        self.cancel_units = 0.0

    def add(self, verdict, ulp_tol, where=None):
        mx, nd, n, nc = verdict
        assert mx <= ulp_tol, (where, mx)
        self.n += n
        self.diff += nd
        self.cancel += nc
        self.cancel_ulp = max(self.cancel_ulp, getattr(verdict, "cancel_ulp", 0))
        self.cancel_units = max(self.cancel_units, getattr(verdict, "cancel_units", 0.0))

    def finish(self, max_diff_fraction, max_cancel_fraction=1e-5, max_cancel_units=CANCEL_UNITS_CEILING):
        # the fraction is a rate: a small sample gets the spread of a count with that mean on top (4 sigma + 4)
        expect = max_diff_fraction * self.n
        assert self.diff <= expect + 4 * expect ** 0.5 + 4, (self.diff, self.n)
        assert self.cancel <= max(2, max_cancel_fraction * self.n), (self.cancel, self.n)
        assert self.cancel_units <= max_cancel_units, (self.cancel_units, self.cancel_ulp)

    def summary(self):
        s = f"elements {self.n}, differing from the oracle (by 1 ULP) {self.diff} ({self.diff / max(self.n, 1):.1e})"
        if self.cancel:
            s += (f", cancellation cases {self.cancel}: at most {self.cancel_ulp} ULP of the (tiny) result = "
                  f"{self.cancel_units:.2f} fp32 roundings of the operand magnitude")
        else:
            s += ", no cancellation case"
        return s


def sample_rows(out, tile_rows, rng):
    """First and last rows, a band across a tile boundary, and a few random rows."""
    rows = {0, out - 1}
    if out > tile_rows:
        bnd = tile_rows * int(rng.integers(1, (out + tile_rows - 1) // tile_rows))
        rows.update(r for r in range(bnd - 2, bnd + 3) if 0 <= r < out)
    rows.update(int(x) for x in rng.integers(0, out, 3))
    return sorted(rows)
