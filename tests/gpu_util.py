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


def compare(oracle, w, a, b, got, idx, gates, scale):
    """Element-wise verdict for one matrix (host bit arrays; b already restricted to w's rows).

    Bar: every element within 1 bf16 ULP of the oracle's single-rounded value.  Where W + dW
    cancels to far below |W| and |dW|, one spacing of the tiny result is smaller than the fp32
    rounding of the sum itself; such an element passes if it is the correct rounding of a value
    within the fp32 accumulation bound of the exact one:
        |got - exact| <= spacing(want)/2 + (r + k + 2) * 2^-24 * (|W| + sum_j |s g_j| |B_j| |A_j|).
    Returns (max_ulp over elements judged by the 1-ULP bar, n_diff, n, n_cancel).
    """
    idx = np.asarray(idx, np.int32)
    gates = np.asarray(gates, np.float32)
    want = oracle.merge(w, a, b, idx, gates, scale)
    d = np.abs(_line(got) - _line(want))
    n_diff = int(np.count_nonzero(d))
    bad = np.argwhere(d > 1)
    n_cancel = 0
    if len(bad):
        exact = oracle.merge(w, a, b, idx, gates, scale, rounded=False)
        to_f = lambda x: wlmod.from_bits(x).double().numpy()
        r = a.shape[1]
        mag = np.abs(to_f(w))
        for e, g in zip(idx, gates):
            mag = mag + abs(float(scale) * float(g)) * (np.abs(to_f(b[e])) @ np.abs(to_f(a[e])))
        bound = (r + len(idx) + 2) * 2.0 ** -24 * mag
        gv, wv = to_f(got), to_f(want)
        for o, i in bad:
            assert abs(gv[o, i] - exact[o, i]) <= 0.5 * _spacing(wv[o, i]) + bound[o, i], \
                (int(o), int(i), float(gv[o, i]), float(exact[o, i]), int(d[o, i]))
            # and it really is a cancellation: the result is tiny next to its operands
            assert abs(exact[o, i]) < 2.0 ** -8 * mag[o, i]
            d[o, i] = 0
            n_cancel += 1
    return int(d.max(initial=0)), n_diff, want.size, n_cancel


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
        self.n = self.diff = self.cancel = 0

    def add(self, verdict, ulp_tol, where=None):
        mx, nd, n, nc = verdict
        assert mx <= ulp_tol, (where, mx)
        self.n += n
        self.diff += nd
        self.cancel += nc

    def finish(self, max_diff_fraction, max_cancel_fraction=1e-5):
        assert self.diff <= max(4, max_diff_fraction * self.n), (self.diff, self.n)
        assert self.cancel <= max(2, max_cancel_fraction * self.n), (self.cancel, self.n)


def sample_rows(out, tile_rows, rng):
    """First and last rows, a band across a tile boundary, and a few random rows."""
    rows = {0, out - 1}
    if out > tile_rows:
        bnd = tile_rows * int(rng.integers(1, (out + tile_rows - 1) // tile_rows))
        rows.update(r for r in range(bnd - 2, bnd + 3) if 0 <= r < out)
    rows.update(int(x) for x in rng.integers(0, out, 3))
    return sorted(rows)
