#!/usr/bin/env python3
"""Benchmark of the AdaFuse hot path on one MI355X.

A step = one token: the pre-gating router on that token's hidden state followed
by one fused switch (SWAP: previous token's experts out, this token's in) over
every adapted matrix of the model, both enqueued on one stream with no host
round trip in between.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line: the metric (switch latency per token, lower is better),
the HBM roofline of the dominant kernel measured with HIP events on the launch
stream, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="llama2_7b_all")
    ap.add_argument("--kernel", default="auto", choices=["auto", "valu", "mfma", "gemm"])
    ap.add_argument("--gemm-form", type=int, default=0, choices=[0, 1, 3, 4],
                    help="ADAFUSE_OPT_GEMM_FORM: 0 library's choice, 1 unrolled, 3 overlapped, 4 chained (eight vertically adjacent tiles per workgroup)")
    ap.add_argument("--gemm-waves", type=int, default=0, choices=[0, 4, 8], help="ADAFUSE_OPT_GEMM_WAVES (0: library's choice)")
    ap.add_argument("--mode", default="swap", choices=["swap", "unmerge"],
                    help="unmerge times the plain W_base->W_work copy over the same tile table")
    ap.add_argument("--inplace", action="store_true",
                    help="paper-literal in-place update (w_work == w_base): SWAP carries 2k experts")
    ap.add_argument("--per-matrix", action="store_true",
                    help="the paper's 'simple merge' ablation: one launch per adapted matrix instead of one for all")
    ap.add_argument("--forward", action="store_true",
                    help="also time the step after the switch: merged GEMVs vs the un-merged dynamic-adapter path")
    ap.add_argument("--graph", action="store_true",
                    help="capture the whole token sequence (T x [pregate, switch]) in one HIP graph and replay it; "
                         "for launch-bound workloads (toy).  Reported separately as graph_us_per_token")
    ap.add_argument("--prefill", type=int, default=0, metavar="T",
                    help="instead of the switch: time adafuse_prefill for T tokens through every matrix of the "
                         "workload (un-merged adapters, per-token decisions) and print that as the JSON line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-copy-ceiling", action="store_true",
                    help="skip the plain-copy launches after the timed loop (for counter runs that average over dispatches)")
    ap.add_argument("--cpu-layers", type=int, default=16,
                    help="layers of the model the oracle is timed on (16 of the 7B shape: about 10 s on 16 host threads)")
    return ap.parse_args()


def read_traffic(workload, kernel_fn):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this kernel and workload.

    The counters cannot be read inside a timed run, so the figure is a stored measurement; it is
    only reported while the library's sources still hash to the stamp the summary carries.
    Returns (bytes or None, note)."""
    from paper_2603_11873_amd.build import source_hash
    name = f"{kernel_fn.replace('_kernel', '')}_{workload}_pmc.txt"
    path = os.path.join(ROOT, "profiles", name)
    traffic = stamp = None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
            elif line.startswith("csrc_sha16:"):
                stamp = line.split(":")[1].strip()
    except OSError:
        return None, f"no counter summary profiles/{name}"
    now = source_hash()
    if stamp != now:
        return None, f"traffic_stale: profiles/{name} was measured on sources {stamp}, the library is built from {now}"
    return traffic, f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/{name}, sources {stamp}"


def cpu_baseline(wl, mats, hidden, router, t, n_layers):
    """Time the oracle (as it stands) on the first n_layers of the model: router for token t,
    then one switch with the oracle's own decision."""
    import adafuse_workloads as wlmod
    import oracle
    per_layer = len(wl.mats)
    sample = mats[: n_layers * per_layer]
    host = [(wlmod.bits(wb), wlmod.bits(a), wlmod.bits(b)) for wb, _, a, b in sample]
    hb, rb = wlmod.bits(hidden[t:t + 1]), wlmod.bits(router)
    oracle.lib()
    t0 = time.perf_counter()
    dec = oracle.pregate(hb, rb, wl.k)
    idx, gates = dec["idx"][0], dec["gates32"][0]
    for w, a, b in host:
        oracle.merge(w, a, b, idx, gates, wl.scale)
    dt = time.perf_counter() - t0
    elems = sum(w.size for w, _, _ in host)
    full = dt * wl.elements / elems
    return {"value": full * 1e6, "unit": "us/token", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"one switch of the first {n_layers} of {wl.layers} layers ({len(host)} matrices, "
                      f"{elems} elements) in {dt:.2f} s, scaled by element count to the full model"}


def forward_context(torch, af, ctx, wl, mats, idx, gates, stream, reps=20):
    """us per token of one pass over all matrices: merged backbone (Eq.3) and dynamic adapters (Eq.2)."""
    dev = mats[0][0].device
    x = torch.randn(sum(m[0].shape[1] for m in mats), device=dev).to(torch.bfloat16)
    y = torch.zeros(sum(m[0].shape[0] for m in mats), dtype=torch.float32, device=dev)
    z = torch.zeros(wl.k * wl.r, dtype=torch.float32, device=dev)
    hi, hg = idx[0].cpu().tolist(), gates[0].cpu().tolist()
    res = {}
    with torch.cuda.stream(stream):
        for name, fn in (("merged_gemv", lambda: ctx.forward_merged(x, y, stream=stream)),
                         ("dynamic_adapter", lambda: ctx.forward_dynamic(hi, hg, wl.scale, x, y, z, stream=stream))):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            res[name + "_us"] = (time.perf_counter() - t0) / reps * 1e6
    res["launches"] = {"merged_gemv": wl.n_mats, "dynamic_adapter": wl.n_mats * (1 + 2 * wl.k)}
    res["note"] = "one GEMV per matrix; the dynamic form adds a down- and an up-projection launch per selected expert"
    return res


def prefill_bench(torch, af, ctx, wl, mats, hidden, router, T, stream, reps):
    """T tokens through every matrix: one adafuse_prefill_group call per set of matrices of a layer that take
    the same input (q, k, v / o / gate, up / down -- the dependency structure of a Llama layer)."""
    dev = mats[0][0].device
    reps_h = (T + wl.T - 1) // wl.T
    h = hidden.repeat(reps_h, 1)[:T].contiguous()
    idx, gates, _ = af.pregate(h, router, wl.k, stream=stream)
    per_layer = len(wl.mats)
    names = [m[0] for m in wl.mats]
    sets = [[names.index(n) for n in grp if n in names] for grp in (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))]
    sets = [g for g in sets if g]
    assert sorted(i for g in sets for i in g) == list(range(per_layer))
    groups = [[layer * per_layer + i for i in g] for layer in range(wl.layers) for g in sets]
    xs = {i: torch.randn((T, i), device=dev).to(torch.bfloat16) for i in {m[0].shape[1] for m in mats}}
    ys = {mi: torch.empty((T, mats[mi][0].shape[0]), dtype=torch.float32, device=dev) for mi in range(per_layer)}
    ws = torch.empty(max(ctx.prefill_group_workspace_bytes(g, T, wl.k) for g in groups[:len(sets)]), dtype=torch.uint8, device=dev)

    def run():
        for g in groups:
            ctx.prefill_group(g, xs[mats[g[0]][0].shape[1]], idx, gates, wl.scale, ys=[ys[mi % per_layer] for mi in g],
                              workspace=ws, stream=stream)

    with torch.cuda.stream(stream):
        t = timed_launches(torch, stream, run, reps, warm=2)
    w_bytes = 2 * wl.elements
    io_bytes = sum(2 * T * m[0].shape[1] + 4 * T * m[0].shape[0] for m in mats)
    flops = 2 * T * wl.elements + 2 * T * wl.k * wl.r * sum(m[0].shape[0] + m[0].shape[1] for m in mats)
    sec = t["mean"] * 1e-6
    hbm = (w_bytes + io_bytes) / sec / 1e9
    tf = flops / sec / 1e12
    bound = "hbm" if T * 2 < 2 * MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS else "mfma"   # flops per W byte = T
    few = T <= 512 and T * wl.k * wl.r <= 8192
    return {
        "metric": "prefill latency, all adapted matrices, un-merged adapters with per-token decisions (us)",
        "value": t["mean"], "unit": "us", "n_gpus": 1, "steps": reps, "warmup": 2, "ms_per_step": t["mean"] * 1e-3,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "tokens": T, "matrices": wl.n_mats, "E": wl.E, "r": wl.r, "k": wl.k,
                   "calls": len(groups), "groups_per_layer": [[names[i] for i in g] for g in sets],
                   "launches": "2 per group" if few else "3 or 4 per matrix",
                   "step": "adafuse_prefill_group on every set of matrices that share an input, one stream"},
        "roofline": {"bound": bound,
                     "achieved": hbm if bound == "hbm" else tf, "peak": HBM_PEAK_GBS if bound == "hbm" else MFMA_BF16_PEAK_TFLOPS,
                     "unit": "GB/s" if bound == "hbm" else "TFLOP/s",
                     "frac": hbm / HBM_PEAK_GBS if bound == "hbm" else tf / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "kernel": ("prefill_gemm_kernel (base and bank products of a group in one launch) + prefill_finish_kernel" if few else
                                "prefill_gemm_kernel (bank and base passes) + prefill_gate_kernel + prefill_sum_kernel"),
                     "hbm_GBs": hbm, "mfma_TFLOPs": tf,
                     "algorithmic_bytes": w_bytes + io_bytes, "algorithmic_flops": flops, "median_us": t["median"]},
    }


def timed_launches(torch, stream, fn, reps, warm=3):
    """Mean and median us of one enqueue of fn on stream, from an event pair around each."""
    for _ in range(warm):
        fn()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record(stream)
        fn()
        b.record(stream)
    torch.cuda.synchronize()
    us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
    return {"mean": sum(us) / len(us), "median": us[len(us) // 2]}


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import adafuse_workloads as wlmod
    import paper_2603_11873_amd as af

    af.load_library()          # fails loudly if the HIP library is not built
    wl = wlmod.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    mats = []
    for layer in range(wl.layers):
        for mi in range(len(wl.mats)):
            wb = wlmod.gen_w(wl, layer, mi, "cuda")
            mats.append((wb, wb if args.inplace else torch.empty_like(wb), wlmod.gen_a_bank(wl, layer, mi, "cuda"),
                         wlmod.gen_b_bank(wl, layer, mi, "cuda")))
    hidden = wlmod.gen_hidden(wl, "cuda")
    router = wlmod.gen_router(wl, "cuda")
    ctx = af.Context(mats, wl.k)
    ctx.set_kernel({"auto": af.KERNEL_AUTO, "valu": af.KERNEL_VALU, "mfma": af.KERNEL_MFMA, "gemm": af.KERNEL_GEMM}[args.kernel])
    if args.gemm_form:
        ctx.set_option(af.OPT_GEMM_FORM, args.gemm_form)
    if args.gemm_waves:
        ctx.set_option(af.OPT_GEMM_WAVES, args.gemm_waves)
    info = ctx.info()
    kernel_name = {af.KERNEL_VALU: "valu", af.KERNEL_MFMA: "mfma", af.KERNEL_GEMM: "gemm"}[info.kernel]

    if args.prefill > 0:
        out = prefill_bench(torch, af, ctx, wl, mats, hidden, router, args.prefill, torch.cuda.Stream(device=dev), max(2, min(args.steps, 20)))
        ctx.close()
        print(json.dumps(out))
        return

    T = wl.T
    idx = torch.empty((T, wl.k), dtype=torch.int32, device=dev)
    gates = torch.empty((T, wl.k), dtype=torch.float32, device=dev)
    stream = torch.cuda.Stream(device=dev)
    mode = af.SWAP if args.mode == "swap" else af.UNMERGE

    switch = ctx.switch_per_matrix if args.per_matrix else ctx.fused_switch

    def step(t, ev=None):
        """Router for token t, then the fused switch from token t-1's decision to t's."""
        cur, prv = t % T, (t - 1) % T
        af.pregate(hidden[cur:cur + 1], router, wl.k, out=(idx[cur:cur + 1], gates[cur:cur + 1], None), stream=stream)
        if ev is not None:
            ev[0].record(stream)
        switch(idx[prv], gates[prv], idx[cur], gates[cur], wl.k, wl.scale, mode, stream=stream)
        if ev is not None:
            ev[1].record(stream)

    with torch.cuda.stream(stream):
        # the decision "before the first token": token T-1's
        af.pregate(hidden, router, wl.k, out=(idx, gates, None), stream=stream)
        for t in range(args.warmup):
            step(t)
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                  for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(args.steps):
            step(args.warmup + t, events[t])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / args.steps
    kernel_ms = [a.elapsed_time(b) for a, b in events]           # the switch launch alone
    # A SWAP whose previous decision is bit-identical to the next returns at once (nothing to do):
    # such launches stay in `value` (they are part of the sequence) but never enter the rate.
    early_outs = 0
    if mode == af.SWAP:
        hi, hg = idx.cpu(), gates.cpu().view(torch.int32)
        keep = []
        for i, ms in enumerate(kernel_ms):
            cur, prv = (args.warmup + i) % T, (args.warmup + i - 1) % T
            if torch.equal(hi[cur], hi[prv]) and torch.equal(hg[cur], hg[prv]):
                early_outs += 1
            else:
                keep.append(ms)
        kernel_ms_all, kernel_ms = kernel_ms, (keep or kernel_ms)
    avg_kernel_s = sum(kernel_ms) / len(kernel_ms) * 1e-3
    alg_bytes = wl.algorithmic_bytes if mode == af.SWAP else 4 * wl.elements
    if args.inplace:   # the previous token's slices are read too
        alg_bytes += wl.algorithmic_bytes - 4 * wl.elements
    achieved = alg_bytes / avg_kernel_s / 1e9
    # the second bound: 2 k r flops per element of the low-rank product (twice that in place), against the dense bf16 MFMA peak
    alg_flops = 0 if mode != af.SWAP and not args.inplace else wl.flops * (2 if args.inplace and mode == af.SWAP else 1)
    srt = sorted(kernel_ms)
    traffic, traffic_note = (read_traffic(wl.name, ctx.switch_kernel_name(wl.k, mode))
                             if mode == af.SWAP and not args.inplace else (None, "not measured for this mode"))

    out = {
        "metric": "fused-switch latency per token, all layers (us) + achieved HBM GB/s vs peak",
        "value": ms_per_step * 1e3,
        "unit": "us/token",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.layers, "matrices": wl.n_mats, "elements": wl.elements,
                   "E": wl.E, "r": wl.r, "k": wl.k, "tokens": T, "scale": wl.scale, "mode": args.mode + ("-inplace" if args.inplace else "") + ("-per-matrix" if args.per_matrix else ""),
                   "launches_per_switch": wl.n_mats if args.per_matrix else 1,
                   "kernel": kernel_name, "tile": [info.tile_rows, info.tile_cols], "workgroups": info.n_tiles,
                   "step": "pregate(1 token) + fused_switch(all matrices), one stream"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_note,
                     "kernel": ctx.switch_kernel_name(wl.k, mode),
                     "algorithmic_bytes_per_launch": alg_bytes, "early_out_launches_excluded": early_outs,
                     "matrix_core": {"achieved": alg_flops / avg_kernel_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                     "frac": alg_flops / avg_kernel_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                                     "algorithmic_flops_per_launch": alg_flops},
                     "kernel_us": {"mean": avg_kernel_s * 1e6, "median": srt[len(srt) // 2] * 1e3,
                                   "p95": srt[int(0.95 * (len(srt) - 1))] * 1e3, "min": srt[0] * 1e3}},
    }
    if args.steps >= T:
        # one full pass over the token sequence (the first T timed launches), launch by launch
        seq = sorted(a.elapsed_time(b) * 1e3 for a, b in events[:T])
        out["roofline"]["kernel_us_one_sequence"] = {
            "tokens": T, "median": seq[len(seq) // 2], "mean": sum(seq) / len(seq), "p95": seq[int(0.95 * (len(seq) - 1))],
            "min": seq[0], "max": seq[-1]}
    if args.graph:
        # the same T steps as one graph: no per-launch host cost between the kernels
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for t in range(T):
                step(t)
        replays = max(1, (args.steps + T - 1) // T)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        out["graph_us_per_token"] = {"value": (time.perf_counter() - t0) / (replays * T) * 1e6, "tokens_per_graph": T,
                                     "replays": replays, "eager_us_per_token": ms_per_step * 1e3}
    with torch.cuda.stream(stream):
        # the router alone, one token per launch (launch-latency bound: us only)
        out["pregate_us"] = timed_launches(
            torch, stream, lambda: af.pregate(hidden[0:1], router, wl.k, out=(idx[0:1], gates[0:1], None), stream=stream), 64)
        # ... and the whole sequence's decisions in one launch (T workgroups); same values into the same buffers
        out["pregate_us"]["all_tokens_one_launch"] = timed_launches(
            torch, stream, lambda: af.pregate(hidden, router, wl.k, out=(idx, gates, None), stream=stream), 16)
        out["pregate_us"]["tokens"] = T
    if wl.repeat_prob > 0 and mode == af.SWAP:
        # tokens that keep the previous token's expert set (fresh gates) vs tokens that change it
        hidx = idx.cpu().tolist()
        cls = {"same_set": [], "new_set": []}
        for i, ms in enumerate(kernel_ms_all):
            t = (args.warmup + i) % T
            same = sorted(hidx[t]) == sorted(hidx[(t - 1) % T])
            cls["same_set" if same else "new_set"].append(ms * 1e3)
        out["roofline"]["kernel_us_by_token"] = {
            k: {"tokens": len(v), "mean": sum(v) / len(v) if v else None} for k, v in cls.items()}
    if args.forward and not args.inplace:
        out["decode_context"] = forward_context(torch, af, ctx, wl, mats, idx, gates, stream)
    if mode == af.SWAP and not args.inplace and not args.per_matrix and not args.no_copy_ceiling:
        # practical ceiling: the plain 128-bit copy W_base -> W_work over the same tile table
        with torch.cuda.stream(stream):
            cp = timed_launches(torch, stream, lambda: ctx.fused_switch(None, None, None, None, wl.k, wl.scale,
                                                                        af.UNMERGE, stream=stream), 16)
            # ... and each direction alone over the same tiles: W_base read and discarded, W_work zeroed
            rd = timed_launches(torch, stream, lambda: ctx.hbm_probe(af.PROBE_READ_BASE, stream=stream), 16)
            wr = timed_launches(torch, stream, lambda: ctx.hbm_probe(af.PROBE_ZERO_WORK, stream=stream), 16)
            last = (args.warmup + args.steps - 1) % T   # leave W_work as the timed loop left it
            ctx.fused_switch(None, None, idx[last], gates[last], wl.k, wl.scale, af.MERGE, stream=stream)
            torch.cuda.synchronize()
        copy_gbs = 4 * wl.elements / (cp["mean"] * 1e-6) / 1e9
        read_gbs, write_gbs = (2 * wl.elements / (x["mean"] * 1e-6) / 1e9 for x in (rd, wr))
        serial_gbs = 2.0 / (1.0 / read_gbs + 1.0 / write_gbs)
        out["roofline"]["copy_kernel"] = {"us": cp["mean"], "GB/s": copy_gbs, "frac_of_peak": copy_gbs / HBM_PEAK_GBS,
                                          "switch_vs_copy": achieved / copy_gbs}
        # what the chip gives one direction at a time, and a pass that did N bytes of each back to back
        out["roofline"]["one_direction"] = {"read_only_GB/s": read_gbs, "write_only_GB/s": write_gbs,
                                            "read_then_write_GB/s": serial_gbs, "switch_vs_read_then_write": achieved / serial_gbs}
    if not args.no_cpu_baseline:
        t = (args.warmup + args.steps - 1) % T
        out["cpu_baseline"] = cpu_baseline(wl, mats, hidden, router, t, min(args.cpu_layers, wl.layers))
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
