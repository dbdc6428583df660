#!/usr/bin/env python3
"""Benchmark of the ternary pointwise-convolution path on one MI355X.

A step is one pass over all 34 pointwise layers of MobileNetV2 (width 1.0, 224x224) at batch
128 -- decode, int8 MFMA accumulation and integer requantisation of every layer -- on
seeded synthetic int8 NHWC inputs already resident in HBM.  Every layer has its own input and
output buffers, so between two uses of a buffer the sweep touches ~880 MB (more than the
256 MB Infinity Cache): the numbers are cache-cold.

Prints ONE JSON line on stdout.  Human-readable per-layer tables go to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published
MFMA_I8_PEAK_TOPS = 5000.0  # MI355X dense int8 MFMA, published
BATCH = 128
SEED = 0x50524F4D + 300


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_name(variant):
    nt, pt, ld, ks1, fullw = variant[:5]
    # last template argument: 0 = the plain epilogues (1 = PReLU, 2 = both)
    if len(variant) > 5 and variant[5]:  # row-cooperative kernel
        return f"void prom::pw_rows_kernel<{nt}, {str(ks1).lower()}, {ld}, 0>(prom::PwArgs)"
    return (f"void prom::pw_stream_kernel<{nt}, {pt}, {ld}, {str(ks1).lower()}, {str(fullw).lower()}, 0>"
            f"(prom::PwArgs)")


def measured_traffic(name):
    """HBM bytes per launch of a kernel from the committed FETCH_SIZE/WRITE_SIZE profile
    (lines 'traffic_bytes_per_launch[<kernel>] = N'); None if the profile does not list it."""
    path = os.path.join(ROOT, "profiles", "pw_sweep_mobilenetv2_b128.hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch[") and f"[{name}]" in line:
                return int(line.rsplit("=", 1)[1])
    except OSError:
        pass
    return None


def settle(torch, launch, ms=20.0):
    """Untimed launches for `ms` before a measurement: the step time of an idle GPU settles only
    after some tens of milliseconds of load (see the preconditioning of the timed region)."""
    t0 = time.perf_counter()
    k = 0
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(20):
            launch(k)
            k += 1
        torch.cuda.synchronize()


def layer_bytes(m, k, nc, residual=False):
    """Algorithmic HBM bytes of one layer: activations in + out (+ residual), 2-bit weights,
    12 bytes of requantisation parameters per output channel."""
    return m * (k + nc) + (m * nc if residual else 0) + ((k + 3) // 4) * nc + 12 * nc


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--precondition-ms", type=float, default=150.0,
                    help="untimed steps for this long before the warm-up steps (0: none): an idle GPU needs "
                         "some 100 steps of this load before the step time settles")
    ap.add_argument("--batch", type=int, default=BATCH, help="images per layer (metric is quoted at 128)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the depthwise / block legs")
    ap.add_argument("--dw-only", action="store_true",
                    help="run the depthwise sweep leg alone and print its record (for profiling)")
    ap.add_argument("--chain-only", action="store_true",
                    help="run the 17-block chain leg alone and print its record (for profiling)")
    ap.add_argument("--gconv-only", action="store_true",
                    help="run the grouped 3x3 legs alone and print their records (for profiling)")
    ap.add_argument("--dw-filter", default=None,
                    help="with --dw-only: HW,C,STRIDE of the one depthwise layer to run, e.g. 56,144,1")
    ap.add_argument("--cpu-sample-images", type=int, default=128)
    ap.add_argument("--zero-fraction", type=float, default=0.5,
                    help="P(weight == 0) of the synthetic ternary weights (the paper reports about 0.31 at "
                         "initialisation and 0.5-0.55 after training); the kernels are dense, so the "
                         "timing does not depend on it")
    ap.add_argument("--no-batching", action="store_true",
                    help="one launch per layer (the library's batching of small independent layers off)")
    ap.add_argument("--streams", type=int, default=1,
                    help="with N > 1: an extra leg that spreads the 34 independent layers over N streams")
    ap.add_argument("--ab", choices=["both", "mfma", "addsub"], default=None,
                    help="instead of the sweep: time the two designs of the pointwise layer "
                         "(MFMA vs add/subtract on the vector ALU) on four representative layers")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU; multi-GPU runs are not part of it "
              "(the path shards by batch with no communication). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2505_03254_amd as P
    from workloads import (make_pw_layer, make_dw_layer, make_block, mobilenetv2_pointwise_layers,
                           mobilenetv2_depthwise_layers)

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    P.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.ab:
        print(json.dumps(ab_study(P, torch, dev, args.ab, args.batch)), flush=True)
        return
    if args.chain_only:
        print(json.dumps(chain_leg(P, torch, dev, args.batch, log)), flush=True)
        return
    if args.gconv_only:
        print(json.dumps(gconv_leg(P, torch, dev, args.batch, log)), flush=True)
        return
    if args.dw_only:
        only = tuple(int(v) for v in args.dw_filter.split(",")) if args.dw_filter else None
        print(json.dumps({"depthwise_sweep": depthwise_leg(P, torch, dev, args.batch, log, only)}), flush=True)
        return
    t_setup = time.time()

    # ---- build the workload ----------------------------------------------------------------
    shapes = mobilenetv2_pointwise_layers()
    layers = []
    for i, s in enumerate(shapes):
        L = make_pw_layer(SEED + i, args.batch, s.hw, s.hw, s.cin, s.cout, p_zero=args.zero_fraction)
        x = torch.from_numpy(L.x).to(dev)
        wp = torch.from_numpy(P.prom_pack_ternary(L.weight)).to(dev)
        rq = P.Requant(torch.from_numpy(L.bias).to(dev), torch.from_numpy(L.mult).to(dev),
                       torch.from_numpy(L.shift).to(dev), 0, 127)
        y = torch.empty((args.batch, s.hw, s.hw, s.cout), dtype=torch.int8, device=dev)
        plan = P.prom_pw_plan_query(args.batch, s.hw, s.hw, s.cin, s.cout)
        # template arguments of the kernel instantiation this layer runs (as rocprofv3 names it)
        variant = (plan["tiles_per_wave"], plan["pixel_tiles"], plan["load_bytes"], s.cin <= 64,
                   s.cout % (16 * plan["tiles_per_wave"]) == 0, plan["row_waves"])
        m = args.batch * s.hw * s.hw
        layers.append(dict(shape=s, L=L, x=x, wp=wp, rq=rq, y=y, plan=plan, variant=variant, m=m,
                           bytes=layer_bytes(m, s.cin, s.cout), ops=2 * m * s.cin * s.cout))
    total_ops = sum(l["ops"] for l in layers)
    total_bytes = sum(l["bytes"] for l in layers)
    log(f"[bench] workload built in {time.time() - t_setup:.1f}s: {len(layers)} layers, "
        f"{total_bytes / 1e6:.1f} MB algorithmic, {total_ops / 1e9:.2f} Gop per step")

    # ---- launch groups: prom_pw_conv_sequence puts independent small layers into one launch
    # (prom::pw_batch_kernel) and independent large layers whose plan it carries into another
    # (prom::pw_bigbatch_kernel); every other layer is its own launch.  A group is what one kernel
    # name covers: a batch, or all single launches of one template instantiation.  The step calls
    # prom_pw_conv_sequence once per group, in the order a single call over all 34 layers would
    # launch them (large batch, single layers, small batch), so that the launches of the dominant
    # group can be bracketed by events.
    for l in layers:
        s_ = l["shape"]
        l["class"] = 0 if args.no_batching else P.prom_pw_batch_class(args.batch, s_.hw, s_.hw, s_.cin, s_.cout)
    BATCH_NAME = {1: "void prom::pw_batch_kernel<0>(prom::PwBatchArgs)",
                  2: "void prom::pw_bigbatch_kernel<0>(prom::PwBatchArgs)"}
    runs = []  # layers that go into one PwSequence call
    for cls in (2, 0, 1):
        members = [l for l in layers if l["class"] == cls]
        if cls == 0 or len(members) == 1:
            runs += [[l] for l in members]
        else:
            runs += [members[i:i + 32] for i in range(0, len(members), 32)]
    groups = {}
    run_names = []
    for r in runs:
        name = BATCH_NAME[r[0]["class"]] if len(r) > 1 else kernel_name(r[0]["variant"])
        run_names.append(name)
        g = groups.setdefault(name, {"bytes": 0, "launches": 0, "layers": []})
        g["bytes"] += sum(l["bytes"] for l in r)
        g["launches"] += 1
        g["layers"] += [l["shape"].name for l in r]
    dom_name = max(groups, key=lambda k: groups[k]["bytes"])
    segments = [(name == dom_name, P.PwSequence([(l["x"], l["wp"], l["shape"].cout, l["rq"], None, l["y"])
                                                 for l in r])) for name, r in zip(run_names, runs)]
    log(f"[bench] {len(runs)} launches per step; dominant kernel: {dom_name} "
        f"({groups[dom_name]['launches']} launch(es), {groups[dom_name]['bytes'] / 1e6:.1f} MB per step)")

    def one_step(events=None):
        for is_dom, seq in segments:
            if is_dom and events is not None:
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                seq.run()
                e1.record()
                events.append((e0, e1))
            else:
                seq.run()

    # ---- measured ceilings of this machine, beside the data-sheet ones: streaming read, streaming
    # write, copy (the library's kernels and torch's device-to-device copy) on 512 MB, and a
    # register-resident int8 MFMA loop.  They run before the timed region on purpose: an idle GPU
    # needs about 30 ms of load to reach its steady clocks (the first 30 steps after a second of
    # idling take 250 us each, the steps after the 120th 224 us), and the figure of interest is the
    # steady one. --------------------------------------------------------------------------------
    nb = 512 << 20
    src = torch.empty(nb, dtype=torch.uint8, device=dev)
    dst = torch.empty(nb, dtype=torch.uint8, device=dev)
    src.random_(0, 255)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)

    def rate(fn, nbytes, reps=5):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3 / reps
            best = t if best is None or t < best else best
        return nbytes / best / 1e9
    # (the compute-only loop first and the copies last: the memory clocks follow the memory traffic)
    mfma_iters = 20000
    mfma_ops = P.prom_mfma_i8_loop(mfma_iters, sink)
    mfma_tops = round(rate(lambda: P.prom_mfma_i8_loop(mfma_iters, sink), mfma_ops, reps=2) / 1e3, 0)
    ceilings = {
        "hbm_read_gbs": round(rate(lambda: P.prom_stream_read(src, sink), nb), 0),
        "hbm_write_gbs": round(rate(lambda: P.prom_stream_write(dst, 1), nb), 0),
        "hbm_copy_torch_gbs": round(rate(lambda: dst.copy_(src), 2 * nb), 0),
        "hbm_copy_gbs": round(rate(lambda: P.prom_copy_bytes(src, dst), 2 * nb), 0),
        "hbm_datasheet_gbs": HBM_PEAK_GBS,
        "mfma_i8_tops": mfma_tops,
        "mfma_i8_datasheet_tops": MFMA_I8_PEAK_TOPS,
    }
    copy_gbs = ceilings["hbm_copy_gbs"]
    log(f"[bench] measured ceilings: {ceilings}")
    # ---- preconditioning (disclosed in the result), warmup, then the timed region ----------------
    # After idling, and also right after the copies above, the first steps are slower than the
    # sustained rate: blocks of 5 steps take 243-264 us per step after a second of idling, 234 after
    # 60 ms of copies, and settle at 221-222 after about 100 steps.  The sustained figure is the one
    # a training or serving loop sees, so the step runs untimed for --precondition-ms first.
    precondition_steps = 0
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.precondition_ms:
        for _ in range(10):
            one_step()
        torch.cuda.synchronize()
        precondition_steps += 10
    for _ in range(max(args.warmup, 1)):
        one_step()
    torch.cuda.synchronize()
    # Events bracket the dominant launch on every EVENT_EVERY-th timed step only: a pair of event
    # records costs the step about 6 us (measured: 229 us with them on every step, 223 without).
    EVENT_EVERY = 10
    events = []
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(events if k % EVENT_EVERY == 0 else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = total_ops / (ms_per_step * 1e-3) / 1e9  # Gop/s
    dom_ms = [e0.elapsed_time(e1) for e0, e1 in events]
    dom_avg_us = 1e3 * sum(dom_ms) / len(dom_ms)
    dom_bytes_per_launch = groups[dom_name]["bytes"] / groups[dom_name]["launches"]
    dom_achieved = dom_bytes_per_launch / (dom_avg_us * 1e-6) / 1e9

    # ---- per-layer table, one launch per layer (the dependent path: in a network a layer reads the
    # previous layer's output, so nothing can share a launch).  Protocol: events around 100
    # back-to-back launches after 10 warm-ups, median of 5 repeats; cache-cold: the launches rotate
    # over enough input/output sets that more than 512 MB are touched between two uses of a set
    # (the Infinity Cache holds 256 MB).  "hot" is the same on one set (cache-assisted, not a
    # roofline figure).  20 ms of untimed launches of the layer come before its warm-ups, so that
    # every row is taken at the GPU's sustained rate. ----------------------------------------------
    per_layer = []
    log(f"{'layer':<13}{'HW':>4}{'Cin':>5}{'Cout':>6} {'plan(NT,PT,ld)':>15} {'cold us':>8} {'GB/s':>8} "
        f"{'%HBM':>6} {'Gop/s':>9} {'%MFMA':>6} {'bound':>6} {'%roof':>6} {'hot us':>7}")
    LAUNCHES, REPEATS, WARM = 100, 5, 10
    for l in layers:
        s = l["shape"]
        nsets = min(128, int(512e6 // l["bytes"]) + 2)
        xs = [l["x"]] + [l["x"].clone() for _ in range(nsets - 1)]
        ys = [l["y"]] + [torch.empty_like(l["y"]) for _ in range(nsets - 1)]
        seqs = [P.PwSequence([(xs[k], l["wp"], s.cout, l["rq"], None, ys[k])]) for k in range(nsets)]

        def timed(sq_list):
            settle(torch, lambda k: sq_list[k % len(sq_list)].run())
            for k in range(WARM):
                sq_list[k % len(sq_list)].run()
            torch.cuda.synchronize()
            reps_us = []
            for _ in range(REPEATS):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                for k in range(LAUNCHES):
                    sq_list[k % len(sq_list)].run()
                e1.record()
                torch.cuda.synchronize()
                reps_us.append(e0.elapsed_time(e1) * 1e3 / LAUNCHES)
            return sorted(reps_us)[len(reps_us) // 2]
        us = timed(seqs)
        hot_us = timed(seqs[:1])
        del xs, ys, seqs
        gbs = l["bytes"] / (us * 1e-6) / 1e9
        gops = l["ops"] / (us * 1e-6) / 1e9
        t_hbm = l["bytes"] / (HBM_PEAK_GBS * 1e3)        # us at the data-sheet bandwidth
        t_mfma = l["ops"] / (MFMA_I8_PEAK_TOPS * 1e6)    # us at the data-sheet int8 MFMA peak
        bound = "hbm" if t_hbm >= t_mfma else "mfma"
        frac = max(t_hbm, t_mfma) / us
        per_layer.append(dict(layer=s.name, us=round(us, 2), hot_us=round(hot_us, 2), gbs=round(gbs, 1),
                              gops=round(gops, 1), bound=bound, frac_roofline=round(frac, 4)))
        log(f"{s.name:<13}{s.hw:>4}{s.cin:>5}{s.cout:>6} {str(l['variant'][:3]):>15} {us:8.2f} {gbs:8.1f} "
            f"{100 * gbs / HBM_PEAK_GBS:6.1f} {gops:9.1f} {100 * gops / (MFMA_I8_PEAK_TOPS * 1e3):6.1f} {bound:>6} "
            f"{100 * frac:6.1f} {hot_us:7.2f}")
    sum_us = sum(p["us"] for p in per_layer)
    log(f"one launch per layer, cache-cold, sum over the 34 layers: {sum_us:.1f} us "
        f"({total_bytes / (sum_us * 1e-6) / 1e9:.0f} GB/s, {100 * total_bytes / (sum_us * 1e-6) / 1e9 / HBM_PEAK_GBS:.1f}% "
        f"of the HBM roofline)  (shared launches: {ms_per_step * 1e3:.1f} us/step)")

    # ---- extra leg: the same 34 independent layers spread round-robin over several streams, so
    # that one layer's launch, prologue and write-back overlap with another layer's streaming ----
    conc = None
    if args.streams > 1:
        streams = [torch.cuda.Stream(device=dev) for _ in range(args.streams)]
        order = sorted(range(len(layers)), key=lambda i: -layers[i]["bytes"])  # big layers first
        per_stream = [[] for _ in streams]
        for rank, i in enumerate(order):
            l = layers[i]
            per_stream[rank % len(streams)].append((l["x"], l["wp"], l["shape"].cout, l["rq"], None, l["y"]))
        stream_seqs = [P.PwSequence(lst) for lst in per_stream]

        def conc_step():
            start = torch.cuda.Event()
            start.record()
            for st, sq in zip(streams, stream_seqs):
                st.wait_event(start)
                sq.run(stream=st)
                done = torch.cuda.Event()
                done.record(st)
                torch.cuda.current_stream().wait_event(done)
        for _ in range(3):
            conc_step()
        torch.cuda.synchronize()
        tc0 = time.perf_counter()
        for _ in range(args.steps):
            conc_step()
        torch.cuda.synchronize()
        conc_ms = (time.perf_counter() - tc0) * 1e3 / args.steps
        conc = {"streams": args.streams, "ms_per_step": round(conc_ms, 4),
                "gops": round(total_ops / (conc_ms * 1e-3) / 1e9, 1),
                "gbs": round(total_bytes / (conc_ms * 1e-3) / 1e9, 1),
                "frac_hbm_roofline": round(total_bytes / (conc_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        log(f"[bench] {args.streams} streams, layers overlapped: {conc_ms * 1e3:.1f} us/step, "
            f"{conc['gbs']:.0f} GB/s ({100 * conc['frac_hbm_roofline']:.1f}% of the HBM roofline)")

    # One pass of the sweep right after that copy has gone through the caches (1 GB of traffic, four
    # times the Infinity Cache): what a pass costs when nothing of it is cached, against the
    # back-to-back figure of the timed region, where a step starts among the dirty lines of the last.
    cold = []
    for _ in range(9):
        P.prom_copy_bytes(src, dst)
        c0 = torch.cuda.Event(enable_timing=True)
        c1 = torch.cuda.Event(enable_timing=True)
        c0.record()
        one_step()
        c1.record()
        torch.cuda.synchronize()
        cold.append(c0.elapsed_time(c1) * 1e3)
    cold_pass_us = sorted(cold)[len(cold) // 2]
    del src, dst
    log(f"[bench] one pass after a cache-flushing copy: {cold_pass_us:.1f} us (median of {len(cold)})")

    result = {
        "metric": "ternary pointwise conv Gop/s and % of roofline, MobileNetV2 layers, batch 128",
        "value": round(value, 1),
        "unit": "Gop/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "precondition_steps": precondition_steps,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": "configs[3]: the 34 ternary pointwise layers of MobileNetV2 1.0 (224x224), "
                               f"batch {args.batch}, int8 NHWC, through prom_pw_conv_sequence",
                   "batch": args.batch, "layers": len(layers), "launches_per_step": len(runs),
                   "weight_zero_fraction": args.zero_fraction},
        "sweep": {"algorithmic_bytes": total_bytes, "dense_equiv_ops": total_ops,
                  "gbs": round(total_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                  "frac_hbm_roofline": round(total_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                  "gadd_per_s": round(value / 2, 1),
                  "sum_layer_event_us": round(sum_us, 1),
                  "sum_layer_frac_hbm_roofline": round(total_bytes / (sum_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                  "copy_kernel_gbs": round(copy_gbs, 0),
                  "frac_of_measured_copy": round(total_bytes / (ms_per_step * 1e-3) / 1e9 / copy_gbs, 4),
                  "pass_after_cache_flush_us": round(cold_pass_us, 1),
                  "layers_overlapped_on_streams": conc},
        "roofline": {"bound": "hbm", "kernel": dom_name,
                     "layers": groups[dom_name]["layers"],
                     "achieved": round(dom_achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(dom_achieved / HBM_PEAK_GBS, 4),
                     "avg_launch_us": round(dom_avg_us, 2),
                     "launches_timed": len(dom_ms),
                     "timing": f"HIP events around the launch on every {EVENT_EVERY}th step of the timed region "
                               "(a pair of event records costs a step about 6 us)",
                     "bytes_per_launch": int(dom_bytes_per_launch),
                     "traffic": measured_traffic(dom_name),
                     "traffic_source": "profiles/pw_sweep_mobilenetv2_b128.hbm_traffic.txt (rocprofv3 --pmc runs of this "
                                       "command; counters cannot be read inside the timed run)",
                     # the whole step (every launch of the sweep, gaps included) against the same peak
                     "step_achieved": round(total_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                     "step_frac": round(total_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     # one launch per layer (what a network, where each layer reads the previous one, runs)
                     "one_launch_per_layer_frac": round(total_bytes / (sum_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)},
        "ceilings": ceilings,
        "per_layer": per_layer,
    }

    # ---- extra legs: depthwise sweep and the fused block of config 4 ---------------------------
    if not args.no_extra:
        result["extra"] = extra_legs(P, torch, dev, args.batch, log)
        from workloads import regnetx_400mf_pointwise_layers, resnext50_32x4d_pointwise_layers
        result["extra"]["pw_regnetx_400mf"] = family_leg(P, torch, dev, args.batch, regnetx_400mf_pointwise_layers(),
                                                         log, "pw_regnetx_400mf")
        result["extra"]["pw_resnext50"] = family_leg(P, torch, dev, args.batch, resnext50_32x4d_pointwise_layers(),
                                                     log, "pw_resnext50")
        # the sweep at other batch sizes and weight zero fractions (the paper: 31 % of the ternary
        # weights are zero at initialisation, up to 55 % in a trained layer; the kernels are dense)
        for key, b_, z_ in (("sweep_batch32", 32, 0.5), ("sweep_batch256", 256, 0.5),
                            ("sweep_zero_fraction_0.31", args.batch, 0.31),
                            ("sweep_zero_fraction_0.55", args.batch, 0.55)):
            result["extra"][key] = quick_sweep(P, torch, dev, b_, z_)
            log(f"[bench] {key}: {result['extra'][key]}")

    # ---- CPU baseline: the oracle on a bounded sample, plus a parity check of that sample ------
    if not args.no_cpu_baseline:
        import oracle
        ns = min(args.cpu_sample_images, args.batch)
        torch.cuda.synchronize()
        ops = 0
        t_cpu = 0.0
        mismatches = 0
        for l in layers:
            L, s = l["L"], l["shape"]
            xs = np.ascontiguousarray(L.x[:ns])
            tc = time.perf_counter()
            want = oracle.pw_conv(xs, L.weight, L.bias, L.mult, L.shift, 0, 127)
            t_cpu += time.perf_counter() - tc
            ops += 2 * ns * s.hw * s.hw * s.cin * s.cout
            got = l["y"][:ns].cpu().numpy()
            bad = int((got != want).sum())
            if bad:
                where = np.argwhere(got != want)
                log(f"[bench] PARITY: layer {s.name} differs from the oracle in {bad} elements, first at {where[0].tolist()}, last at {where[-1].tolist()}")
            mismatches += bad
        # the same oracle with one thread, on the first image of every layer (bounded: about 0.5 Gop)
        all_threads = oracle.max_threads()
        oracle.set_threads(1)
        ops1, t1cpu = 0, 0.0
        for l in layers:
            L, s = l["L"], l["shape"]
            xs = np.ascontiguousarray(L.x[:1])
            tc = time.perf_counter()
            oracle.pw_conv(xs, L.weight, L.bias, L.mult, L.shift, 0, 127)
            t1cpu += time.perf_counter() - tc
            ops1 += 2 * s.hw * s.hw * s.cin * s.cout
        oracle.set_threads(all_threads)
        result["cpu_baseline"] = {"value": round(ops / t_cpu / 1e9, 2), "unit": "Gop/s",
                                  "cores": all_threads, "kind": "oracle",
                                  "sample": f"first {ns} of {args.batch} images of every layer "
                                            f"({ops / 1e9:.1f} Gop, {t_cpu:.1f} s)",
                                  "parity_mismatches_vs_gpu": mismatches,
                                  "single_thread": {"value": round(ops1 / t1cpu / 1e9, 2), "unit": "Gop/s", "cores": 1,
                                                    "sample": f"first image of every layer ({ops1 / 1e9:.2f} Gop, "
                                                              f"{t1cpu:.1f} s)"}}
        log(f"[bench] oracle: {ops / t_cpu / 1e9:.2f} Gop/s on {all_threads} threads, "
            f"{ops1 / t1cpu / 1e9:.2f} Gop/s on one; GPU outputs of the sample differ in {mismatches} elements")

    # ---- extra leg: the same sweep as a PReLU network (the paper's MobileNetV2 variant: PReLU
    # after every expand layer and the head, none after the project layers) -----------------------
    if not args.no_extra:
        result.setdefault("extra", {})["prelu_sweep"] = prelu_leg(P, torch, dev, layers, args, total_bytes,
                                                                  not args.no_cpu_baseline, log)

    print(json.dumps(result), flush=True)


def quick_sweep(P, torch, dev, batch, zero_fraction, steps=20):
    """The 34-layer sweep through prom_pw_conv_sequence at another batch size or weight zero
    fraction: seeded weights and parameters, random activations (no parity check here: the parity
    tests cover these shapes), same timing as the main timed region."""
    from workloads import make_pw_layer, mobilenetv2_pointwise_layers
    shapes = mobilenetv2_pointwise_layers()
    nbytes = sum(layer_bytes(batch * s.hw * s.hw, s.cin, s.cout) for s in shapes)
    ops = sum(2 * batch * s.hw * s.hw * s.cin * s.cout for s in shapes)
    # a sweep whose tensors would fit the 256 MB last-level cache (batch 32: 220 MB) rotates over
    # several sets of them, so that no step finds its input cached by the step before
    nsets = max(1, -(-600_000_000 // nbytes))
    params = []
    for i, s in enumerate(shapes):
        L = make_pw_layer(SEED + 7000 + i, 1, 1, 1, s.cin, s.cout, p_zero=zero_fraction)
        params.append((torch.from_numpy(P.prom_pack_ternary(L.weight)).to(dev),
                       P.Requant(torch.from_numpy(L.bias).to(dev), torch.from_numpy(L.mult).to(dev),
                                 torch.from_numpy(L.shift).to(dev), 0, 127)))
    seqs = []
    for _ in range(nsets):
        seq_layers = []
        for s, (wp, rq) in zip(shapes, params):
            x = torch.randint(0, 128, (batch, s.hw, s.hw, s.cin), dtype=torch.int8, device=dev)
            y = torch.empty((batch, s.hw, s.hw, s.cout), dtype=torch.int8, device=dev)
            seq_layers.append((x, wp, s.cout, rq, None, y))
        seqs.append(P.PwSequence(seq_layers))
    for k in range(60 * nsets):  # (to the sustained rate, as the main timed region)
        seqs[k % nsets].run()
    torch.cuda.synchronize()
    steps *= nsets
    t0 = time.perf_counter()
    for k in range(steps):
        seqs[k % nsets].run()
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) * 1e6 / steps
    return {"batch": batch, "weight_zero_fraction": zero_fraction, "tensor_sets_in_rotation": nsets, "us": round(us, 1),
            "gops": round(ops / (us * 1e-6) / 1e9, 1), "gbs": round(nbytes / (us * 1e-6) / 1e9, 1),
            "frac_hbm_roofline": round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}


def family_leg(P, torch, dev, batch, shapes, log, tag):
    """The pointwise layers of another architecture family (RegNetX-400MF, ResNeXt-50 32x4d) at the
    benchmark's batch: every unique shape timed by the per-layer protocol (one launch per layer,
    100 launches after 10 warm-ups, median of 5, rotating over enough buffer sets to stay
    cache-cold) against the roofline that binds it (HBM at 8 TB/s or the int8 matrix units at
    5 Pop/s), and all layers of the network in one prom_pw_conv_sequence call.  Seeded weights and
    parameters, random activations (the parity tests cover these shapes, full outputs)."""
    from workloads import make_pw_layer
    uniq = {}
    for sh in shapes:
        uniq.setdefault((sh.hw, sh.cin, sh.cout, sh.residual), []).append(sh.name)
    rows, tensors = [], {}
    log(f"[bench] {tag}: {len(shapes)} pointwise layers, {len(uniq)} unique shapes, batch {batch}")
    for i, ((hw, k, n, res), names) in enumerate(uniq.items()):
        L = make_pw_layer(SEED + 9000 + i, 1, 1, 1, k, n)
        wp = torch.from_numpy(P.prom_pack_ternary(L.weight)).to(dev)
        rq = P.Requant(torch.from_numpy(L.bias).to(dev), torch.from_numpy(L.mult).to(dev),
                       torch.from_numpy(L.shift).to(dev), -128 if res else 0, 127)
        m = batch * hw * hw
        nbytes, ops = layer_bytes(m, k, n, res), 2 * m * k * n
        nsets = min(64, int(512e6 // nbytes) + 2)
        xs = [torch.randint(0, 128, (batch, hw, hw, k), dtype=torch.int8, device=dev) for _ in range(nsets)]
        ys = [torch.empty((batch, hw, hw, n), dtype=torch.int8, device=dev) for _ in range(nsets)]
        r = torch.randint(-64, 64, (batch, hw, hw, n), dtype=torch.int8, device=dev) if res else None
        seqs = [P.PwSequence([(xs[j], wp, n, rq, r, ys[j])]) for j in range(nsets)]
        settle(torch, lambda j: seqs[j % nsets].run())
        for j in range(10):
            seqs[j % nsets].run()
        torch.cuda.synchronize()
        reps = []
        for _ in range(5):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for j in range(100):
                seqs[j % nsets].run()
            e1.record()
            torch.cuda.synchronize()
            reps.append(e0.elapsed_time(e1) * 1e3 / 100)
        us = sorted(reps)[len(reps) // 2]
        t_hbm, t_mfma = nbytes / (HBM_PEAK_GBS * 1e3), ops / (MFMA_I8_PEAK_TOPS * 1e6)
        rows.append({"hw": hw, "cin": k, "cout": n, "residual": res, "count": len(names), "us": round(us, 2),
                     "bound": "hbm" if t_hbm >= t_mfma else "mfma",
                     "frac_roofline": round(max(t_hbm, t_mfma) / us, 4),
                     "gbs": round(nbytes / us / 1e3, 1), "tops": round(ops / us / 1e6, 1),
                     "roofline_us": max(t_hbm, t_mfma)})
        log(f"  {hw:>4}x{hw:<4}{k:>5} ->{n:>5} res={int(res)} x{len(names):<2} {us:8.2f} us  "
            f"{rows[-1]['bound']:>4}-bound  {100 * rows[-1]['frac_roofline']:5.1f} % of its roofline")
        tensors[(hw, k, n, res)] = (xs[0], wp, n, rq, r, ys[0])
        del xs, ys, seqs
    # the whole network's layers in one call (independent here: the library may share launches).
    # Every layer has tensors of its own, as in the network (layers of one shape that read the same
    # input would find it cached, and layers that write the same buffer are ordered, not
    # concurrent); a network that would fit the last-level cache rotates over several sets.
    total = sum(layer_bytes(batch * sh.hw * sh.hw, sh.cin, sh.cout, sh.residual) for sh in shapes)
    nsets = max(1, -(-600_000_000 // total))
    seqs = []
    for _ in range(nsets):
        seq_layers = []
        for sh in shapes:
            x, wp, n, rq, r, y = tensors[(sh.hw, sh.cin, sh.cout, sh.residual)]
            seq_layers.append((torch.randint(0, 128, x.shape, dtype=torch.int8, device=dev), wp, n, rq,
                               torch.randint(-64, 64, y.shape, dtype=torch.int8, device=dev) if r is not None else None,
                               torch.empty_like(y)))
        seqs.append(P.PwSequence(seq_layers))
    del tensors
    settle(torch, lambda j: seqs[j % nsets].run(), ms=40.0)
    reps = 20 * nsets
    t0 = time.perf_counter()
    for j in range(reps):
        seqs[j % nsets].run()
    torch.cuda.synchronize()
    seq_us = (time.perf_counter() - t0) * 1e6 / reps
    sum_us = sum(r["us"] * r["count"] for r in rows)
    roof_us = sum(r.pop("roofline_us") * r["count"] for r in rows)
    log(f"[bench] {tag}: one launch per layer {sum_us:.1f} us ({100 * roof_us / sum_us:.1f} % of the per-layer "
        f"rooflines' sum {roof_us:.1f} us); one sequence call {seq_us:.1f} us ({100 * roof_us / seq_us:.1f} %)")
    return {"batch": batch, "layers": len(shapes), "sum_layer_us": round(sum_us, 1),
            "roofline_us": round(roof_us, 1), "frac_roofline": round(roof_us / sum_us, 4),
            "one_sequence_call_us": round(seq_us, 1), "one_sequence_call_frac_roofline": round(roof_us / seq_us, 4),
            "tensor_sets_in_rotation": nsets,
            "per_shape": rows}


def prelu_leg(P, torch, dev, layers, args, total_bytes, check, log):
    import numpy as np
    from workloads import prelu_mult_neg
    seq_layers, prelu_layers = [], []
    for i, l in enumerate(layers):
        s, L = l["shape"], l["L"]
        is_act = not s.name.endswith("project")
        mneg = prelu_mult_neg(SEED + 500 + i, L.mult) if is_act else None
        rq = P.Requant(l["rq"].bias, l["rq"].mult, l["rq"].shift, -128, 127,
                       torch.from_numpy(mneg).to(dev) if is_act else None)
        seq_layers.append((l["x"], l["wp"], s.cout, rq, None, l["y"]))
        if is_act:
            prelu_layers.append((l, mneg))
    seq = P.PwSequence(seq_layers)
    for _ in range(3):
        seq.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        seq.run()
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) * 1e6 / args.steps
    out = {"prelu_layers": len(prelu_layers), "us": round(us, 1),
           "gbs": round(total_bytes / (us * 1e-6) / 1e9, 1),
           "frac_hbm_roofline": round(total_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
    if check:
        import oracle
        bad = 0
        for l, mneg in prelu_layers:
            L = l["L"]
            want = oracle.pw_conv(np.ascontiguousarray(L.x[:2]), L.weight, L.bias, L.mult, L.shift, -128, 127,
                                  mult_neg=mneg)
            bad += int((l["y"][:2].cpu().numpy() != want).sum())
        out["parity_mismatches_vs_oracle"] = bad
    log(f"[bench] PReLU sweep ({len(prelu_layers)} of {len(layers)} layers with PReLU): {us:.1f} us/step, "
        f"{out['gbs']:.0f} GB/s")
    return out


def ab_study(P, torch, dev, which, batch):
    """Design A (int8 MFMA, prom_pw_conv) against design B (add/subtract on the vector ALU,
    prom_pw_conv_addsub) on four layers of the sweep, cache-cold (rotating buffer sets)."""
    from workloads import make_pw_layer
    out = {"metric": "A/B of the pointwise designs, us per launch", "batch": batch, "layers": []}
    for name, hw, cin, cout in (("b2.expand", 112, 16, 96), ("b3.project", 56, 144, 24),
                                ("b8.expand", 14, 64, 384), ("b5.expand", 28, 32, 192)):
        m = batch * hw * hw
        nbytes = layer_bytes(m, cin, cout)
        sets = max(2, int(600e6 // nbytes) + 1)
        L = make_pw_layer(SEED + 4000 + cin, 1, 1, 1, cin, cout)
        xs = [torch.randint(0, 128, (batch, hw, hw, cin), dtype=torch.int8, device=dev) for _ in range(sets)]
        ys = [torch.empty((batch, hw, hw, cout), dtype=torch.int8, device=dev) for _ in range(sets)]
        wp = torch.from_numpy(P.prom_pack_ternary(L.weight)).to(dev)
        rq = P.Requant(torch.from_numpy(L.bias).to(dev), torch.from_numpy(L.mult).to(dev),
                       torch.from_numpy(L.shift).to(dev), 0, 127)

        def timeit(fn, reps=10):
            for i in range(2):
                fn(xs[i % sets], wp, cout, rq, None, ys[i % sets])
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(reps):
                fn(xs[i % sets], wp, cout, rq, None, ys[i % sets])
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps
        row = {"layer": name, "cin": cin, "cout": cout, "pixels": m,
               "hbm_ideal_us": round(nbytes / (HBM_PEAK_GBS * 1e3), 2)}
        if which in ("both", "mfma"):
            row["mfma_us"] = round(timeit(P.prom_pw_conv), 2)
        if which in ("both", "addsub"):
            row["addsub_us"] = round(timeit(P.prom_pw_conv_addsub), 2)
        out["layers"].append(row)
        log(f"[ab] {row}")
        del xs, ys
    return out


def depthwise_leg(P, torch, dev, batch, log, only=None):
    """The 17 depthwise 3x3 layers of MobileNetV2 at the benchmark's batch: the whole sweep through
    one prom_dw_conv_sequence call (independent layers), and every layer alone by the per-layer
    protocol (cache-cold, one launch per layer)."""
    from workloads import make_dw_layer, mobilenetv2_depthwise_layers
    dws = []
    for i, d in enumerate(mobilenetv2_depthwise_layers()):
        if only is not None and (d.hw_in, d.c, d.stride) != only:
            continue
        D = make_dw_layer(SEED + 1000 + i, 1, d.hw_in, d.hw_in, d.c, d.stride)
        x = torch.randint(0, 128, (batch, d.hw_in, d.hw_in, d.c), dtype=torch.int8, device=dev)
        w = torch.from_numpy(D.weight).to(dev)
        rq = P.Requant(torch.from_numpy(D.bias).to(dev), torch.from_numpy(D.mult).to(dev),
                       torch.from_numpy(D.shift).to(dev), 0, 127)
        ho = (d.hw_in - 1) // d.stride + 1
        y = torch.empty((batch, ho, ho, d.c), dtype=torch.int8, device=dev)
        dws.append((d, x, w, rq, y, batch * d.c * (d.hw_in ** 2 + ho ** 2)))

    # all layers with one host call (independent layers: the library may share a launch)
    # (over several sets of tensors where one set would fit the 256 MB last-level cache)
    nbytes = sum(b for *_, b in dws)
    nsets_seq = max(1, -(-600_000_000 // nbytes)) if only is None else 1
    dw_seqs = [P.DwSequence([(x, w, d.stride, rq, y) for d, x, w, rq, y, _b in dws])]
    for _ in range(nsets_seq - 1):
        dw_seqs.append(P.DwSequence([(torch.randint(0, 128, x.shape, dtype=torch.int8, device=dev), w, d.stride, rq,
                                      torch.empty_like(y)) for d, x, w, rq, y, _b in dws]))
    settle(torch, lambda k: dw_seqs[k % nsets_seq].run(), ms=40.0)
    reps = 20 * nsets_seq
    t0 = time.perf_counter()
    for k in range(reps):
        dw_seqs[k % nsets_seq].run()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    del dw_seqs
    per_layer = []
    for d, x, w, rq, y, nb in dws:
        nsets = min(64, int(512e6 // nb) + 2)
        xs = [x] + [x.clone() for _ in range(nsets - 1)]
        ys = [y] + [torch.empty_like(y) for _ in range(nsets - 1)]
        seqs = [P.DwSequence([(xs[k], w, d.stride, rq, ys[k])]) for k in range(nsets)]
        settle(torch, lambda k: seqs[k % nsets].run(), ms=10.0)
        reps_us = []
        for _ in range(5):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for k in range(100):
                seqs[k % nsets].run()
            e1.record()
            torch.cuda.synchronize()
            reps_us.append(e0.elapsed_time(e1) * 1e3 / 100)
        us = sorted(reps_us)[2]
        per_layer.append({"layer": d.name, "hw": d.hw_in, "c": d.c, "stride": d.stride, "us": round(us, 2),
                          "gbs": round(nb / us / 1e3, 1), "frac_hbm_roofline": round(nb / us / 1e3 / HBM_PEAK_GBS, 4)})
        del xs, ys, seqs
    res = {"layers": len(dws), "us": round(dt * 1e6, 1), "gbs": round(nbytes / dt / 1e9, 1),
           "frac_hbm_roofline": round(nbytes / dt / 1e9 / HBM_PEAK_GBS, 4),
           "tensor_sets_in_rotation": nsets_seq,
           "sum_layer_us": round(sum(p["us"] for p in per_layer), 1), "per_layer": per_layer}
    log(f"[bench] depthwise sweep: {dt * 1e6:.1f} us, {nbytes / dt / 1e9:.0f} GB/s "
        f"({100 * res['frac_hbm_roofline']:.1f} % of the HBM roofline); per layer (cold): "
        + ", ".join(f"{p['hw']}x{p['c']}s{p['stride']} {p['us']:.1f}" for p in per_layer))
    return res


def chain_leg(P, torch, dev, batch, log):
    """The 17 inverted-residual blocks of MobileNetV2 in network order (4 stride-2 depthwise layers),
    each fed with the previous block's output, at `batch` and at batch 8 (also replayed from a HIP
    graph); block 1 (no expansion) is a depthwise + a projection call."""
    import numpy as np
    from workloads import make_dw_layer, make_pw_layer, make_block, mobilenetv2_blocks
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    out = {}

    def time_chain(batch):
        blocks = mobilenetv2_blocks()
        cur = torch.randint(0, 128, (batch, blocks[0].hw_in, blocks[0].hw_in, blocks[0].cin), dtype=torch.int8,
                            device=dev)
        steps, fused, io_bytes, mid_bytes, ws_bytes = [], [], 0, 0, 0
        for i, b in enumerate(blocks):
            hw, ho = b.hw_in, (b.hw_in - 1) // b.stride + 1
            y = torch.empty((batch, ho, ho, b.cout), dtype=torch.int8, device=dev)
            io_bytes += batch * (hw * hw * b.cin + ho * ho * b.cout)
            if b.t == 1:
                D = make_dw_layer(SEED + 3000 + i, 1, hw, hw, b.cin, b.stride, make_x=False)
                Q = make_pw_layer(SEED + 3100 + i, 1, hw, hw, b.cin, b.cout, act_window=(-128, 127), make_x=False)
                mid = torch.empty((batch, ho, ho, b.cin), dtype=torch.int8, device=dev)
                mid_bytes += 2 * mid.numel()
                steps.append(("dwpw", cur, mid, y, b, t(D.weight), P.Requant(t(D.bias), t(D.mult), t(D.shift), 0, 127),
                              t(P.prom_pack_ternary(Q.weight)), P.Requant(t(Q.bias), t(Q.mult), t(Q.shift), -128, 127)))
            else:
                Bk = make_block(SEED + 3200 + i, 1, hw, hw, b.cin, b.t, b.cout, b.stride)
                e, d, p = Bk.expand, Bk.dw, Bk.project
                rq3 = [P.Requant(t(l.bias), t(l.mult), t(l.shift), l.act_min, l.act_max) for l in (e, d, p)]
                ws_bytes = max(ws_bytes, P.prom_block_workspace_size(batch, hw, hw, b.cin, Bk.chid, b.cout, b.stride))
                is_fused = P.prom_block_is_fused(batch, hw, hw, b.cin, Bk.chid, b.cout, b.stride)
                if is_fused:
                    fused.append(b.name)
                else:
                    mid_bytes += 2 * batch * Bk.chid * (hw * hw + ho * ho)
                steps.append(("block", cur, None, y, b, Bk.chid, t(P.prom_pack_ternary(e.weight)), t(d.weight),
                              t(P.prom_pack_ternary(p.weight)), rq3, Bk.add_residual))
            cur = y
        ws = torch.empty(ws_bytes, dtype=torch.int8, device=dev)

        def chain():
            for st in steps:
                if st[0] == "dwpw":
                    _, xi, mid, yo, b, wd_, rqd, wp_, rqp = st
                    P.prom_dw_conv(xi, wd_, b.stride, rqd, mid)
                    P.prom_pw_conv(mid, wp_, b.cout, rqp, None, yo)
                else:
                    _, xi, _m, yo, b, chid, we_, wd_, wp_, rq3, addres = st
                    P.prom_block(xi, chid, b.cout, b.stride, we_, rq3[0], wd_, rq3[1], wp_, rq3[2], addres, ws, yo)
        settle(torch, lambda k: chain(), ms=40.0)
        reps = 10
        t0 = time.perf_counter()
        for _ in range(reps):
            chain()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps

        dt_graph = None
        if batch <= 8:
            # the same chain captured once in a HIP graph and replayed: what a serving loop would do
            graph = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    chain()
            torch.cuda.current_stream().wait_stream(side)
            settle(torch, lambda k: graph.replay(), ms=40.0)
            tg = time.perf_counter()
            for _ in range(20):
                graph.replay()
            torch.cuda.synchronize()
            dt_graph = (time.perf_counter() - tg) / 20
        return dt, fused, io_bytes, mid_bytes, dt_graph

    dt, fused, io_bytes, mid_bytes, _g = time_chain(batch)
    dt8, fused8, _io8, _mid8, dt8_graph = time_chain(8)
    out["block_chain_batch8"] = {"us": round(dt8 * 1e6, 1), "us_as_hip_graph": round(dt8_graph * 1e6, 1),
                                 "one_kernel_blocks": fused8}
    log(f"[bench] 17-block chain at batch 8: {dt8 * 1e6:.1f} us per pass, {dt8_graph * 1e6:.1f} us replayed from a "
        f"HIP graph; one kernel: {', '.join(fused8)}")
    out["block_chain"] = {"blocks": 17, "us": round(dt * 1e6, 1), "one_kernel_blocks": fused,
                          "block_io_mb": round(io_bytes / 1e6, 1),
                          "intermediate_traffic_of_unfused_blocks_mb": round(mid_bytes / 1e6, 1),
                          "gbs_incl_intermediates": round((io_bytes + mid_bytes) / dt / 1e9, 1),
                          "frac_hbm_roofline_of_block_io": round(io_bytes / dt / 1e9 / HBM_PEAK_GBS, 4)}
    log(f"[bench] 17-block chain: {dt * 1e6:.1f} us per pass, one kernel: {', '.join(fused)}; "
        f"{io_bytes / 1e6:.0f} MB block inputs+outputs, {mid_bytes / 1e6:.0f} MB intermediates of unfused blocks")
    return out


def gconv_leg(P, torch, dev, batch, log):
    """The grouped 3x3 convolutions of RegNetX-400MF and ResNeXt-50 32x4d at the given batch."""
    out = {}
    from workloads import make_gconv_layer, regnetx_400mf_grouped_layers, resnext50_32x4d_grouped_layers
    for key, shapes in (("gconv_regnetx_400mf", regnetx_400mf_grouped_layers()),
                        ("gconv_resnext50_32x4d", resnext50_32x4d_grouped_layers())):
        # a family whose tensors fit the last-level cache (256 MB) is timed over several sets of
        # them in rotation, so that no step finds its input still cached from the step before
        one = batch * sum(g.c * (g.hw_in ** 2 + ((g.hw_in - 1) // g.stride + 1) ** 2) for g in shapes)
        nsets = max(1, -(-600_000_000 // one))
        sets = []
        for s_ in range(nsets):
            gl = []
            for i, g in enumerate(shapes):
                G = make_gconv_layer(SEED + 3000 + i, 1, 4, 4, g.c, g.gs, g.stride)
                x = torch.randint(0, 128, (batch, g.hw_in, g.hw_in, g.c), dtype=torch.int8, device=dev)
                if s_ == 0:
                    w = torch.from_numpy(G.weight).to(dev)
                    wf = torch.from_numpy(P.prom_gconv_pack(G.weight)).to(dev)  # weights prepared once per layer
                    rq = P.Requant(torch.from_numpy(G.bias).to(dev), torch.from_numpy(G.mult).to(dev),
                                   torch.from_numpy(G.shift).to(dev), 0, 127)
                else:
                    w, wf = sets[0][i][2]
                    rq = sets[0][i][3]
                ho = (g.hw_in - 1) // g.stride + 1
                y = torch.empty((batch, ho, ho, g.c), dtype=torch.int8, device=dev)
                gl.append((g, x, (w, wf), rq, y, batch * g.c * (g.hw_in ** 2 + ho ** 2), batch * ho * ho * g.c * 9 * g.gs))
            sets.append(gl)
        gl = sets[0]
        # the layers of the sweep are independent: one call for all (those of one matrix-core kernel
        # share a launch), and layer by layer for comparison
        gseqs = [P.GconvSequence([(x, w, g.stride, rq, y, wf) for g, x, (w, wf), rq, y, _b, _m in s_])
                 for s_ in sets]
        settle(torch, lambda k: gseqs[k % nsets].run(), ms=40.0)  # the sustained rate, as for the other legs
        reps = 10 * nsets
        tg0 = time.perf_counter()
        for k in range(reps):
            gseqs[k % nsets].run()
        torch.cuda.synchronize()
        dg = (time.perf_counter() - tg0) / reps
        for s_ in sets:
            for g, x, (w, wf), rq, y, _b, _m in s_:
                P.prom_gconv3x3(x, w, g.stride, rq, y, w_frag=wf)
        torch.cuda.synchronize()
        reps = 5 * nsets
        tg0 = time.perf_counter()
        for k in range(reps):
            for g, x, (w, wf), rq, y, _b, _m in sets[k % nsets]:
                P.prom_gconv3x3(x, w, g.stride, rq, y, w_frag=wf)
        torch.cuda.synchronize()
        dg1 = (time.perf_counter() - tg0) / reps
        gbytes = sum(b for *_, b, _m in gl)
        gmacs = sum(m for *_, m in gl)
        out[key] = {"layers": len(gl), "us": round(dg * 1e6, 1), "gbs": round(gbytes / dg / 1e9, 1),
                    "frac_hbm_roofline": round(gbytes / dg / 1e9 / HBM_PEAK_GBS, 4),
                    "useful_gmac_per_s": round(gmacs / dg / 1e9, 1), "api": "prom_gconv3x3_sequence",
                    "us_layer_by_layer": round(dg1 * 1e6, 1), "tensor_sets_in_rotation": nsets}
        log(f"[bench] {key}: {len(gl)} layers, {dg * 1e6:.1f} us in one call ({dg1 * 1e6:.1f} us layer by layer), "
            f"{gbytes / dg / 1e9:.0f} GB/s, {gmacs / dg / 1e12:.1f} Tmac/s useful")
        del gl, sets, gseqs
    return out


def extra_legs(P, torch, dev, batch, log):
    """Depthwise layers of MobileNetV2 at the same batch, and config 4's block."""
    import numpy as np
    from workloads import make_dw_layer, make_block, mobilenetv2_depthwise_layers
    out = {"depthwise_sweep": depthwise_leg(P, torch, dev, batch, log)}

    B = make_block(SEED + 2000, 64, 28, 28, 32, 6)
    e, d, p = B.expand, B.dw, B.project
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    rqs = [P.Requant(t(l.bias), t(l.mult), t(l.shift), l.act_min, l.act_max) for l in (e, d, p)]
    ws = torch.empty(P.prom_block_workspace_size(B.n, B.h, B.w, B.cin, B.chid, B.cout, 1),
                     dtype=torch.int8, device=dev)
    # rotate over enough input/output sets that the footprint between reuses exceeds the cache
    xs = [t(B.x) for _ in range(8)]
    ys = [torch.empty_like(xs[0]) for _ in range(8)]
    we, wd, wp = t(P.prom_pack_ternary(e.weight)), t(d.weight), t(P.prom_pack_ternary(p.weight))

    def run(i):
        P.prom_block(xs[i % 8], B.chid, B.cout, 1, we, rqs[0], wd, rqs[1], wp, rqs[2], True, ws, ys[i % 8])
    for i in range(8):
        run(i)
    torch.cuda.synchronize()
    reps = 40
    t0 = time.perf_counter()
    for i in range(reps):
        run(i)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    m = B.n * B.h * B.w
    compulsory = m * (B.cin + B.cout)
    out["block_config4"] = {"us": round(dt * 1e6, 1),
                            "fused": P.prom_block_is_fused(B.n, B.h, B.w, B.cin, B.chid, B.cout, 1),
                            "compulsory_gbs": round(compulsory / dt / 1e9, 1),
                            "pw_gops": round(2 * m * B.cin * B.chid * 2 / dt / 1e9, 1)}
    log(f"[bench] block (config 4): {dt * 1e6:.1f} us per call")
    del xs, ys

    out.update(chain_leg(P, torch, dev, batch, log))

    # weight preparation: float32 weights of all 34 pointwise and 17 depthwise layers through the
    # device quantisers (ternary absmean straight into the packed layout, 8-bit absmax)
    from workloads import float_conv_weights, mobilenetv2_pointwise_layers
    pws = [torch.from_numpy(float_conv_weights(SEED + 4000 + i, s_.cout, s_.cin)).to(dev)
           for i, s_ in enumerate(mobilenetv2_pointwise_layers())]
    dwf = [torch.from_numpy(float_conv_weights(SEED + 4100 + i, d.c, 9).reshape(d.c, 3, 3)).to(dev)
           for i, d in enumerate(mobilenetv2_depthwise_layers())]

    def prep():
        for w_ in pws:
            P.prom_quantize_pw_absmean(w_)
        for w_ in dwf:
            P.prom_quantize_dw_absmax(w_)
    prep()
    torch.cuda.synchronize()
    tq0 = time.perf_counter()
    for _ in range(3):
        prep()
    torch.cuda.synchronize()
    dq = (time.perf_counter() - tq0) / 3
    nweights = sum(w_.numel() for w_ in pws) + sum(w_.numel() for w_ in dwf)
    out["weight_prep"] = {"layers": len(pws) + len(dwf), "weights": nweights, "us": round(dq * 1e6, 1),
                          "note": "51 small launches; host call overhead dominates"}
    log(f"[bench] weight preparation: {nweights} float32 weights of {len(pws) + len(dwf)} layers in {dq * 1e6:.0f} us")

    # dynamic per-sample activation quantisation (float32 -> int8, one absmax scale per image)
    xa = torch.randn((batch, 56, 56, 144), dtype=torch.float32, device=dev)
    qa = torch.empty(xa.shape, dtype=torch.int8, device=dev)
    sa = torch.empty(batch, dtype=torch.float32, device=dev)
    for _ in range(2):
        P.prom_quantize_activation_absmax(xa, q=qa, scale=sa)
    torch.cuda.synchronize()
    ta0 = time.perf_counter()
    for _ in range(10):
        P.prom_quantize_activation_absmax(xa, q=qa, scale=sa)
    torch.cuda.synchronize()
    da = (time.perf_counter() - ta0) / 10
    alg = xa.numel() * 5  # read once as float32, write int8
    out["activation_quant"] = {"shape": list(xa.shape), "us": round(da * 1e6, 1),
                               "algorithmic_gbs": round(alg / da / 1e9, 1),
                               "frac_hbm_roofline": round(alg / da / 1e9 / HBM_PEAK_GBS, 4),
                               "note": "two passes over the float32 input (maximum, then quantise)"}
    log(f"[bench] activation quantiser {list(xa.shape)}: {da * 1e6:.1f} us, {alg / da / 1e9:.0f} GB/s algorithmic")
    del xa, qa

    # The same quantiser fused into the layer that produces the activations (b3.expand of MobileNetV2,
    # 24 -> 144 at 56x56): int8 in, int8 out with one dynamic scale per image, the float32 tensor
    # never written.  Algorithmic bytes: the layer's input and output once.
    from workloads import make_pw_layer
    Lf = make_pw_layer(SEED + 8000, 1, 1, 1, 24, 144)
    xf = torch.randint(-127, 128, (batch, 56, 56, 24), dtype=torch.int8, device=dev)
    wpf = torch.from_numpy(P.prom_pack_ternary(Lf.weight)).to(dev)
    gen = torch.Generator(device="cpu").manual_seed(SEED)
    x_step = (torch.rand(batch, generator=gen) * 0.05 + 0.002).to(dev)
    w_scale = (torch.rand(144, generator=gen) * 0.2 + 0.01).to(dev)
    fbias = torch.randn(144, generator=gen).to(dev)
    qf = torch.empty((batch, 56, 56, 144), dtype=torch.int8, device=dev)
    amaxf = torch.empty(batch, dtype=torch.float32, device=dev)
    scalef = torch.empty(batch, dtype=torch.float32, device=dev)

    def run_dynq():
        P.prom_pw_conv_dynq(xf, wpf, 144, x_step, w_scale, fbias, True, q=qf, amax=amaxf, scale=scalef)
    settle(torch, lambda k: run_dynq())
    tf0 = time.perf_counter()
    for _ in range(20):
        run_dynq()
    torch.cuda.synchronize()
    df = (time.perf_counter() - tf0) / 20
    algf = batch * 56 * 56 * (24 + 144)
    out["activation_quant_fused"] = {
        "layer": "24 -> 144 at 56x56 (b3.expand), ReLU, dynamic per-image output scale", "batch": batch,
        "us": round(df * 1e6, 1), "algorithmic_gbs": round(algf / df / 1e9, 1),
        "frac_hbm_roofline": round(algf / df / 1e9 / HBM_PEAK_GBS, 4),
        "unfused_bytes_per_output": 13, "fused_bytes_per_output": round(2 * 24 / 144 + 1, 2),
        "note": "three launches: clear, layer with maximum-only epilogue, layer with quantising epilogue; "
                "bit-exact against the oracle in tests/test_gpu_dynq.py"}
    log(f"[bench] layer with fused dynamic activation scale (24->144 at 56x56): {df * 1e6:.1f} us, "
        f"{algf / df / 1e9:.0f} GB/s algorithmic ({100 * algf / df / 1e9 / HBM_PEAK_GBS:.1f} % of the HBM roofline)")
    del xf, qf

    out.update(gconv_leg(P, torch, dev, batch, log))
    return out


if __name__ == "__main__":
    main()
