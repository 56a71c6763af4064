#!/usr/bin/env python3
"""Benchmark of the DGQ quantized-inference hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input of
the chosen workload: for every (activation bits, weight bits) mode, every linear
layer runs dgq_quantize_act + dgq_linear; every cross-attention runs
dgq_xattn_logq at each code width.  Inputs are resident in HBM before the timed
region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config5|config2+3]
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

PEAK_INT8_TOPS = 5000.0   # MI355X dense int8 MFMA, TOP/s
PEAK_HBM_GBS = 8000.0     # MI355X HBM3E, GB/s
TRAFFIC_NOTE = os.path.join(ROOT, "profiles", "k_linear_a8_config5_hbm_traffic.md")


def measured_traffic():
    """HBM bytes per launch of the dominant kernel, as measured with rocprofv3 --pmc and
    recorded in the committed summary (a line `traffic_bytes_per_launch: N`); None if absent."""
    try:
        for ln in open(TRAFFIC_NOTE):
            if ln.startswith("traffic_bytes_per_launch:"):
                return float(ln.split(":")[1])
    except OSError:
        pass
    return None
METRIC = "dgq_linear int8 TOPS (% MFMA peak) + xattn_logq GB/s (% HBM), 1 MI355X"


def cpu_model():
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.lower().startswith("model name"):
                return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def measure_ceilings(torch, dgq, dev, which=("mfma", "stream")):
    """What this very box delivers: the bare int8 matrix instruction and plain streaming
    kernels over a buffer eight times the 256 MB memory-side cache (best of three each)."""
    import ctypes as C
    L = dgq.lib()
    L.dgq_probe_mfma_i8.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.dgq_probe_stream.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.c_void_p]
    stream = torch.cuda.current_stream()
    sp = C.c_void_p(stream.cuda_stream)
    out = {}

    def best_us(fn, n=3):
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(n):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3
            best = us if best is None else min(best, us)
        return best

    if "mfma" in which:
        blocks, iters = 1024, 4000   # four workgroups of four waves per CU: four waves per SIMD
        sink = torch.empty(blocks * 256, dtype=torch.int32, device=dev)

        def run_mfma():
            if L.dgq_probe_mfma_i8(blocks, iters, C.c_void_p(sink.data_ptr()), sp) != 0:
                raise RuntimeError(L.dgq_last_error().decode())
        us = best_us(run_mfma)
        assert int(sink[0]) == 32 * iters, "the matrix-instruction probe computed something else"
        ops = blocks * 4.0 * iters * 4 * 2 * 32 * 32 * 32
        out["mfma_i8_tops"] = round(ops / us / 1e6, 1)
        del sink
    if "stream" in which:
        nbytes = 1 << 31
        src = torch.ones(nbytes // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        for mode, key, moved in ((0, "hbm_read_gbs", nbytes), (1, "hbm_write_gbs", nbytes),
                                 (2, "hbm_copy_gbs", 2 * nbytes)):
            def run_stream(mode=mode):
                if L.dgq_probe_stream(C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()), C.c_size_t(nbytes),
                                      mode, C.c_void_p(sink.data_ptr()), sp) != 0:
                    raise RuntimeError(L.dgq_last_error().decode())
            us = best_us(run_stream)
            out[key] = round(moved / us / 1e3, 1)
        L.dgq_probe_write_tiles.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
        for oc in (640, 5120):   # the fp32 output of the narrow and of the wide layers, 2 GiB each
            rows_t = nbytes // (4 * oc) // 128 * 128

            def run_tiles(oc=oc, rows_t=rows_t):
                if L.dgq_probe_write_tiles(C.c_void_p(dst.data_ptr()), rows_t, oc, sp) != 0:
                    raise RuntimeError(L.dgq_last_error().decode())
            us = best_us(run_tiles)
            out["tile_write_gbs_o%d" % oc] = round(4.0 * rows_t * oc / us / 1e3, 1)
        del src, dst
    torch.cuda.synchronize()
    return out


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config5", choices=["config5", "config2+3", "config4"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--step-only", action="store_true",
                    help="skip the measurements beside the step (fused gated epilogue, K-means "
                         "grouping, timestep sweep): the profiler then sees the step's launches only")
    ap.add_argument("--calib-batch", type=int, default=2,
                    help="batch elements of fresh data used for (untimed) calibration")
    ap.add_argument("--probe-copy", action="store_true",
                    help="run only a plain elementwise copy of 1 GiB (reads 1 GiB, writes 1 GiB), "
                         "three times: the reference that scales the profiler's HBM byte counters")
    ap.add_argument("--probe-mfma", action="store_true",
                    help="run only the bare v_mfma_i32_32x32x32_i8 loop and print its rate")
    ap.add_argument("--probe-stream", action="store_true",
                    help="run only the streaming read / write / copy kernels over 2 GiB and print their rates")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured ceilings (bare matrix instruction, streaming kernels)")
    ap.add_argument("--probe-selfattn", action="store_true",
                    help="run only dgq_selfattn_logq on 16 x 10 heads x 4096 tokens x 64, 8-bit codes, "
                         "three times: the launches the profiler's counters are read for")
    return ap.parse_args()


def workload(name):
    import dgq_inputs as di
    if name == "config5":
        c = di.config5()
        desc = ("config5: SDXL-scale sweep, 1024x1024, batch 8x2; linears [65536x640] and "
                "[16384x1280] (q,k,v,out, text k/v from 2048, ff.in, ff.out), G=128, A8W8 and "
                "A4W8; cross-attention 16x10 heads x 4096 queries x 77 keys, d=64, 4- and 8-bit codes")
        return c, desc
    if name == "config4":
        c4 = di.config4()
        lin, att, reps = [], [], {}
        for st in c4["stages"]:
            for ent in st["linears"]:
                lin.append(ent)
                reps[ent[0]] = st["reps"]
            for a in st["attention"]:
                att.append(a)
                reps[a[0]] = st["reps"]
        c = dict(seed=c4["seed"], linears=lin, modes=c4["modes"], attention=att,
                 attn_bits=c4["attn_bits"], reps=reps)
        desc = ("config4: every DGQ linear and cross-attention of one transformer block at each of the "
                "four stages of an SD-v1.4 UNet step, 512x512, batch 2 (64x64/320, 32x32/640, 16x16/1280, "
                "8x8/1280; blocks per stage 5/5/5/1 listed as reps), A8W8 and A8W4, 8-bit attention codes")
        return c, desc
    c2, c3 = di.config2(), di.config3()
    c = dict(seed=c2["seed"], linears=c2["linears"], modes=c2["modes"],
             attention=c3["attention"], attn_bits=c3["attn_bits"])
    desc = ("config2+3: 64x64 latent of SD-v1.4, batch 2; linears [8192x320] (q,k,v,out, ff.in, "
            "ff.out), G=64, A8W8 and A4W8; cross-attention 2x8 heads x 4096 x 77, d=40")
    return c, desc


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus %d refused); "
              "the one-GPU figure is the whole-job figure." % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import dgq_inputs as di
    import paper_2501_04304_amd as dgq

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dgq.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.probe_copy:
        n = 1 << 28
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps(dict(probe="copy", read_bytes=4 * n, write_bytes=4 * n, launches=3)))
        return
    if args.probe_mfma or args.probe_stream:
        which = (("mfma",) if args.probe_mfma else ()) + (("stream",) if args.probe_stream else ())
        print(json.dumps(dict(probe="ceilings", **measure_ceilings(torch, dgq, dev, which))))
        return
    if args.probe_selfattn:
        B_, N_, H_, d_ = 16, 4096, 10, 64
        c_ = di.selfattn_case(77, 1, N_, H_, d_)
        qs, ks, vs = (torch.from_numpy(c_[n]).to(dev).expand(B_, N_, H_, d_).contiguous() for n in ("Q", "K", "V"))
        ones = torch.ones(B_, dtype=torch.float32, device=dev)
        outs = torch.empty_like(qs)
        for _ in range(3):
            dgq.dgq_selfattn_logq(qs, ks, vs, 8, ones, out=outs)
        torch.cuda.synchronize()
        print(json.dumps(dict(probe="selfattn", B=B_, N=N_, H=H_, d=d_, launches=3)))
        return
    ceilings = None if args.no_ceilings else measure_ceilings(torch, dgq, dev)
    cfg, desc = workload(args.workload)

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # ---------------- set-up (untimed): inputs, calibration, weights, outputs -------------
    t_setup = time.time()
    layers = []
    for li, (name, M, B, N, C, O, G) in enumerate(cfg["linears"]):
        seed = di.layer_seed(cfg["seed"], li)
        run = di.linear_case(seed, B, N, C, O)
        cal = di.linear_case(seed, min(B, args.calib_batch), N, C, O, calib=True, with_weight=False)
        x = up(run["X"])
        w = up(run["W"])
        xc = up(cal["X"])
        ent = dict(name=name, M=M, B=B, N=N, C=C, O=O, G=G, x=x, seed=seed, modes={})
        for (ab, wb) in cfg["modes"]:
            g = dgq.dgq_calibrate_groups(xc, ab, G, 2)
            wt = dgq.dgq_pack_weight(g, w, None, wb)
            codes = torch.empty(dgq.codes_shape(g, M), dtype=torch.int8, device=dev)
            cls = torch.empty(M, dtype=torch.uint8, device=dev)
            ent["modes"][(ab, wb)] = dict(g=g, wt=wt, codes=codes, cls=cls, Kp=g.info.k_padded, wb=wb)
        ent["y"] = torch.empty((M, O), dtype=torch.float32, device=dev)
        del w, xc
        layers.append(ent)
    attns = []
    for ai, (name, B, N, H, d, nk, d_ctx) in enumerate(cfg["attention"]):
        c = di.attention_case(cfg["seed"] + 500 + ai, B, N, H, d, nk=nk, d_ctx=d_ctx)
        attns.append(dict(name=name, B=B, N=N, H=H, d=d, nk=nk, q=up(c["Q"]), k=up(c["K"]),
                          v=up(c["V"]), kb=up(c["key_bias"]),
                          out=torch.empty((B, N, H, d), dtype=torch.float32, device=dev),
                          s=torch.empty(B, dtype=torch.float32, device=dev),
                          ws=torch.empty(max(16, dgq.dgq_xattn_workspace_bytes(B, N, H, d, nk)),
                                         dtype=torch.uint8, device=dev)))
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    # ---------------- the step, with HIP events around every call ------------------------
    stream = torch.cuda.current_stream()
    calls = []  # (kind, key, algorithmic units)

    def plan():
        for (ab, wb) in cfg["modes"]:
            for ent in layers:
                m = ent["modes"][(ab, wb)]
                # algorithmic bytes per row: 4 C read, C (8-bit) or C / 2 (4-bit) code bytes and one
                # class byte written; the padding positions the kernel also writes are overhead
                qbytes = ent["M"] * (ent["C"] * 4 + ent["C"] * (1 if ab == 8 else 0.5) + 1)
                calls.append(("quantize_a%d" % ab, (ent, m), qbytes))
                calls.append(("linear_a%d" % ab, (ent, m), 2.0 * ent["M"] * ent["C"] * ent["O"]))
        for bits in cfg["attn_bits"]:
            for a in attns:
                abytes = 2.0 * a["B"] * a["N"] * a["H"] * a["d"] * 4  # Q read once + Out written
                calls.append(("xattn_b%d" % bits, (a, bits), abytes))
    plan()

    # Arguments are marshalled once (pointers, sizes, stream); inside the step each call is
    # one ctypes call into the C ABI, so that the host keeps ahead of the 10-20 us kernels.
    import ctypes as C
    L = dgq.lib()
    sp = C.c_void_p(stream.cuda_stream)

    def ptr(t):
        return C.c_void_p(t.data_ptr())

    def prepared(kind, key, sp=sp):
        if kind.startswith("quantize"):
            ent, m = key
            a = (C.c_void_p(m["g"].handle), ptr(ent["x"]), C.c_int64(ent["M"]), ptr(m["codes"]),
                 ptr(m["cls"]), sp)
            return L.dgq_quantize_act, a
        if kind.startswith("linear"):
            ent, m = key
            a = (C.c_void_p(m["g"].handle), C.c_void_p(m["wt"].handle), ptr(m["codes"]),
                 ptr(m["cls"]), C.c_int64(ent["M"]), ptr(ent["y"]), None, None, C.c_size_t(0), sp)
            return L.dgq_linear, a
        a_, bits = key
        a = (ptr(a_["q"]), ptr(a_["k"]), ptr(a_["v"]), ptr(a_["kb"]), a_["B"], a_["N"], a_["H"],
             a_["d"], a_["nk"], bits, ptr(a_["out"]), ptr(a_["s"]), None, ptr(a_["ws"]),
             C.c_size_t(a_["ws"].numel()), sp)
        return L.dgq_xattn_logq, a

    prep = [prepared(kind, key) for (kind, key, _) in calls]

    def run_call(ci):
        fn, a = prep[ci]
        rc = fn(*a)
        if rc != 0:
            raise dgq.DgqError(rc, L.dgq_last_error().decode())

    def step(events=None):
        for ci, (kind, key, _) in enumerate(calls):
            if events is not None:
                events[ci][0].record(stream)
            run_call(ci)
            if events is not None:
                events[ci][1].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the timed region: exactly `steps` steps, synchronised on both sides
    t0 = time.perf_counter()
    for k in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    # the same steps once more with a pair of HIP events around every call, for the
    # per-kernel figures: the 132 event records per step cost the step about a tenth, so they
    # stay out of the region `value` is computed from (their step time is reported beside it)
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in calls] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(ev[k])
    torch.cuda.synchronize()
    ms_per_step_events = (time.perf_counter() - t0) * 1e3 / args.steps

    # the step once more as one captured HIP graph (the hot calls only enqueue kernels, so
    # a caller may do this); reported beside ms_per_step, not used for `value`
    ms_per_step_graph = None
    if not args.step_only:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        spg = C.c_void_p(side.cuda_stream)
        prep_g = [prepared(kind, key, spg) for (kind, key, _) in calls]
        with torch.cuda.stream(side):
            for fn, a in prep_g:
                fn(*a)
            torch.cuda.synchronize()
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph, stream=side):
                for fn, a in prep_g:
                    if fn(*a) != 0:
                        raise dgq.DgqError(-1, L.dgq_last_error().decode())
        torch.cuda.synchronize()
        gph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            gph.replay()
        torch.cuda.synchronize()
        ms_per_step_graph = (time.perf_counter() - t0) * 1e3 / args.steps
        stream.wait_stream(side)

    # the step with the 1232-row prompt projections (each under one wave of workgroups: the
    # chip is mostly idle while they run) on a second stream of the same priority, beside the
    # layers of the latent path; forked from and joined to the main stream inside every step.
    # Reported beside ms_per_step, not used for `value`.
    ms_per_step_two_streams = None
    small = [ci for ci, (kind, key, _) in enumerate(calls)
             if not kind.startswith("xattn") and key[0]["M"] * 16 < max(e["M"] for e in layers)]
    if not args.step_only and small:
        side2 = torch.cuda.Stream()
        sp2 = C.c_void_p(side2.cuda_stream)
        prep2 = {ci: prepared(calls[ci][0], calls[ci][1], sp2) for ci in small}
        fork, join = torch.cuda.Event(), torch.cuda.Event()

        def step2():
            fork.record(stream)
            side2.wait_event(fork)
            for ci in small:
                fn, a = prep2[ci]
                if fn(*a) != 0:
                    raise dgq.DgqError(-1, L.dgq_last_error().decode())
            join.record(side2)
            for ci in range(len(calls)):
                if ci not in prep2:
                    run_call(ci)
            stream.wait_event(join)

        for _ in range(max(1, args.warmup)):
            step2()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step2()
        torch.cuda.synchronize()
        ms_per_step_two_streams = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---------------- per-kernel figures ----------------------------------------------------
    agg = {}
    for k in range(args.steps):
        for ci, (kind, key, units) in enumerate(calls):
            a = agg.setdefault(kind, dict(ms=0.0, units=0.0, launches=0))
            a["ms"] += ev[k][ci][0].elapsed_time(ev[k][ci][1])
            a["units"] += units
            a["launches"] += 1
    kernels = {}
    for kind, a in sorted(agg.items()):
        sec = a["ms"] * 1e-3
        if kind.startswith("linear"):
            ach, peak, unit, bound = a["units"] / sec / 1e12, PEAK_INT8_TOPS, "TOP/s", "mfma"
        else:
            ach, peak, unit, bound = a["units"] / sec / 1e9, PEAK_HBM_GBS, "GB/s", "hbm"
        pm = None
        if ceilings:
            # the contraction against the bare matrix instruction; the quantizer (reads 4 bytes
            # per byte it writes) against the streaming read; the attention (reads as much as it
            # writes) against the streaming copy
            pm = (ceilings["mfma_i8_tops"] if bound == "mfma" else
                  ceilings["hbm_read_gbs"] if kind.startswith("quantize") else ceilings["hbm_copy_gbs"])
        kernels[kind] = dict(bound=bound, achieved=round(ach, 2), peak=peak, unit=unit,
                             frac=round(ach / peak, 4), peak_measured=pm,
                             frac_of_measured=(round(ach / pm, 4) if pm else None),
                             avg_call_us=round(a["ms"] * 1e3 / a["launches"], 2),
                             calls_per_step=a["launches"] // args.steps)
    # per-layer view of the 8-bit contraction: % of the MFMA peak and % of the layer's own
    # roofline min(MFMA peak, algorithmic HBM bytes at the HBM peak)
    per_layer = []
    for ci, (kind, key, units) in enumerate(calls):
        if kind != "linear_a8":
            continue
        ent, m = key
        us = sum(ev[k][ci][0].elapsed_time(ev[k][ci][1]) for k in range(args.steps)) * 1e3 / args.steps
        byt = ent["M"] * m["Kp"] + ent["O"] * m["Kp"] + 4.0 * ent["M"] * ent["O"] + ent["M"]
        t_roof = max(units / (PEAK_INT8_TOPS * 1e12), byt / (PEAK_HBM_GBS * 1e9))
        per_layer.append(dict(layer=ent["name"], M=ent["M"], C=ent["C"], O=ent["O"], us=round(us, 2),
                              tops=round(units / us / 1e6, 1),
                              frac_mfma=round(units / us / 1e6 / PEAK_INT8_TOPS, 4),
                              frac_roofline=round(t_roof * 1e6 / us, 4)))
    # config 4: every call of the step as a table (one transformer block per stage; `reps` =
    # blocks of that stage in the UNet), and the UNet-wide time the table adds up to
    layer_table = None
    unet_ms = None
    if args.workload == "config4":
        layer_table, unet_ms = [], 0.0
        for ci, (kind, key, units) in enumerate(calls):
            us = sum(ev[k][ci][0].elapsed_time(ev[k][ci][1]) for k in range(args.steps)) * 1e3 / args.steps
            ent = key[0]
            reps = cfg["reps"][ent["name"]]
            row = dict(call=kind, layer=ent["name"], reps=reps, us=round(us, 2))
            if kind.startswith("xattn"):
                row.update(B=ent["B"], N=ent["N"], H=ent["H"], d=ent["d"], gbs=round(units / us / 1e3, 1))
            else:
                row.update(M=ent["M"], C=ent["C"], O=ent["O"])
                if kind.startswith("linear"):
                    row.update(w_bits=key[1]["wb"], tops=round(units / us / 1e6, 1))
                else:
                    row.update(gbs=round(units / us / 1e3, 1))
            layer_table.append(row)
            unet_ms += reps * us * 1e-3
    total_ops = sum(u for (kind, _, u) in calls if kind.startswith("linear"))
    value = total_ops / (ms_per_step * 1e-3) / 1e12
    dom = kernels["linear_a8"]
    roofline = dict(kernel="k_linear<8,false> (dgq_linear, 8-bit activation codes)",
                    bound="mfma", achieved=dom["achieved"], peak=PEAK_INT8_TOPS, unit="TOP/s",
                    frac=dom["frac"], peak_measured=dom["peak_measured"],
                    frac_of_measured=dom["frac_of_measured"],
                    traffic=measured_traffic() if args.workload == "config5" else None,
                    avg_launch_us=dom["avg_call_us"],
                    launches_per_step=dom["calls_per_step"])

    # ---------------- beyond the step: the gated feed-forward epilogue fused ----------------
    # (outside the timed step and outside `value`: the step keeps the unfused layers)
    fused = []
    for ent in layers:
        if args.step_only or not ent["name"].endswith("ff.in") or ent["O"] % 256:
            continue
        yg = torch.empty((ent["M"], ent["O"] // 2), dtype=torch.float32, device=dev)
        for (ab, wb) in cfg["modes"]:
            m = ent["modes"][(ab, wb)]
            a = (C.c_void_p(m["g"].handle), C.c_void_p(m["wt"].handle), ptr(m["codes"]),
                 ptr(m["cls"]), C.c_int64(ent["M"]), ptr(yg), sp)
            for _ in range(2):
                if L.dgq_linear_geglu(*a) != 0:
                    raise dgq.DgqError(-1, L.dgq_last_error().decode())
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            n_rep = 10
            e0.record(stream)
            for _ in range(n_rep):
                L.dgq_linear_geglu(*a)
            e1.record(stream)
            torch.cuda.synchronize()
            us_f = e0.elapsed_time(e1) * 1e3 / n_rep
            ci = [i for i, (kind, key, _) in enumerate(calls)
                  if kind == "linear_a%d" % ab and key[0] is ent][0]
            us_u = sum(ev[k][ci][0].elapsed_time(ev[k][ci][1]) for k in range(args.steps)) * 1e3 / args.steps
            ops = 2.0 * ent["M"] * ent["C"] * ent["O"]
            fused.append(dict(layer=ent["name"], act_bits=ab, us_fused=round(us_f, 2),
                              us_linear_alone=round(us_u, 2), tops_fused=round(ops / us_f / 1e6, 1)))
        # what the unfused pipeline pays on top of the plain layer: an elementwise pass over
        # y (here torch's own kernels: gelu of the gate half, then the product)
        oh = ent["O"] // 2
        for _ in range(2):
            torch.mul(ent["y"][:, :oh], torch.nn.functional.gelu(ent["y"][:, oh:]), out=yg)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(5):
            torch.mul(ent["y"][:, :oh], torch.nn.functional.gelu(ent["y"][:, oh:]), out=yg)
        e1.record(stream)
        torch.cuda.synchronize()
        us_sep = e0.elapsed_time(e1) * 1e3 / 5
        for f in fused:
            if f["layer"] == ent["name"]:
                f["us_separate_activation_pass"] = round(us_sep, 2)
        del yg

    # ---------------- beyond the step: the single-dimension grouping of Section 3.3 ----------
    # K = 16 clusters of pixels or of channels (dgq_calibrate_kmeans) on two layers, A8W8,
    # next to the same layers under the step's pixel-class x channel-group grid; and one
    # layer swept over T = 25 per-timestep table entries (Eq. 7), each step with its own handle.
    def time_calls(fn, a, n_rep=10):
        # best of three rounds: the chip's clock settles over the first few hundred microseconds
        # of a new kernel mix, and single rounds of the same call differ by up to 10 %
        for _ in range(2):
            if fn(*a) != 0:
                raise dgq.DgqError(-1, L.dgq_last_error().decode())
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(n_rep):
                fn(*a)
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / n_rep
            best = us if best is None or us < best else best
        return best

    def step_us(kind, ent):
        ci = [i for i, (k_, key, _) in enumerate(calls) if k_ == kind and key[0] is ent][0]
        return sum(ev[k][ci][0].elapsed_time(ev[k][ci][1]) for k in range(args.steps)) * 1e3 / args.steps

    kmeans = []
    sweep = None
    if args.workload == "config5" and not args.step_only:
        for ent in layers:
            if ent["name"] not in ("hi.q", "lo.ff.out"):
                continue
            cal = di.linear_case(ent["seed"], min(ent["B"], args.calib_batch), ent["N"], ent["C"],
                                 ent["O"], calib=True, with_weight=False)
            xc = up(cal["X"])
            w = up(di.linear_case(ent["seed"], 1, 2, ent["C"], ent["O"])["W"])
            for dim, dname in ((dgq.DIM_PIXEL, "pixel"), (dgq.DIM_CHANNEL, "channel")):
                g = dgq.dgq_calibrate_kmeans(xc, 8, 16, dim)
                wt = dgq.dgq_pack_weight(g, w, None, 8)
                codes = torch.empty(dgq.codes_shape(g, ent["M"]), dtype=torch.int8, device=dev)
                cls = torch.empty(ent["M"], dtype=torch.uint8, device=dev)
                us_q = time_calls(L.dgq_quantize_act, (C.c_void_p(g.handle), ptr(ent["x"]),
                                                       C.c_int64(ent["M"]), ptr(codes), ptr(cls), sp))
                us_l = time_calls(L.dgq_linear, (C.c_void_p(g.handle), C.c_void_p(wt.handle), ptr(codes),
                                                 ptr(cls), C.c_int64(ent["M"]), ptr(ent["y"]), None,
                                                 None, C.c_size_t(0), sp))
                ops = 2.0 * ent["M"] * ent["C"] * ent["O"]
                kmeans.append(dict(layer=ent["name"], dimension=dname, clusters=16,
                                   pixel_classes=g.info.n_pixel_classes, channel_groups=g.info.n_groups,
                                   k_padded=g.info.k_padded, d_star=("pixel" if g.info.dstar else "channel"),
                                   us_quantize=round(us_q, 2), us_linear=round(us_l, 2),
                                   tops_linear=round(ops / us_l / 1e6, 1),
                                   us_quantize_grid=round(step_us("quantize_a8", ent), 2),
                                   us_linear_grid=round(step_us("linear_a8", ent), 2)))
                wt.free()
                g.free()
                del codes, cls
            if ent["name"] == "hi.q":
                T = 25
                hs = []
                for t in range(T):
                    xt = xc * float(1.0 + 0.5 * np.sin(0.7 * t))  # the range drifts with the step
                    g = dgq.dgq_calibrate_kmeans(xt, 8, 16, dgq.DIM_CHANNEL)
                    hs.append((g, dgq.dgq_pack_weight(g, w, None, 8)))
                    del xt
                kp = max(g.info.k_padded for g, _ in hs)
                codes = torch.empty((ent["M"] // 16 + 1) * (kp // 64) * 1024, dtype=torch.int8, device=dev)
                cls = torch.empty(ent["M"], dtype=torch.uint8, device=dev)
                argsq = [(C.c_void_p(g.handle), ptr(ent["x"]), C.c_int64(ent["M"]), ptr(codes), ptr(cls), sp)
                         for g, _ in hs]
                argsl = [(C.c_void_p(g.handle), C.c_void_p(wt.handle), ptr(codes), ptr(cls),
                          C.c_int64(ent["M"]), ptr(ent["y"]), None, None, C.c_size_t(0), sp) for g, wt in hs]

                def sweep_once():
                    for t in range(T):
                        if L.dgq_quantize_act(*argsq[t]) != 0 or L.dgq_linear(*argsl[t]) != 0:
                            raise dgq.DgqError(-1, L.dgq_last_error().decode())
                sweep_once()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                sweep_once()
                sweep_once()
                e1.record(stream)
                torch.cuda.synchronize()
                sweep = dict(layer=ent["name"], timesteps=T, dimension="channel", clusters=16,
                             us_per_timestep=round(e0.elapsed_time(e1) * 1e3 / (2 * T), 2),
                             table_bytes=T * 16 * 2 * 4)
                for g, wt in hs:
                    wt.free()
                    g.free()
                del codes, cls
            del xc, w

    # ---------------- beyond the step: the prompt's key and value projections as one layer ---
    # A block's cross-attention projects the same 77-token context twice (to keys and to
    # values).  The step times them as the two layers they are; here the context is quantized
    # once and contracted with the two weight matrices stacked ([O_k + O_v, C]), whose
    # output's column halves are K and V.
    prompt_kv, qkv = [], []
    if args.workload == "config5" and not args.step_only:
        def stacked(names):
            group = [e for e in layers if e["name"] in names]
            if len(group) != len(names):
                return None
            e0 = group[0]
            m = e0["modes"][(8, 8)]
            M = e0["M"]
            ws_ = [up(di.linear_case(e["seed"], 1, 2, e["C"], e["O"])["W"]) for e in group]
            wt2 = dgq.dgq_pack_weight(m["g"], torch.cat(ws_, 0).contiguous(), None, 8)
            O2 = sum(e["O"] for e in group)
            y2 = torch.empty((M, O2), dtype=torch.float32, device=dev)
            us_q = time_calls(L.dgq_quantize_act, (C.c_void_p(m["g"].handle), ptr(e0["x"]), C.c_int64(M),
                                                   ptr(m["codes"]), ptr(m["cls"]), sp))
            us_l = time_calls(L.dgq_linear, (C.c_void_p(m["g"].handle), C.c_void_p(wt2.handle),
                                             ptr(m["codes"]), ptr(m["cls"]), C.c_int64(M), ptr(y2), None,
                                             None, C.c_size_t(0), sp))
            sep = sum(step_us("quantize_a8", e) + step_us("linear_a8", e) for e in group)
            wt2.free()
            return dict(layers=[e["name"] for e in group], M=M, C=e0["C"], O=O2,
                        us_quantize_once=round(us_q, 2), us_linear_stacked=round(us_l, 2),
                        us_layers_in_step=round(sep, 2))
        for pre in ("hi", "lo"):
            r = stacked((pre + ".xk", pre + ".xv"))
            if r:
                r["us_two_layers_in_step"] = r["us_layers_in_step"]
                prompt_kv.append(r)
            # the q, k and v projections of a self-attention block read one tensor as well
            r = stacked((pre + ".q", pre + ".k", pre + ".v"))
            if r:
                qkv.append(r)

    # ---------------- beyond the step: 4-bit weights stored two per byte --------------------
    # A8W4 on two layers: the handle that keeps one weight per byte against the nibble-packed
    # handle, whose weights a small kernel widens into a workspace before the contraction.
    w4 = []
    if args.workload == "config5" and not args.step_only:
        for ent in layers:
            if ent["name"] not in ("hi.ff.in", "lo.ff.out", "hi.q"):
                continue
            m = ent["modes"][(8, 8)]
            M = ent["M"]
            w = up(di.linear_case(ent["seed"], 1, 2, ent["C"], ent["O"])["W"])
            wide = dgq.dgq_pack_weight(m["g"], w, None, 4)
            packed = dgq.dgq_pack_weight(m["g"], w, None, 4).pack_nibbles()
            ws = torch.empty(dgq.dgq_linear_workspace_bytes(m["g"], packed, M), dtype=torch.uint8, device=dev)
            base = (C.c_void_p(m["g"].handle), None, ptr(m["codes"]), ptr(m["cls"]), C.c_int64(M), ptr(ent["y"]), None)
            us_w = time_calls(L.dgq_linear, base[:1] + (C.c_void_p(wide.handle),) + base[2:] + (None, C.c_size_t(0), sp))
            us_p = time_calls(L.dgq_linear, base[:1] + (C.c_void_p(packed.handle),) + base[2:] +
                              (ptr(ws), C.c_size_t(ws.numel()), sp))
            w4.append(dict(layer=ent["name"], M=M, C=ent["C"], O=ent["O"], us_byte_per_weight=round(us_w, 2),
                           us_nibble_packed=round(us_p, 2), weight_bytes=wide.device_bytes(),
                           weight_bytes_nibble_packed=packed.device_bytes()))
            wide.free()
            packed.free()
            del w, ws

    # ---------------- beyond the step: ff.in -> ff.out chained without the fp32 activation --
    # The gated layer writes the following layer's codes (dgq_linear_geglu_requant) against
    # the two calls it replaces: dgq_linear_geglu writing fp32 and dgq_quantize_act reading
    # it back.  The following layer: 16 channel clusters, 8-bit codes, calibrated on the
    # first 4096 rows of the gated layer's own output.
    chain = []
    if args.workload == "config5" and not args.step_only:
        for ent in layers:
            if not ent["name"].endswith("ff.in") or ent["O"] % 256:
                continue
            m = ent["modes"][(8, 8)]
            M, oh = ent["M"], ent["O"] // 2
            w = up(di.linear_case(ent["seed"], 1, 2, ent["C"], ent["O"])["W"])
            h = torch.empty((M, oh), dtype=torch.float32, device=dev)
            a_g = (C.c_void_p(m["g"].handle), C.c_void_p(m["wt"].handle), ptr(m["codes"]),
                   ptr(m["cls"]), C.c_int64(M), ptr(h), sp)
            us_g = time_calls(L.dgq_linear_geglu, a_g)
            for next_grouping in ("16 channel clusters", "blocks of 128 channels"):
                if next_grouping.startswith("16"):
                    g2 = dgq.dgq_calibrate_kmeans(h[:4096], 8, 16, dgq.DIM_CHANNEL)
                else:
                    g2 = dgq.dgq_calibrate_groups(h[:4096], 8, 128, 1)
                wf = dgq.dgq_pack_weight_gated_for(m["g"], g2, w, None, 8)
                codes2 = torch.empty(dgq.codes_shape(g2, M), dtype=torch.int8, device=dev)
                cls2 = torch.empty(M, dtype=torch.uint8, device=dev)
                us_q = time_calls(L.dgq_quantize_act, (C.c_void_p(g2.handle), ptr(h), C.c_int64(M),
                                                       ptr(codes2), ptr(cls2), sp))
                us_c = time_calls(L.dgq_linear_geglu_requant,
                                  (C.c_void_p(m["g"].handle), C.c_void_p(wf.handle), ptr(m["codes"]),
                                   ptr(m["cls"]), C.c_int64(M), ptr(codes2), ptr(cls2), sp))
                ops = 2.0 * M * ent["C"] * ent["O"]
                chain.append(dict(layer=ent["name"], next_grouping=next_grouping, next_channels=oh,
                                  next_k_padded=g2.info.k_padded,
                                  us_geglu_fp32=round(us_g, 2), us_quantize_next=round(us_q, 2),
                                  us_chained=round(us_c, 2), tops_chained=round(ops / us_c / 1e6, 1),
                                  bytes_not_moved=int(2 * 4 * M * oh)))
                wf.free()
                g2.free()
                del codes2, cls2
            del w, h

    # ---------------- beyond the step: the attention product on the quantized value tensor ---
    value_quant = []
    if not args.step_only:
        for a_ in attns:
            vhat = torch.empty_like(a_["v"])
            us_v = time_calls(L.dgq_quantize_value, (ptr(a_["v"]), a_["B"], a_["nk"], a_["H"], a_["d"], 8,
                                                     ptr(vhat), None, None, sp))
            us_a = time_calls(L.dgq_xattn_logq, (ptr(a_["q"]), ptr(a_["k"]), ptr(vhat), ptr(a_["kb"]), a_["B"],
                                                 a_["N"], a_["H"], a_["d"], a_["nk"], 8, ptr(a_["out"]),
                                                 ptr(a_["s"]), None, ptr(a_["ws"]),
                                                 C.c_size_t(a_["ws"].numel()), sp))
            # the log quantizer without dynamic quantization: the scale is given (here: what the
            # dynamic call just found), the kernel makes one pass over Q
            s_own = torch.empty_like(a_["s"])
            us_s = time_calls(L.dgq_xattn_logq_static, (ptr(a_["q"]), ptr(a_["k"]), ptr(a_["v"]), ptr(a_["kb"]),
                                                        a_["B"], a_["N"], a_["H"], a_["d"], a_["nk"], 8,
                                                        ptr(a_["s"]), ptr(a_["out"]), ptr(s_own), None, sp))
            # the same product on V^'s integer codes by shifts and adds (4-bit probability codes;
            # fp32 vector kernels, one thread per query and head)
            vcodes = torch.empty(a_["v"].shape, dtype=torch.uint8, device=dev)
            vparams = torch.empty((a_["B"], a_["H"], 2), dtype=torch.float32, device=dev)
            L.dgq_quantize_value(ptr(a_["v"]), a_["B"], a_["nk"], a_["H"], a_["d"], 8, ptr(vhat), ptr(vcodes),
                                 ptr(vparams), sp)
            us_i = time_calls(L.dgq_xattn_logq_intv, (ptr(a_["q"]), ptr(a_["k"]), ptr(vcodes), ptr(vparams),
                                                      ptr(a_["kb"]), a_["B"], a_["N"], a_["H"], a_["d"],
                                                      a_["nk"], 4, ptr(a_["out"]), ptr(a_["s"]), None, None, sp),
                              n_rep=3)
            nominal = 2.0 * a_["B"] * a_["N"] * a_["H"] * a_["d"] * 4
            value_quant.append(dict(attention=a_["name"], v_bits=8, attn_bits=8,
                                    us_attention_integer_shift_add_b4=round(us_i, 2),
                                    us_quantize_value=round(us_v, 2), us_attention_on_v_hat=round(us_a, 2),
                                    us_attention_given_scale=round(us_s, 2),
                                    gbs_attention_given_scale=round(nominal / us_s / 1e3, 1)))
            del vhat

    # ---------------- beyond the step: self-attention with log2-quantized probabilities ------
    # The 4096-token self-attention of the 64 x 64 latent at the sweep's batch (16 prompts x 10
    # heads of 64) with 8-bit codes against the scale 1.  Flops: the method's two products,
    # 4 N^2 d per (prompt, head); the kernel issues four times that on the matrix cores (the
    # logits twice, each as three fp16 products, and P^ V as two bf16 products).
    self_attn = []
    if args.workload == "config5" and not args.step_only:
        for (B_, N_, H_, d_) in ((16, 4096, 10, 64), (16, 1024, 20, 64)):
            c_ = di.selfattn_case(77, 1, N_, H_, d_)
            qs, ks, vs = (up(c_[n]).expand(B_, N_, H_, d_).contiguous() for n in ("Q", "K", "V"))
            outs = torch.empty_like(qs)
            ones = torch.ones(B_, dtype=torch.float32, device=dev)
            wss = torch.empty(int(L.dgq_selfattn_workspace_bytes(B_, N_, H_, d_)), dtype=torch.uint8, device=dev)
            us = time_calls(L.dgq_selfattn_logq, (ptr(qs), ptr(ks), ptr(vs), B_, N_, H_, d_, 8, ptr(ones),
                                                  ptr(outs), None, None, ptr(wss), C.c_size_t(wss.numel()), sp),
                            n_rep=5)
            flops = 4.0 * B_ * H_ * N_ * N_ * d_
            self_attn.append(dict(B=B_, N=N_, H=H_, d=d_, attn_bits=8, us=round(us, 1),
                                  tflops_method=round(flops / us / 1e6, 1),
                                  tflops_issued=round(4 * flops / us / 1e6, 1),
                                  frac_f16_mfma_peak_issued=round(4 * flops / us / 1e6 / 2500.0, 4),
                                  workspace_bytes=int(wss.numel())))
            del qs, ks, vs, outs, wss

    # ---------------- beyond the step: 3 x 3 convolutions of the U-Net's residual blocks -----
    # 16 maps of 64 x 64 x 640 and of 32 x 32 x 1280, A8W8, channel groups of 128 and one pixel
    # class (16 free-size clusters would pad every cluster of every tap to 64 positions): quantize once
    # per pixel, unfold the codes (dgq_conv3x3_codes), contract over 9 K' positions.
    conv = []
    if args.workload == "config5" and not args.step_only:
        for (B_, H_, W_, C_) in ((16, 64, 64, 640), (16, 32, 32, 1280)):
            M_ = B_ * H_ * W_
            cs = di.linear_case(91, 1, H_ * W_, C_, 8)
            xs = up(cs["X"]).repeat(B_, 1)
            g1 = dgq.dgq_calibrate_groups(xs[:H_ * W_], 8, 128, 1)
            g9 = dgq.dgq_groups_for_conv3x3(g1)
            w9 = torch.randn((C_, 9 * C_), dtype=torch.float32, device=dev) * 0.02
            wt9 = dgq.dgq_pack_weight(g9, w9, None, 8)
            c1 = torch.empty(dgq.codes_shape(g1, M_), dtype=torch.int8, device=dev)
            cl1 = torch.empty(M_, dtype=torch.uint8, device=dev)
            c9 = torch.empty(dgq.codes_shape(g9, M_), dtype=torch.int8, device=dev)
            y9 = torch.empty((M_, C_), dtype=torch.float32, device=dev)
            us_q = time_calls(L.dgq_quantize_act, (C.c_void_p(g1.handle), ptr(xs), C.c_int64(M_), ptr(c1), ptr(cl1), sp))
            us_u = time_calls(L.dgq_conv3x3_codes, (C.c_void_p(g9.handle), ptr(c1), B_, H_, W_, ptr(c9), sp))
            us_l = time_calls(L.dgq_linear, (C.c_void_p(g9.handle), C.c_void_p(wt9.handle), ptr(c9), ptr(cl1),
                                             C.c_int64(M_), ptr(y9), None, None, C.c_size_t(0), sp))
            # the same convolution with the nine taps gathered by the contraction's loads: the
            # quantizer writes three shifted copies of the codes, nothing is unfolded
            L.dgq_conv3x3_codes3_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
            L.dgq_conv3x3_codes3_bytes.restype = C.c_size_t
            c3 = torch.empty(int(L.dgq_conv3x3_codes3_bytes(C.c_void_p(g9.handle), B_, H_, W_)),
                             dtype=torch.int8, device=dev)
            us_q3 = time_calls(L.dgq_quantize_act_conv3x3, (C.c_void_p(g1.handle), C.c_void_p(g9.handle), ptr(xs),
                                                            B_, H_, W_, ptr(c3), ptr(cl1), sp))
            us_l3 = time_calls(L.dgq_linear_conv3x3, (C.c_void_p(g9.handle), C.c_void_p(wt9.handle), ptr(c3),
                                                      ptr(cl1), B_, H_, W_, ptr(y9), sp))
            ops = 2.0 * M_ * 9 * C_ * C_
            conv.append(dict(B=B_, H=H_, W=W_, C=C_, O=C_, k_padded=g9.info.k_padded,
                             us_quantize_three_copies=round(us_q3, 2), us_linear_gathering=round(us_l3, 2),
                             tops_linear_gathering=round(ops / us_l3 / 1e6, 1),
                             tops_whole_gathering=round(ops / (us_q3 + us_l3) / 1e6, 1),
                             us_quantize=round(us_q, 2), us_unfold_codes=round(us_u, 2),
                             gbs_unfold=round((c1.numel() + c9.numel()) / us_u / 1e3, 1),
                             us_linear=round(us_l, 2), tops_linear=round(ops / us_l / 1e6, 1),
                             tops_whole=round(ops / (us_q + us_u + us_l) / 1e6, 1)))
            wt9.free()
            g9.free()
            g1.free()
            del xs, w9, c1, cl1, c9, y9, c3

    # ---------------- CPU baseline: the oracle on a bounded sample --------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        # one thread on one core: pin the process for the oracle leg and restore it afterwards
        allowed = sorted(os.sched_getaffinity(0))
        pinned = allowed[0]
        os.sched_setaffinity(0, {pinned})
        t_ops = 0.0
        t_sec = 0.0
        frac = 24
        for ent in layers:
            if ent["M"] < 4096:
                continue
            rows = max(8, ent["M"] // frac)
            xs = ent["x"][:rows].cpu().numpy()
            li = [e["name"] for e in layers].index(ent["name"])
            seed = di.layer_seed(cfg["seed"], li)
            wnp = di.linear_case(seed, 1, 2, ent["C"], ent["O"])["W"]
            og = oracle.calibrate(xs, 8, ent["G"], 2)
            owq, osw = oracle.quantize_weight(wnp, 8)  # offline on both sides: not timed
            t1 = time.perf_counter()
            oq = oracle.quantize_act(og, xs)
            oracle.linear(og, oq["q"], oq["cls"], owq, osw, None)
            t_sec += time.perf_counter() - t1
            t_ops += 2.0 * rows * ent["C"] * ent["O"]
        os.sched_setaffinity(0, set(allowed))
        cpu = dict(value=round(t_ops / t_sec / 1e12, 6), unit="TOPS", cores=1, kind="oracle",
                   cpu_model=cpu_model(), nproc=os.cpu_count(), cores_allowed=len(allowed),
                   pinned_to_core=pinned,
                   sample=("first 1/%d of the rows of every large linear layer, A8W8, quantize + "
                           "contraction, single thread pinned to one core; %.1f s of CPU work" % (frac, t_sec)))

    line = dict(metric=METRIC, value=round(value, 2), unit="TOPS", n_gpus=1, steps=args.steps,
                warmup=args.warmup, ms_per_step=round(ms_per_step, 4),
                ms_per_step_with_event_records=round(ms_per_step_events, 4),
                ms_per_step_as_hip_graph=(round(ms_per_step_graph, 4) if ms_per_step_graph else None),
                ms_per_step_two_streams=(round(ms_per_step_two_streams, 4) if ms_per_step_two_streams else None),
                higher_is_better=True,
                scaling="weak", vs_baseline=None, dtype="int8", data="synthetic",
                config=dict(workload=desc, linear_ops_per_step=total_ops,
                            calls_per_step=len(calls), setup_s=round(t_setup, 1)),
                roofline=roofline, ceilings_measured=ceilings, kernels=kernels, linear_a8_layers=per_layer,
                layer_table=layer_table, ms_whole_unet_from_table=(round(unet_ms, 3) if unet_ms else None),
                linear_geglu=fused, ff_chain=chain, kmeans_grouping=kmeans, timestep_sweep=sweep, prompt_kv_stacked=prompt_kv, self_qkv_stacked=qkv, w4_nibble_packed=w4, value_quant=value_quant, self_attention=self_attn, conv3x3=conv, cpu_baseline=cpu)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
