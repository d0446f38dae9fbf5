#!/usr/bin/env python3
"""Benchmark of the DBF decode hot path on one MI355X.

Workload (the configuration the headline metric is quoted on): Llama-2-7B
attention-projection shape n_in = n_out = 4096, k = 2048 (1.0 bit/weight), batch-1
decode.  One layer holds only 2 MiB of sign bits -- less than a kernel launch
costs and small enough to sit in cache -- so the sustained number is measured on
a stream of 512 DISTINCT layers (1 GiB of signs, four times the 256 MB last-level
cache and about what one decode step of a 7B model streams) with independent
inputs, run as one dbf_stack_gemv call.  One "step" is one pass of the whole path
(x.b -> B stage -> .m -> A stage -> .a -> fp16 y) over all of them; the same stream
at 256 and 1024 layers is reported next to it (the launch head and tail are fixed
costs per step).  Inputs are resident in HBM before timing starts.

Prints ONE JSON line.  `value` is the achieved rate on ALGORITHMIC bytes
(sign bits + fp16 scale vectors + x + y; no padding, no scratch, no re-reads).
Extra keys report the per-layer time in the stream, the cache-warm latency of a
single isolated layer, the prefill rate, and the CPU oracle timed on this machine.
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

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16 matrix-core peak
MFMA_I8_PEAK_TOPS = 5000.0     # dense int8 matrix-core peak
MFMA_F32_PEAK_TFLOPS = 157.3   # dense fp32 matrix-core peak


def algorithmic_bytes(n_in, n_out, k, batch):
    """Bytes one layer product has to move: packed signs, three fp16 vectors, x in, y out."""
    bits = k * (n_in + n_out) / 8.0
    vecs = 2.0 * (n_in + n_out + k)
    io = 2.0 * batch * (n_in + n_out)
    stage_b = k * n_in / 8.0 + 2.0 * (n_in + k) + 2.0 * batch * n_in
    stage_a = k * n_out / 8.0 + 2.0 * n_out + 2.0 * batch * n_out
    return bits + vecs + io, stage_b, stage_a


def kernel_source_hash():
    """First 16 hex digits of the SHA-256 of the sources that decide what the decode launch does and reads (the
    kernel, the launch plans, the shared structs): counter readings are quoted only for the sources they were
    taken on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2505_11076_amd", "csrc")
    for name in ("dbf_gemv_mfma.hip", "dbf_api.hip", "dbf_internal.h", "dbf_kernels.h"):
        with open(os.path.join(csrc, name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


class Protocol:
    """How every rate in this file is timed, so that all figures of one output line stand on the same footing:
      1. settle: the step itself, back to back and untimed, for at least `settle_ms` of GPU time.  (After idle
         -- the host packs layers between measurements -- the shader clock is cut back about 1.5 ms into the
         load and needs about 60 ms to come back; without this phase a short run measures that transient.)
      2. `warmup` untimed steps;
      3. `steps` timed steps between two HIP events on the launch stream, nothing else in between.
    run() returns (ms per step, a dict that states what was actually done)."""

    def __init__(self, torch, steps, warmup, settle_ms):
        self.torch, self.steps, self.warmup, self.settle_ms = torch, int(steps), int(warmup), float(settle_ms)

    def run(self, step, steps=None, warmup=None):
        torch = self.torch
        steps = self.steps if steps is None else int(steps)
        warmup = self.warmup if warmup is None else int(warmup)
        ev = torch.cuda.Event
        settle_steps, settle_ms = 0, 0.0
        if self.settle_ms > 0:
            # bursts of steps until the phase has lasted settle_ms on the GPU's own clock: a first short one gives
            # the step time (its very first launch is slow), the later ones are sized from what has been seen
            s0 = ev(enable_timing=True)
            s0.record()
            burst = 4
            while True:
                for _ in range(burst):
                    step()
                s1 = ev(enable_timing=True)
                s1.record()
                s1.synchronize()
                settle_steps += burst
                settle_ms = s0.elapsed_time(s1)
                if settle_ms >= self.settle_ms:
                    break
                per_step = max(settle_ms / settle_steps, 1e-3)
                burst = max(4, int((self.settle_ms - settle_ms) / per_step) + 1)
        for _ in range(warmup):
            step()
        e0, e1 = ev(enable_timing=True), ev(enable_timing=True)
        e0.record()
        for _ in range(steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        return ms, {"steps": steps, "warmup": warmup, "settle_ms": round(settle_ms, 1), "settle_steps": settle_steps}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200, help="timed steps (of the main run and of every sub-measurement)")
    ap.add_argument("--warmup", type=int, default=20, help="untimed steps right before the timed ones")
    ap.add_argument("--settle-ms", type=float, default=200.0,
                    help="before the warm-up steps of every measurement the same step runs back to back, untimed, for "
                         "at least this many ms of GPU time: after an idle phase (the host packs layers) the shader "
                         "clock starts high, is cut back about 1.5 ms into the load and takes about 60 ms to come "
                         "back (profiles/decode_cold_start_config2_stream512.txt); reported as `settle` in the output")
    ap.add_argument("--layers", type=int, default=512,
                    help="distinct layers in the stream (config2); 512 layers = 1.07 GB of sign bits, about what "
                         "one decode step of a 7B model streams; 256 and 1024 are reported next to it")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--kind", choices=["auto", "valu", "mfma", "mfma_split"], default="auto")
    ap.add_argument("--workload", choices=["config2", "config5"], default="config2",
                    help="config2: 256 distinct 4096x4096 k=2048 layers (the headline); config5: the 224 linear "
                         "layers of a Llama-2-7B-shaped decoder at 1.5 bits/weight as the main workload")
    ap.add_argument("--no-config5", action="store_true", help="skip the extra 224-layer stack measurement")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--prefill-only", action="store_true",
                    help="only the prefill (matrix-core) measurement: what the prefill rocprofv3 summary is taken on")
    ap.add_argument("--table4", action="store_true",
                    help="only the second workload: the layer sizes of the paper's matrix-vector timing table "
                         "(Llama-3 shapes, 1 / 1.5 / 2 / 2.3 bits per weight), isolated latency and streamed rate")
    ap.add_argument("--prune", action="store_true",
                    help="only the middle-channel pruning measurement (dbf_prune_middle on two config-4 shaped layers)")
    ap.add_argument("--svid", action="store_true",
                    help="only the SVID projection measurement (dbf_svid on a 4096 x 4096 and an 11008 x 4096 matrix)")
    ap.add_argument("--admm", action="store_true",
                    help="only the ADMM update measurement (dbf_admm_step for a 4096 x 4096 weight at 1 and 2 bits)")
    ap.add_argument("--decoder-pass", action="store_true",
                    help="only the dependent token pass: the 224 linear layers of the Llama-2-7B-shaped decoder as 128 dependent "
                         "calls (q,k,v / o / gate,up / down per block), eager and as one captured graph, batch 1, 4, 16")
    ap.add_argument("--stack-sizes", action="store_true",
                    help="only the call time of stacks of 1 ... 128 layers at batch 1 ... 16 (default kind): where a call "
                         "is bound by its launches and where by the stream")
    ap.add_argument("--stream-only", action="store_true",
                    help="only the timed stream of layers (what the rocprofv3 summaries are taken on)")
    ap.add_argument("--cold-series", type=int, default=0, metavar="N",
                    help="only a time series: after the set-up (GPU idle while the layers are packed) and an extra idle "
                         "pause, N steps back to back with a HIP event between every two; prints the per-step times")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy and a 1 GiB streaming read of known size, so that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings can be scaled to bytes")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="no GPU work: read the counter_collection CSVs of two rocprofv3 --pmc runs (FETCH_SIZE, then "
                         "WRITE_SIZE) of `bench.py --stream-only --copy-calibration ...`, scale the readings by what the "
                         "same counters read for the 1 GiB copy / 1 GiB read of that run, and write profiles/traffic.json "
                         "for the workload named by the other flags")
    ap.add_argument("--no-table4", action="store_true", help="skip the 1- and 2-bit rows of the second workload")
    ap.add_argument("--knob", action="append", default=[], metavar="K=V",
                    help="set tuning knob K (number, include/dbf.h) to V before anything is packed; repeatable; for A/B runs")
    args = ap.parse_args()
    if args.traffic_from:
        print(json.dumps(traffic_from(args)))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path uses no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2505_11076_amd import binding as B
    from paper_2505_11076_amd import inputs as I

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.lib()
    for kv in args.knob:
        knob, val = kv.split("=")
        B.dbf_tuning_set(int(knob), int(val))
    kind = {"auto": B.GEMV_AUTO, "valu": B.GEMV_VALU, "mfma": B.GEMV_MFMA, "mfma_split": B.GEMV_MFMA_SPLIT}[args.kind]
    proto = Protocol(torch, args.steps, args.warmup, args.settle_ms)
    if args.prefill_only:
        st = torch.cuda.current_stream().cuda_stream
        print(json.dumps({"prefill": prefill_bench(B, I, torch, np, st, proto), "mfma_probe": mfma_probe(B, torch, st)}))
        return
    if args.prune:
        print(json.dumps({"prune_middle": prune_bench(B, I, torch, np)}))
        return
    if args.svid:
        print(json.dumps({"svid": svid_bench(B, I, torch, np, torch.cuda.current_stream().cuda_stream, proto)}))
        return
    if args.admm:
        print(json.dumps({"admm": admm_bench(B, I, torch, np, torch.cuda.current_stream().cuda_stream, proto)}))
        return
    if args.decoder_pass:
        print(json.dumps({"decoder_pass": decoder_pass_bench(B, I, torch, np, proto)}))
        return
    if args.stack_sizes:
        print(json.dumps({"stack_sizes": stack_sizes_bench(B, I, torch, np, kind, torch.cuda.current_stream().cuda_stream, proto)}))
        return
    if args.table4:
        print(json.dumps({"table4": table4_bench(B, I, torch, np, args.batch, kind,
                                                 torch.cuda.current_stream().cuda_stream, proto)}))
        return
    cfg = I.CONFIG2
    n_in, n_out, k = cfg["n_in"], cfg["n_out"], cfg["k"]
    batch = args.batch
    stream = torch.cuda.current_stream().cuda_stream
    if args.workload == "config2":
        specs = [dict(n_in=n_in, n_out=n_out, k=k)] * args.layers
        cfg_no = 2
        workload = ("llama2-7b attention projection n_in=4096 n_out=4096 k=2048 (1.0 bpw), "
                    "batch-%d decode GEMV, %d distinct layers per step" % (batch, len(specs)))
        metric = ("DBF layer decode achieved HBM GB/s on algorithmic bytes (batch %d, 4096x4096, k=2048, "
                  "stream of %d distinct layers)" % (batch, len(specs)))
    else:
        specs = I.llama2_7b_stack_shapes()
        cfg_no = 5
        workload = ("llama2-7b decoder, all %d linear layers at 1.5 bpw (4096x4096 k=3072, 4096x11008 and "
                    "11008x4096 k=4477), batch-%d decode GEMV, independent inputs per layer" % (len(specs), batch))
        metric = ("DBF layer decode achieved HBM GB/s on algorithmic bytes (batch %d, %d-layer llama2-7b stack "
                  "at 1.5 bpw)" % (batch, len(specs)))
    R = len(specs)

    # ---- the stream of distinct layers ----------------------------------------------------------
    t0 = time.time()
    layers, stack, x_all, y_all = build_stream(B, I, torch, np, specs, cfg_no, batch)
    setup_s = time.time() - t0

    def step():
        B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, stream, kind)

    if args.cold_series:
        print(json.dumps(cold_series(torch, np, step, args.cold_series, R, setup_s)))
        return

    ms_per_step, main_protocol = proto.run(step)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        src.random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)                                               # reads 1 GiB, writes 1 GiB
        B.dbf_probe_read(src.data_ptr(), src.numel(), 0, stream)     # reads 1 GiB, writes nothing
        torch.cuda.synchronize()
        del src, dst

    # per-kernel durations, HIP events around each launch on the same stream
    msB, msA = [], []
    for _ in range(max(5, min(args.steps, 30))):
        b_, a_ = B.dbf_stack_gemv_timed(stack, x_all.data_ptr(), y_all.data_ptr(), batch, stream, kind)
        msB.append(b_)
        msA.append(a_)
    msB_avg, msA_avg = float(np.mean(msB)), float(np.mean(msA))

    per_layer = [algorithmic_bytes(sp["n_in"], sp["n_out"], sp["k"], batch) for sp in specs]
    bytes_step = float(sum(p[0] for p in per_layer))
    bytes_layer, bytes_b, bytes_a = bytes_step / R, sum(p[1] for p in per_layer) / R, sum(p[2] for p in per_layer) / R
    value = bytes_step / (ms_per_step * 1e-3) / 1e9
    ncg = 1 if batch <= 8 else 2
    if args.kind in ("auto", "mfma"):
        # One launch does both stages of every layer, so a step IS one kernel: its average
        # duration is taken from the HIP events around the back-to-back timed steps (the
        # per-launch events of the timed entry point add a few microseconds of launch latency).
        if batch == 1 or args.kind != "auto":
            # (<operand column groups, column pieces, shared quantised input, single chunk, wavefronts per
            #  workgroup, fp4 sign operands>: rows of up to 14080 columns stay in LDS as one chunk at batch 1,
            #  which all benchmark shapes are)
            dom, dom_ms, dom_bytes = ("dbf_items_mfma_kernel<%d, false, 0, %s, 4, false> (B and A stages fused)"
                                      % (ncg, "true" if batch == 1 else "true|false")), ms_per_step, bytes_layer * R
        elif msB_avg >= msA_avg:  # batches of 2 and more: input quantiser + items, per stage
            dom, dom_ms, dom_bytes = "B-stage launches (dbf_quantise_inputs_kernel + dbf_items_mfma_kernel<%d, false, 1|2|3, false>)" % ncg, msB_avg, bytes_b * R
        else:
            dom, dom_ms, dom_bytes = "A-stage launches (dbf_quantise_inputs_kernel + dbf_items_mfma_kernel<%d, false, 1|2|3, false>)" % ncg, msA_avg, bytes_a * R
    elif msB_avg >= msA_avg:
        dom, dom_ms, dom_bytes = "B-stage launch", msB_avg, bytes_b * R
    else:
        dom, dom_ms, dom_bytes = "A-stage launch", msA_avg, bytes_a * R
    if args.kind == "valu":
        dom += " of dbf_stage_valu_kernel"
    elif args.kind == "mfma_split":
        dom += " of dbf_items_mfma_kernel<%d, false, 0, true|false>" % ncg
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    # HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE counter runs (profiles/traffic.json, written by
    # --traffic-from): quoted only if it was measured on this kernel, these sources and this workload.
    traffic, traffic_note = None, "no counter run recorded for this kernel / workload"
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            rec = json.load(open(tpath))
            want = {"workload": args.workload, "layers_per_step": R, "batch": batch, "kernel_variant": args.kind}
            if rec.get("source_sha16") != kernel_source_hash():
                traffic_note = "stale: the kernel sources changed after the counter run (profiles/traffic.json)"
            elif any(rec.get(k_) != v_ for k_, v_ in want.items()):
                traffic_note = "the recorded counter run is for another workload"
            elif not dom.startswith(rec.get("kernel", "?")):
                traffic_note = "the recorded counter run is for another kernel"
            else:
                traffic, traffic_note = rec.get("bytes_per_launch"), "rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a 1 GiB copy"
        except Exception as exc:
            traffic_note = "profiles/traffic.json unreadable: %r" % (exc,)

    # ---- isolated single layer, cache warm -----------------------------------------------------
    iso = None
    if not args.stream_only:
        iso = isolated_latency(B, torch, np, layers[0], x_all[: batch * specs[0]["n_in"]],
                               y_all[: batch * specs[0]["n_out"]], batch, stream, kind)

    out = {
        "metric": metric,
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32 (int8 x int8 matrix-core sums of 16-bit fixed-point inputs; fp32 scales)"
                 if args.kind != "valu" else "f32",
        "data": "synthetic",
        "config": {"workload": workload,
                   "kernel_variant": args.kind, "layers_per_step": R, "batch": batch},
        "us_per_layer_in_stream": round(ms_per_step * 1e3 / R, 4),
        "layer_products_per_s": round(R / (ms_per_step * 1e-3), 1),
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "isolated_layer_us": iso,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 2), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_note": traffic_note, "avg_launch_ms": round(dom_ms, 5),
                     "first_launch_ms": round(msB_avg, 5), "second_launch_ms": round(msA_avg, 5),
                     "algorithmic_bytes_per_launch": dom_bytes},
        "settle": dict(main_protocol, what="the same step, back to back and untimed, before the warm-up steps: after "
                       "the idle set-up the shader clock is cut back ~1.5 ms into the load and needs ~60 ms to return "
                       "(profiles/decode_cold_start_config2_stream512.txt); every sub-measurement of this line does the "
                       "same and states its own steps / warmup / settle_ms under `protocol`"),
        "setup_s": round(setup_s, 2),
    }

    # ---- practical HBM read ceiling: a plain streaming read of 1 GiB ---------------------------
    if not args.stream_only:
        ceiling = read_ceiling(B, torch, stream)
        out["hbm_read_ceiling_GBps"] = round(ceiling, 1)
        out["frac_of_read_ceiling"] = round(value / ceiling, 4)
        out["roofline"]["frac_of_read_ceiling"] = round(achieved / ceiling, 4)

    # ---- the same stream at other lengths (launch head and tail are fixed costs per step) ------
    if args.workload == "config2" and not args.stream_only:
        by_len = {str(R): {"ms_per_step": round(ms_per_step, 5), "GBps": round(value, 2), "protocol": main_protocol}}
        for R2 in (256, 1024):
            if R2 == R:
                continue
            try:
                by_len[str(R2)] = stream_length_bench(B, I, torch, np, layers, specs[0], R2, batch, kind, stream, proto)
            except Exception as exc:  # reported, never hidden
                by_len[str(R2)] = {"error": repr(exc)}
        out["by_stream_length"] = by_len
        if batch == 1:
            # the same stream at the other batch sizes of the workload (configuration 2: batch 4 and 16)
            by_batch = {"1": {"ms_per_step": round(ms_per_step, 5), "GBps": round(value, 2), "protocol": main_protocol}}
            for b2 in (2, 4, 8, 16):
                try:
                    by_batch[str(b2)] = stream_length_bench(B, I, torch, np, layers, specs[0], R, b2, kind, stream, proto)
                except Exception as exc:  # reported, never hidden
                    by_batch[str(b2)] = {"error": repr(exc)}
            out["by_batch"] = by_batch

    stack.close()
    for l in layers:
        l.close()
    del x_all, y_all

    # ---- the 224-layer decoder stack (second decode workload) -----------------------------------
    if args.workload == "config2" and not args.no_config5 and not args.stream_only:
        try:
            out["config5_stack"] = config5_bench(B, I, torch, np, batch, kind, stream, proto)
        except Exception as exc:  # reported, never hidden
            out["config5_stack"] = {"error": repr(exc)}

    # ---- the same 224 layers as a decoder has to call them: 128 dependent calls per token pass -------------------
    if args.workload == "config2" and not args.no_config5 and not args.stream_only and batch == 1:
        try:
            out["decoder_pass_dependent_calls"] = decoder_pass_bench(B, I, torch, np, proto)
        except Exception as exc:
            out["decoder_pass_dependent_calls"] = {"error": repr(exc)}

    # ---- the MLP shapes of configuration 3 (gate / up and down projection at ~1 and ~2 bits per weight) ----------
    if args.workload == "config2" and not args.no_table4 and not args.stream_only:
        try:
            cfgs = [dict(c, bits=round(c["k"] * (c["n_in"] + c["n_out"]) / (c["n_in"] * c["n_out"]), 2)) for c in I.CONFIG3]
            out["config3_mlp"] = table4_bench(B, I, torch, np, batch, kind, stream, proto, cfgs=cfgs)
        except Exception as exc:  # reported, never hidden
            out["config3_mlp"] = {"error": repr(exc)}

    # ---- second workload: the layer sizes of the paper's matrix-vector timing table, 1 and 2 bits per weight --
    if args.workload == "config2" and not args.no_table4 and not args.stream_only:
        try:
            out["table4"] = table4_bench(B, I, torch, np, batch, kind, stream, proto, bits_only=(1.0, 2.0))
        except Exception as exc:  # reported, never hidden
            out["table4"] = {"error": repr(exc)}

    # ---- prefill (matrix-core path) ---------------------------------------------------------------
    if not args.no_prefill and not args.stream_only:
        try:
            out["prefill"] = prefill_bench(B, I, torch, np, stream, proto)
            out["mfma_probe"] = mfma_probe(B, torch, stream)
        except Exception as exc:  # reported, never hidden
            out["prefill"] = {"error": repr(exc)}

    # ---- the CPU oracle on this machine's cores (a baseline, not the target) ---------------------
    if not args.no_cpu_baseline and not args.stream_only:
        sp0 = specs[0]
        out["cpu_baseline"] = cpu_baseline(I, np, sp0["n_in"], sp0["n_out"], sp0["k"], batch,
                                           per_layer[0][0], cfg_no, R)

    print(json.dumps(out))


def traffic_from(args):
    """HBM bytes per launch of the decode kernel from two counter runs (see --traffic-from).  The counters count in
    units that differ between machines, so each is scaled by its reading for a transfer of known size in the
    same run: FETCH_SIZE by the 1 GiB streaming read of dbf_probe_read_kernel, WRITE_SIZE by the 1 GiB device copy
    (the dispatch with the largest reading that is not one of this library's kernels)."""
    import csv

    def per_dispatch(path, counter):
        acc = {}
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != counter:
                continue
            key = (int(r["Dispatch_Id"]), r["Kernel_Name"])
            acc[key] = acc.get(key, 0.0) + float(r["Counter_Value"])
        return acc

    gib = float(1 << 30)
    fetch = per_dispatch(args.traffic_from[0], "FETCH_SIZE")
    write = per_dispatch(args.traffic_from[1], "WRITE_SIZE")
    probe = [v for (d, n), v in fetch.items() if "dbf_probe_read_kernel" in n]
    copy_w = max(v for (d, n), v in write.items() if "dbf_" not in n)
    if not probe or copy_w <= 0:
        raise SystemExit("the counter runs hold no calibration dispatches (run bench.py with --copy-calibration)")
    fetch_unit, write_unit = gib / (sum(probe) / len(probe)), gib / copy_w
    kf = sorted((d, n, v) for (d, n), v in fetch.items() if "dbf_items_mfma_kernel" in n)
    kw = sorted((d, n, v) for (d, n), v in write.items() if "dbf_items_mfma_kernel" in n)
    if not kf or not kw:
        raise SystemExit("no decode kernel dispatches in the counter runs")
    import re
    name = re.search(r"dbf_items_mfma_kernel<[^>]*>", kf[0][1]).group(0)
    fb = sum(v for _, _, v in kf) / len(kf) * fetch_unit
    wb = sum(v for _, _, v in kw) / len(kw) * write_unit
    rec = {"kernel": name, "workload": args.workload, "layers_per_step": args.layers if args.workload == "config2" else 224,
           "batch": args.batch, "kernel_variant": args.kind, "source_sha16": kernel_source_hash(),
           "bytes_per_launch": int(round(fb + wb)), "fetch_bytes": int(round(fb)), "write_bytes": int(round(wb)),
           "fetch_size_count_bytes": fetch_unit, "write_size_count_bytes": write_unit,
           "dispatches_averaged": [len(kf), len(kw)],
           "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on bench.py --stream-only --copy-calibration "
                     "(commands in profiles/decode_fused_kernel_config2_stream512.txt)"}
    with open(os.path.join(ROOT, "profiles", "traffic.json"), "w") as fh:
        json.dump(rec, fh, indent=1)
        fh.write("\n")
    return rec


def cold_series(torch, np, step, n, layers_per_step, setup_s):
    """Per-step times of the first n steps after the GPU has been idle (the set-up packs layers on the host;
    one more second of sleep on top), from HIP events recorded between the steps on the launch stream."""
    torch.cuda.synchronize()
    time.sleep(1.0)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(n):
        step()
        ev[i + 1].record()
    t_issue = time.perf_counter() - t0
    torch.cuda.synchronize()
    t_all = time.perf_counter() - t0
    us = np.array([ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(n)])
    cum_ms = np.cumsum(us) / 1e3

    def mean(a, b):
        return round(float(us[a:b].mean()), 2) if b <= n and b > a else None

    windows = {}
    for a, b in ((0, 1), (1, 5), (5, 25), (25, 50), (50, 100), (100, 200), (200, 300), (300, 500), (500, 1000),
                 (1000, 2000)):
        if b <= n:
            windows["%d-%d" % (a, b)] = {"mean_us": mean(a, b), "min_us": round(float(us[a:b].min()), 2),
                                         "max_us": round(float(us[a:b].max()), 2),
                                         "ends_at_ms": round(float(cum_ms[b - 1]), 2)}
    return {"cold_series": {"layers_per_step": layers_per_step, "steps": n, "setup_s": round(setup_s, 2),
                            "idle_before_s": 1.0, "host_issue_s": round(t_issue, 4), "host_total_s": round(t_all, 4),
                            "windows": windows, "first_40_us": [round(float(v), 1) for v in us[:40]],
                            "every_25th_us": [round(float(v), 1) for v in us[::25]]}}


def build_stream(B, I, torch, np, specs, cfg_no, batch):
    """Packs one distinct random layer per spec, builds the stack and its input / output blocks
    (x and y of the layers back to back, independent N(0,1) inputs per layer)."""
    layers = []
    for i, sp in enumerate(specs):
        L = I.make_layer(sp["n_in"], sp["n_out"], sp["k"], seed=I.seed_for(cfg_no, i))
        layers.append(B.dbf_pack_bits(sp["n_in"], sp["n_out"], sp["k"], L.A_bits, L.B_bits, L.a, L.m, L.b))
    stack = B.dbf_stack_create(layers)
    rng = np.random.default_rng(I.seed_for(cfg_no, 999))
    n_x = sum(batch * sp["n_in"] for sp in specs)
    n_y = sum(batch * sp["n_out"] for sp in specs)
    x_host = I.random_activations_fp16(rng, 1, n_x)
    x_all = torch.from_numpy(x_host.view(np.int16).copy()).cuda().view(torch.float16).reshape(-1)
    y_all = torch.zeros(n_y, dtype=torch.float16, device="cuda")
    torch.cuda.synchronize()
    return layers, stack, x_all, y_all


def stream_length_bench(B, I, torch, np, layers, spec, R2, batch, kind, stream, proto):
    """The config-2 stream with R2 distinct layers: reuses the packed layers of the main run (and
    packs more if R2 is larger); returns the step time and the achieved rate, timed like the main run."""
    extra = []
    for i in range(len(layers), R2):
        L = I.make_layer(spec["n_in"], spec["n_out"], spec["k"], seed=I.seed_for(2, i))
        extra.append(B.dbf_pack_bits(spec["n_in"], spec["n_out"], spec["k"], L.A_bits, L.B_bits, L.a, L.m, L.b))
    use = (list(layers) + extra)[:R2]
    stack = B.dbf_stack_create(use)
    try:
        rng = np.random.default_rng(I.seed_for(2, 998))
        x_host = I.random_activations_fp16(rng, 1, R2 * batch * spec["n_in"])
        x = torch.from_numpy(x_host.view(np.int16).copy()).cuda().view(torch.float16).reshape(-1)
        y = torch.zeros(R2 * batch * spec["n_out"], dtype=torch.float16, device="cuda")
        ms, protocol = proto.run(lambda: B.dbf_stack_gemv(stack, x.data_ptr(), y.data_ptr(), batch, stream, kind))
        nbytes = algorithmic_bytes(spec["n_in"], spec["n_out"], spec["k"], batch)[0] * R2
        return {"ms_per_step": round(ms, 5), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 2), "protocol": protocol}
    finally:
        stack.close()
        for l in extra:
            l.close()


def config5_bench(B, I, torch, np, batch, kind, stream, proto):
    """One decode pass over all 224 linear layers of the Llama-2-7B-shaped stack (1.21 GB of signs)."""
    specs = I.llama2_7b_stack_shapes()
    layers, stack, x_all, y_all = build_stream(B, I, torch, np, specs, 5, batch)
    try:
        ms, protocol = proto.run(lambda: B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, stream, kind))
        nbytes = float(sum(algorithmic_bytes(sp["n_in"], sp["n_out"], sp["k"], batch)[0] for sp in specs))
        gbps = nbytes / (ms * 1e-3) / 1e9
        res = {"layers": len(specs), "batch": batch, "ms_per_token_pass": round(ms, 5),
               "token_passes_per_s": round(1e3 / ms, 1), "GBps": round(gbps, 2),
               "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4), "algorithmic_bytes": nbytes, "protocol": protocol,
               "note": "all linear layers of a 32-block decoder at 1.5 bits/weight, one stack call per pass, "
                       "independent inputs per layer (no attention / norms between them)"}
        if batch == 1:  # the workload's other batch size: 16 tokens per pass through the same stack
            b2 = 16
            del x_all, y_all
            rng = np.random.default_rng(I.seed_for(5, 997))
            x_host = I.random_activations_fp16(rng, 1, sum(b2 * sp["n_in"] for sp in specs))
            x2 = torch.from_numpy(x_host.view(np.int16).copy()).cuda().view(torch.float16).reshape(-1)
            y2 = torch.zeros(sum(b2 * sp["n_out"] for sp in specs), dtype=torch.float16, device="cuda")
            ms2, protocol2 = proto.run(lambda: B.dbf_stack_gemv(stack, x2.data_ptr(), y2.data_ptr(), b2, stream, kind))
            nb2 = float(sum(algorithmic_bytes(sp["n_in"], sp["n_out"], sp["k"], b2)[0] for sp in specs))
            res["batch16"] = {"ms_per_pass": round(ms2, 5), "tokens_per_s": round(b2 * 1e3 / ms2, 1),
                              "GBps": round(nb2 / (ms2 * 1e-3) / 1e9, 2), "protocol": protocol2}
        return res
    finally:
        stack.close()
        for l in layers:
            l.close()


# The paper's Table 4 (RTX 4090, fp16 activations, batch 1), microseconds per matrix-vector product, by
# (n_out, n_in) and bits per weight; printed next to this machine's numbers as context only.
PAPER_TABLE4_US = {
    (4096, 4096): {2.3: 29, 2.0: 27, 1.5: 24, 1.0: 20},
    (4096, 14336): {2.3: 56, 2.0: 51, 1.5: 43, 1.0: 37},
    (8192, 8192): {2.3: 64, 2.0: 58, 1.5: 51, 1.0: 38},
    (8192, 28672): {2.3: 167, 2.0: 149, 1.5: 115, 1.0: 84},
}


def table4_bench(B, I, torch, np, batch, kind, stream, proto, bits_only=None, cfgs=None):
    """Every (shape, bits per weight) of the second workload (or the shapes in `cfgs`): the isolated call (cache
    warm) and a stream of distinct copies of the layer (at least 512 MB of signs, at most 256 copies) in one
    stack call per step."""
    rows = []
    for ci, cfg in enumerate(I.table4_configs() if cfgs is None else cfgs):
        if bits_only is not None and cfg["bits"] not in bits_only:
            continue
        n_in, n_out, k = cfg["n_in"], cfg["n_out"], cfg["k"]
        nbytes = algorithmic_bytes(n_in, n_out, k, batch)[0]
        R = int(min(256, max(2, -(-(512 << 20) // nbytes))))
        specs = [dict(n_in=n_in, n_out=n_out, k=k)] * R
        layers, stack, x_all, y_all = build_stream(B, I, torch, np, specs, 6, batch)
        try:
            xs = x_all[: batch * n_in]
            ys = y_all[: batch * n_out]
            iso = isolated_latency(B, torch, np, layers[0], xs, ys, batch, stream, kind)
            ms, protocol = proto.run(lambda: B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, stream, kind))
            gbps = nbytes * R / (ms * 1e-3) / 1e9
            rows.append({"n_out": n_out, "n_in": n_in, "bits": cfg["bits"], "k": k,
                         "isolated_us_p50": iso["p50"], "back_to_back_us": iso["back_to_back_us"],
                         "stream_layers": R, "stream_us_per_layer": round(ms * 1e3 / R, 3),
                         "stream_GBps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
                         "protocol": protocol, "paper_rtx4090_us": PAPER_TABLE4_US.get((n_out, n_in), {}).get(cfg["bits"])})
        finally:
            stack.close()
            for l in layers:
                l.close()
            del x_all, y_all
    return {"batch": batch, "rows": rows,
            "note": "isolated = one dbf_gemv call, cache warm (p50 of 200 event pairs); stream = distinct copies of "
                    "the layer in one dbf_stack_gemv call per step, signs read from HBM; paper column: its Table 4 "
                    "on an RTX 4090, another machine, context only"}


def decoder_pass_bench(B, I, torch, np, proto, n_blocks=32):
    """The linear layers of a Llama-2-7B-shaped decoder at 1.5 bits per weight run the way a decoder has to run them:
    per block four DEPENDENT calls -- the group q, k, v on one input, o on (a stand-in for) the attention output, the
    group gate, up on o's output, down on gate's output, whose result is the next block's input -- i.e. 128 calls and
    (at batch 1) 256 launches per token pass, against ONE launch when the 224 layers are independent (config 5).
    Timed eagerly and as one captured HIP graph; attention, norms and activations are left out (stand-ins read what
    the previous call wrote, so every call waits for its predecessor)."""
    shapes = dict(sq=dict(n_in=4096, n_out=4096, k=3072), up=dict(n_in=4096, n_out=11008, k=4477),
                  down=dict(n_in=11008, n_out=4096, k=4477))
    layers, blocks = [], []
    for b in range(n_blocks):
        def mk(name, idx):
            sp = shapes[name]
            L = I.make_layer(sp["n_in"], sp["n_out"], sp["k"], seed=I.seed_for(5, 2000 + 8 * b + idx))
            layer = B.dbf_pack_bits(sp["n_in"], sp["n_out"], sp["k"], L.A_bits, L.B_bits, L.a, L.m, L.b)
            layers.append(layer)
            return layer
        q, k_, v, o = mk("sq", 0), mk("sq", 1), mk("sq", 2), mk("sq", 3)
        g, u, d = mk("up", 4), mk("up", 5), mk("down", 6)
        blocks.append((B.dbf_stack_create_grouped([q, k_, v], [3]), B.dbf_stack_create([o]),
                       B.dbf_stack_create_grouped([g, u], [2]), B.dbf_stack_create([d])))
    nbytes1 = float(n_blocks * (4 * algorithmic_bytes(4096, 4096, 3072, 1)[0] + 2 * algorithmic_bytes(4096, 11008, 4477, 1)[0]
                                + algorithmic_bytes(11008, 4096, 4477, 1)[0]))
    res = {"blocks": n_blocks, "calls_per_pass": 4 * n_blocks}
    try:
        for batch in (1, 4, 16):
            h = [torch.randn(batch * 4096, device="cuda").half() for _ in range(2)]
            yqkv = torch.zeros(3 * batch * 4096, dtype=torch.float16, device="cuda")
            yo = torch.zeros(batch * 4096, dtype=torch.float16, device="cuda")
            ygu = torch.zeros(2 * batch * 11008, dtype=torch.float16, device="cuda")

            def token_pass(stream):
                for i, (s1, s2, s3, s4) in enumerate(blocks):
                    B.dbf_stack_gemv(s1, h[i & 1].data_ptr(), yqkv.data_ptr(), batch, stream)
                    B.dbf_stack_gemv(s2, yqkv.data_ptr(), yo.data_ptr(), batch, stream)
                    B.dbf_stack_gemv(s3, yo.data_ptr(), ygu.data_ptr(), batch, stream)
                    B.dbf_stack_gemv(s4, ygu.data_ptr(), h[(i + 1) & 1].data_ptr(), batch, stream)

            cur = torch.cuda.current_stream().cuda_stream
            ms_eager, protocol = proto.run(lambda: token_pass(cur))
            graph = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                graph.capture_begin()
                token_pass(side.cuda_stream)
                graph.capture_end()
            torch.cuda.current_stream().wait_stream(side)
            ms_graph, _ = proto.run(graph.replay)
            del graph
            res["batch%d" % batch] = {"eager_us_per_pass": round(ms_eager * 1e3, 1), "graph_us_per_pass": round(ms_graph * 1e3, 1),
                                      "graph_us_per_call": round(ms_graph * 1e3 / (4 * n_blocks), 2),
                                      "tokens_per_s_graph": round(batch * 1e3 / ms_graph, 1), "protocol": protocol}
        res["sign_and_vector_bytes_per_pass"] = nbytes1
        res["note"] = ("dependent calls: each reads what the previous one wrote; the independent 224-layer stack of config 5 "
                       "streams the same bytes in one launch (config5_stack)")
        return res
    finally:
        for st in blocks:
            for s_ in st:
                s_.close()
        for l in layers:
            l.close()


def stack_sizes_bench(B, I, torch, np, kind, stream, proto):
    """One dbf_stack_gemv per step on stacks of 1 ... 128 copies of a layer (independent inputs), batch 1 ... 16:
    microseconds per call, back to back.  Short stacks are bound by their launches (two at batch 1, four above),
    long ones by the stream."""
    res = {}
    for n_in, n_out, k in ((4096, 4096, 2048), (4096, 11008, 2985), (11008, 4096, 2985)):
        base = [I.make_layer(n_in, n_out, k, seed=I.seed_for(6, i)) for i in range(4)]
        rows = {}
        for R in (1, 3, 8, 24, 64, 128):
            layers = [B.dbf_pack_bits(n_in, n_out, k, base[i % 4].A_bits, base[i % 4].B_bits, base[i % 4].a, base[i % 4].m,
                                      base[i % 4].b) for i in range(R)]
            stack = B.dbf_stack_create(layers)
            row = {}
            for batch in (1, 2, 4, 8, 16):
                x = torch.randn(R * batch * n_in, device="cuda").half()
                y = torch.zeros(R * batch * n_out, dtype=torch.float16, device="cuda")
                ms, _ = proto.run(lambda: B.dbf_stack_gemv(stack, x.data_ptr(), y.data_ptr(), batch, stream, kind))
                row["batch%d" % batch] = round(ms * 1e3, 1)
            rows["layers%d" % R] = row
            stack.close()
            for l in layers:
                l.close()
        res["%dx%d_k%d" % (n_in, n_out, k)] = rows
    return {"us_per_call": res, "protocol": {"steps": proto.steps, "warmup": proto.warmup, "settle_ms": proto.settle_ms}}


def prune_bench(B, I, torch, np):
    """dbf_prune_middle from 2 to 1.5 bits per weight on the two prefill-shaped layers: the whole call
    (allocation of the new layer, three gather kernels, its launch plan; synchronous) and the sign
    bytes it has to move (kept signs read once, new signs written once)."""
    res = {}
    for cfg in I.CONFIG4:
        n_in, n_out, k = cfg["n_in"], cfg["n_out"], cfg["k"]
        k2 = I.CONFIG4_PRUNED_K[(n_out, n_in)]
        L = I.make_layer(n_in, n_out, k, seed=I.seed_for(4, n_in))
        layer = B.dbf_pack_bits(n_in, n_out, k, L.A_bits, L.B_bits, L.a, L.m, L.b)
        keep = np.sort(np.random.default_rng(I.seed_for(4, 77)).choice(k, size=k2, replace=False)).astype(np.int32)
        times = []
        for _ in range(7):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            pruned = B.dbf_prune_middle(layer, keep)
            times.append(time.perf_counter() - t0)
            pruned.close()
        layer.close()
        moved = 2.0 * k2 * (n_in + n_out) / 8.0
        ms = float(np.median(times)) * 1e3
        res["%dx%d_k%d_to_%d" % (n_in, n_out, k, k2)] = {
            "ms_per_call": round(ms, 3), "sign_bytes_moved": moved, "GBps_whole_call": round(moved / (ms * 1e-3) / 1e9, 1),
            "note": "whole synchronous call incl. device allocation and plan upload; kernel times: profiles/prune_middle.txt"}
    return res


def svid_bench(B, I, torch, np, stream, proto, iters=8):
    """dbf_svid (signs + `iters` rounds of power iteration) on two factor-sized fp32 matrices.  Bytes:
    Z is read once for the signs and twice per round (row dots, column dots); the packed signs and
    the vectors are negligible next to it."""
    res = {}
    for rows, cols in ((4096, 4096), (11008, 4096)):
        Z = I.make_svid_matrix(rows, cols, I.seed_for(8, rows))
        z = torch.from_numpy(Z).cuda()
        a = torch.zeros(rows, dtype=torch.float32, device="cuda")
        m = torch.zeros(cols, dtype=torch.float32, device="cuda")
        bits = torch.zeros(B.dbf_tiled_bytes(rows, cols), dtype=torch.uint8, device="cuda")
        wsb = B.dbf_svid_workspace_bytes(rows, cols)
        ws = torch.zeros(wsb, dtype=torch.uint8, device="cuda")
        args = (z.data_ptr(), rows, cols, iters, a.data_ptr(), m.data_ptr(), bits.data_ptr(), ws.data_ptr(), wsb, stream)
        ms, protocol = proto.run(lambda: B.dbf_svid(*args))
        nbytes = (2.0 * iters + 1.0) * rows * cols * 4.0
        t0 = time.time()
        from oracle import dbf_oracle as O
        O.svid(Z.astype(np.float64), iters)
        cpu_s = time.time() - t0
        # (the library makes both products of a round in ONE pass over Z for matrices of 24 Mi entries and more with rows of
        #  at most 24576 values; the algorithmic bytes above keep the two-pass count, so the rate on them can pass the peak)
        one_pass = rows * cols >= (24 << 20) and cols <= 24576 and cols % 4 == 0
        passes = (iters + 1) if one_pass else (2 * iters + 1)
        res["%dx%d_iters%d" % (rows, cols, iters)] = {
            "ms_per_call": round(ms, 4), "algorithmic_bytes": nbytes, "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "passes_over_Z_made": passes,
            "GBps_on_passes_made": round(passes * rows * cols * 4.0 / (ms * 1e-3) / 1e9, 1),
            "cpu_oracle_s": round(cpu_s, 3), "protocol": protocol}
    return res


def admm_bench(B, I, torch, np, stream, proto, svid_iters=2, rho=1.0):
    """The ADMM update for the factor of a 4096 x 4096 weight with q = 2048 and q = 4096 middle channels (1 and 2
    bits per weight), starting from the PACKED fixed factor: dbf_admm_prepare forms C = B^T W and
    Minv = (B^T B + rho I)^-1 on the device (once per outer iteration; timed on its own), dbf_admm_step is the
    repeated part.  In the step the q x q x r fp32 contraction dominates (2 q^2 r flops, priced against the fp32
    matrix-core peak); around it the step reads or writes a q x r fp32 matrix 7 + 2 * svid_iters times.  The
    preparation is 2 p q^2 (B^T B) + 2 p q r (B^T W) + q^3 / 3 (Cholesky) + q^3 / 3 (inverse of the factor) +
    2 q^3 (its Gram matrix) flops."""
    from oracle import dbf_oracle as O
    res = {}
    for p, q, r in ((4096, 2048, 4096), (4096, 4096, 4096)):
        S_B, m2, b, W, S, a, m, U = I.make_admm_packed_problem(p, q, r, I.seed_for(9, q))
        dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
        d = {"bitsB": dev(B.dbf_tile_host(q, p, B.dbf_signs_to_bits_host(S_B))), "m2": dev(m2), "b": dev(b), "W": dev(W),
             "Minv": torch.zeros((q, q), dtype=torch.float32, device="cuda"),
             "C": torch.zeros((q, r), dtype=torch.float32, device="cuda"),
             "a": dev(a), "m": dev(m), "U": dev(U), "bits": dev(B.dbf_tile_host(q, r, B.dbf_signs_to_bits_host(S))),
             "flag": torch.zeros(1, dtype=torch.int32, device="cuda")}
        pwsb = B.dbf_admm_prepare_workspace_bytes(p, q, r)
        pws = torch.zeros(pwsb, dtype=torch.uint8, device="cuda")
        pargs = (d["bitsB"].data_ptr(), d["m2"].data_ptr(), d["b"].data_ptr(), d["W"].data_ptr(), p, q, r, rho,
                 d["Minv"].data_ptr(), d["C"].data_ptr(), pws.data_ptr(), pwsb, d["flag"].data_ptr(), stream)
        ms_prep, protocol_prep = proto.run(lambda: B.dbf_admm_prepare(*pargs))
        assert int(d["flag"].item()) == 0
        wsb = B.dbf_admm_workspace_bytes(q, r)
        ws = torch.zeros(wsb, dtype=torch.uint8, device="cuda")
        args = (d["Minv"].data_ptr(), d["C"].data_ptr(), q, r, rho, svid_iters, d["a"].data_ptr(), d["m"].data_ptr(),
                d["bits"].data_ptr(), d["U"].data_ptr(), ws.data_ptr(), wsb, stream)
        # (every call is the next ADMM iteration on the updated iterate)
        ms, protocol = proto.run(lambda: B.dbf_admm_step(*args))
        flops = 2.0 * q * q * r
        prep_flops = 2.0 * p * q * q + 2.0 * p * q * r + 2.0 * q ** 3 / 3.0 + 2.0 * q ** 3
        nbytes = (7.0 + 2.0 * svid_iters) * q * r * 4.0 + 4.0 * q * q
        t0 = time.time()
        Minv64, C64 = O.admm_constants(O.fixed_factor_dense(S_B, b, m2), W, rho)
        cpu_prep_s = time.time() - t0
        t0 = time.time()
        O.admm_step_from(Minv64, C64, rho, S.astype(np.float64), a.astype(np.float64), m.astype(np.float64),
                         U.astype(np.float64), svid_iters)
        cpu_s = time.time() - t0
        res["q%d_r%d_svid%d" % (q, r, svid_iters)] = {
            "ms_per_step": round(ms, 4), "contraction_flops": flops,
            "tflops_whole_step": round(flops / (ms * 1e-3) / 1e12, 2),
            "frac_of_f32_mfma_peak_whole_step": round(flops / (ms * 1e-3) / 1e12 / MFMA_F32_PEAK_TFLOPS, 4),
            "elementwise_bytes": nbytes, "cpu_oracle_s": round(cpu_s, 3), "protocol": protocol,
            "prepare": {"ms": round(ms_prep, 4), "flops": prep_flops,
                        "tflops": round(prep_flops / (ms_prep * 1e-3) / 1e12, 2),
                        "frac_of_f32_mfma_peak": round(prep_flops / (ms_prep * 1e-3) / 1e12 / MFMA_F32_PEAK_TFLOPS, 4),
                        "cpu_oracle_s": round(cpu_prep_s, 3), "protocol": protocol_prep}}
    return res


def isolated_latency(B, torch, np, layer, xs, ys, batch, stream, kind):
    """One layer launched alone, cache warm: per-call latency (two dependent launches) and the
    back-to-back rate of the same call."""
    lat = []
    for _ in range(20):
        B.dbf_gemv(layer, xs.data_ptr(), ys.data_ptr(), batch, stream, kind)
    torch.cuda.synchronize()
    for _ in range(200):
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record()
        B.dbf_gemv(layer, xs.data_ptr(), ys.data_ptr(), batch, stream, kind)
        a1.record()
        a1.synchronize()
        lat.append(a0.elapsed_time(a1) * 1e3)
    lat = np.sort(np.array(lat))
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a0.record()
    for _ in range(500):
        B.dbf_gemv(layer, xs.data_ptr(), ys.data_ptr(), batch, stream, kind)
    a1.record()
    torch.cuda.synchronize()
    return {"p10": round(float(lat[20]), 2), "p50": round(float(lat[100]), 2), "p90": round(float(lat[180]), 2),
            "back_to_back_us": round(a0.elapsed_time(a1) * 1e3 / 500, 3),
            "note": "one layer, cache warm, launch bound"}


def read_ceiling(B, torch, stream):
    probe = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    probe.random_(0, 255)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    for _ in range(2):
        B.dbf_probe_read(probe.data_ptr(), probe.numel(), sink.data_ptr(), stream)
    torch.cuda.synchronize()
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    p0.record()
    for _ in range(5):
        B.dbf_probe_read(probe.data_ptr(), probe.numel(), sink.data_ptr(), stream)
    p1.record()
    torch.cuda.synchronize()
    return probe.numel() * 5 / (p0.elapsed_time(p1) * 1e-3) / 1e9


def prefill_bench(B, I, torch, np, stream, proto):
    """Both config-4 shapes at T = 2048.  TFLOP/s counts the factored work 2*T*k*(n_in+n_out) and is priced
    against the dense fp16 matrix-core peak (the kernel issues twice the multiply-adds, two int8 planes, at
    twice the fp16 rate: the same fraction against the int8 peak)."""
    res = {}
    for cfg in I.CONFIG4:
        n_in, n_out, k, T = cfg["n_in"], cfg["n_out"], cfg["k"], cfg["T"]
        L = I.make_layer(n_in, n_out, k, seed=I.seed_for(4, n_in))
        layer = B.dbf_pack_bits(n_in, n_out, k, L.A_bits, L.B_bits, L.a, L.m, L.b)
        ws_bytes = B.dbf_gemm_workspace_bytes(layer, T)
        if ws_bytes == 0:
            layer.close()
            raise RuntimeError("dbf_gemm not available")
        X = I.make_activations(T, n_in, I.seed_for(4, n_in))
        x = torch.from_numpy(X.view(np.int16).copy()).cuda().view(torch.float16)
        y = torch.zeros((T, n_out), dtype=torch.float16, device="cuda")
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        flops = 2.0 * T * k * (n_in + n_out)
        ms, protocol = proto.run(lambda: B.dbf_gemm(layer, x.data_ptr(), y.data_ptr(), T, ws.data_ptr(), ws_bytes, stream))
        tf = flops / (ms * 1e-3) / 1e12
        res["%dx%d_k%d_T%d" % (n_in, n_out, k, T)] = {
            "ms": round(ms, 4), "tflops": round(tf, 2), "frac_of_f16_mfma_peak": round(tf / MFMA_F16_PEAK_TFLOPS, 4),
            "variant": "int8 matrix cores, 16-bit fixed-point activations", "protocol": protocol}
        # few tokens (latency bound): up to 32 run as decode batches, up to 512 with the columns of a stage cut into shares
        few = {}
        for Tf in (16, 32, 64, 256):
            ms_f, _ = proto.run(lambda: B.dbf_gemm(layer, x.data_ptr(), y.data_ptr(), Tf, ws.data_ptr(), ws_bytes, stream))
            few["T%d" % Tf] = round(ms_f * 1e3, 1)
        res["%dx%d_k%d_T%d" % (n_in, n_out, k, T)]["us_per_call_few_tokens"] = few
        layer.close()
    return res


def mfma_probe(B, torch, stream):
    """What the int8 matrix pipe sustains (fraction of the 5.0 POP/s data-sheet peak) at two wavefronts
    per SIMD, for the prefill kernel's instruction (16x16x64) and the 8-pass one (32x32x32), bare and
    with the ANDs that make the sign operand: the ceiling the prefill stage kernel is compared with."""
    res = {"unit": "fraction of %.0f TOP/s" % MFMA_I8_PEAK_TOPS, "wavefronts_per_simd": 2}
    iters = 2000
    for name, wide, ands in (("i8_16x16x64", False, False), ("i8_16x16x64_sign_ands", False, True),
                             ("i8_32x32x32", True, False), ("i8_32x32x32_sign_ands", True, True)):
        B.dbf_probe_mfma(wide, ands, 2, iters, 0, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ops = B.dbf_probe_mfma(wide, ands, 2, iters, 0, stream)
        e1.record()
        torch.cuda.synchronize()
        res[name] = round(ops / (e0.elapsed_time(e1) * 1e-3) / 1e12 / MFMA_I8_PEAK_TOPS, 4)
    return res


def cpu_baseline(I, np, n_in, n_out, k, batch, bytes_layer, cfg_no=2, n_layers=256):
    """Times the oracle as it stands on a bounded sample: one layer of the stream, dense mode
    (decode signs, form W' in fp64, multiply), repeated a few times."""
    from oracle import dbf_oracle as O
    threads = os.cpu_count() or 1
    try:
        from threadpoolctl import threadpool_info
        for info in threadpool_info():
            if info.get("user_api") == "blas":
                threads = int(info.get("num_threads", threads))
    except Exception:
        pass
    L = I.make_layer(n_in, n_out, k, seed=I.seed_for(cfg_no, 0))
    X = I.make_activations(batch, n_in, I.seed_for(cfg_no, 0))
    # about 12 s of oracle work: the dense mode (the headline sample), then the staged mode beside it
    times = []
    t_end = time.time() + 8.0
    while len(times) < 3 or (time.time() < t_end and len(times) < 24):
        t0 = time.time()
        O.forward_from_packed(X, L, "dense")
        times.append(time.time() - t0)
        if time.time() > t_end + 40:
            break
    sec = float(np.median(times))
    staged = []
    t_end = time.time() + 4.0
    while len(staged) < 2 or (time.time() < t_end and len(staged) < 12):
        t0 = time.time()
        O.forward_from_packed(X, L, "staged")
        staged.append(time.time() - t0)
        if time.time() > t_end + 40:
            break
    return {"value": round(bytes_layer / sec / 1e9, 6), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": "1 of the %d-layer stream: one %dx%d k=%d layer, batch %d, dense fp64 oracle "
                      "(decode signs, form W', multiply), median of %d runs" % (n_layers, n_in, n_out, k, batch,
                                                                               len(times)),
            "seconds_per_layer": round(sec, 4), "layer_products_per_s": round(1.0 / sec, 4),
            "staged_seconds_per_layer": round(float(np.median(staged)), 4),
            "staged_note": "the same layer through the oracle's staged mode (decode signs, the forward-pass "
                           "expression left to right in fp64), median of %d runs" % len(staged)}


if __name__ == "__main__":
    main()
