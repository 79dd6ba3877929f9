#!/usr/bin/env python3
"""Benchmark of the NQKV hot path on one MI355X.

One "step" is one pass of the whole hot path over the largest single-GPU workload, the
OPT-30B-shaped layer C5 (batch 16, 56 heads, head_dim 128, 16384 cached tokens, 4-bit codes,
block 64, Student-t keys): quantize the whole prefill cache (K and V in one launch), then one
decode step in one launch (quantize and append the new token's key and value, fused
dequantize + attention over all 16385 tokens).  Inputs are synthetic (seeded, recipe of
paper_2505_16210_amd/workloads.py) and resident in HBM before the timed region.

Prints ONE JSON line.
  value      effective fp16 KV GB/s of the step: 2 bytes x (K and V elements quantized + K and V
             elements attended over) per second
  roofline   the dominant kernel of that step (the quantizer: about four fifths of the step time),
             timed live with events between the launches of the timed region, and beside it
             (`decode_step`) the fused decode kernel of the same step, live and in steady state;
             `configs` lists quantize / decode attention / fused decode step for C2, C3, C4 and the
             six C5 variants (k in {2,3,4} x block in {64,128}), each timed through HIP-graph replays
             (no host launch gaps) over rotating cache copies (no reads served from the last-level
             cache); `traffic` is measured in this run by two rocprofv3 counter passes over a child
             process (null when the profiler is not usable)
  kernels    further per-kernel figures (dequantize, the paper's own decode flow, length mixes,
             paged cache, several queries per step, the C2 decode loop and its launch floor)
  cpu_baseline  the CPU oracle timed on this machine's host cores on half of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import shutil
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
# The step's cache is allocated with room for this many tokens after the prompt (one page of the
# paged layout).  The capacity sets the distance between the (batch, head) slabs of the cache, and
# both kernels are sensitive to it: with room for 16 to 4096 tokens the step takes 1.89-1.91 ms, with
# 128 (slabs 1 MiB + 8 KiB apart, which piles them onto few memory channels) 1.96 ms; with room for
# exactly one token every other slab starts in the middle of a 128-byte line, which cost the decode
# launch 11 % before the kernel learnt to start its items on a line.
STEP_HEADROOM = 256
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth
CALIB_BYTES = 1 << 30    # size of the plain copy that scales the HBM byte counters


def log(msg):
    """progress on stderr (stdout carries the one JSON line)"""
    print("[bench %6.1fs] %s" % (time.perf_counter() - _T0, msg), file=sys.stderr, flush=True)


_T0 = time.perf_counter()


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--configs", default="C2,C3,C4,C5",
                    help="configurations whose kernels are timed for roofline.configs")
    ap.add_argument("--no-sweep", action="store_true", help="C5: only 4-bit block 64 (default: k in {2,3,4} x block in {64,128})")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the `kernels` section (dequantize, paper flow, length mixes, paged, several queries, C2 loop)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--traffic", choices=("live", "none"), default="live",
                    help="live: measure HBM bytes of the roofline kernel with two rocprofv3 counter passes over a child process")
    ap.add_argument("--kernel-launches", type=int, default=120, help="timed launches per kernel entry (>= 100)")
    ap.add_argument("--cold", type=int, default=1, help="1: rotate buffers to defeat the last-level cache")
    ap.add_argument("--timeline", default="",
                    help="instead of the benchmark: per-phase timestamps from inside the decode kernel for these "
                         "configurations (e.g. C4,C3,C2), using the measurement build libnqkv_timeline.so "
                         "(python paper_2505_16210_amd/build.py --timeline); prints a text report")
    ap.add_argument("--kernels-only", default="",
                    help="for profiler runs (rocprofv3 --kernel-trace / --pmc ... -- python3 bench.py --kernels-only C3,C4,C5): "
                         "a plain 1 GiB copy kernel (the yardstick HBM byte counters are scaled by), then quantize, decode "
                         "attention, fused decode step and dequantize of these configurations, three eager launches each; "
                         "no timing, no JSON")
    return ap.parse_args()


# ---------------------------------------------------------------------------------------------
# HBM traffic of the roofline kernel, measured in this run: rocprofv3 --pmc over a child process
# ---------------------------------------------------------------------------------------------
def kernels_only(config_names, sweep):
    """Runs under a profiler: a plain copy of known size, then the kernels of the named configurations."""
    import torch
    from paper_2505_16210_amd import benchaux, nqkv, workloads
    dev = torch.device("cuda:0")
    a = torch.ones(CALIB_BYTES // 4, dtype=torch.int32, device=dev)
    b = torch.empty_like(a)
    for _ in range(3):
        benchaux.copy(b, a)
    torch.cuda.synchronize()
    del a, b
    for cn in config_names:
        cfg = workloads.CONFIGS[cn]
        B, H, D, S = cfg.B, cfg.H, cfg.D, cfg.S
        g = workloads.make_generator(cfg, dev)
        K, V = workloads.make_kv(cfg, dev, g, n_tokens=S + 1)
        q = workloads.make_q(cfg, dev, g)
        out = torch.empty_like(q)
        variants = [(kb, bl) for kb in (4, 3, 2) for bl in (64, 128)] if (cn == "C5" and sweep) else [(cfg.bits, cfg.block)]
        for kb, bl in variants:
            lv = nqkv.build_codebook(kb)
            desc = nqkv.make_desc(B, H, D, kb, bl, S + STEP_HEADROOM)
            kc, ks = nqkv.alloc_cache(desc, dev)
            vc, vs = nqkv.alloc_cache(desc, dev)
            ws = torch.zeros(2 << 20, dtype=torch.uint8, device=dev)
            back = torch.empty(B, H, S, D, dtype=torch.float16, device=dev)
            for _ in range(3):
                nqkv.quantize_kv_pair(desc, lv, K[:, :, :S], V[:, :, :S], kc, ks, vc, vs, 0)
                nqkv.decode_step(desc, lv, q, K[:, :, S:], V[:, :, S:], kc, ks, vc, vs, S, 1.0, out=out, workspace=ws)
                nqkv.decode_attention(desc, lv, q, kc, ks, vc, vs, S + 1, 1.0, out=out, workspace=ws)
                nqkv.dequantize_kv(desc, lv, kc, ks, 0, S, out=back)
            torch.cuda.synchronize()
            del kc, ks, vc, vs, back
            torch.cuda.empty_cache()
        del K, V
        torch.cuda.empty_cache()


def _counter_per_dispatch(db_path, counter):
    """{kernel name: average counter value per dispatch} from a rocprofv3 results database."""
    import collections
    import sqlite3
    db = sqlite3.connect(db_path)
    rows = db.execute("select kernel_name, counter_name, value, dispatch_id from counters_collection").fetchall()
    per = collections.defaultdict(float)
    for kn, cn, v, did in rows:
        if cn == counter:
            per[(kn, did)] += v
    agg = collections.defaultdict(list)
    for (kn, _), v in per.items():
        agg[kn].append(v)
    return {kn: sum(v) / len(v) for kn, v in agg.items()}


def measure_traffic_live():
    """HBM bytes per launch of the C5 kernels: FETCH_SIZE and WRITE_SIZE (KiB per dispatch), one
    counter per rocprofv3 run, each scaled by what the same counter reads for a plain 1 GiB copy.
    Must run before this process touches the GPU.  Returns a dict or a string saying why not."""
    prof = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(prof):
        return "rocprofv3 not found"
    if any("rocprof" in os.environ.get(v, "").lower() for v in ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES", "ROCPROFILER_REGISTER_FORCE_LOAD")):
        return "this run is itself under a profiler"
    got = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        outdir = tempfile.mkdtemp(prefix="nqkv_pmc_", dir="/tmp")
        try:
            env = dict(os.environ, TMPDIR="/tmp")
            cmd = [prof, "--pmc", counter, "-d", outdir, "-o", "p", "--", sys.executable, os.path.join(ROOT, "bench.py"), "--kernels-only", "C5", "--no-sweep"]
            r = subprocess.run(cmd, cwd="/tmp", env=env, capture_output=True, text=True, timeout=240)
            if r.returncode != 0:
                return "rocprofv3 --pmc %s exited with %d: %s" % (counter, r.returncode, (r.stderr or r.stdout)[-200:].replace("\n", " "))
            dbs = [os.path.join(dp, f) for dp, _, fs in os.walk(outdir) for f in fs if f.endswith("_results.db")]
            if not dbs:
                return "no results database from rocprofv3 --pmc %s" % counter
            got[counter] = _counter_per_dispatch(dbs[0], counter)
            log("counter pass %s done" % counter)
        except Exception as e:      # a missing profiler must not cost the benchmark its result
            return "%s pass failed: %s" % (counter, str(e)[:200])
        finally:
            shutil.rmtree(outdir, ignore_errors=True)

    def pick(counter, needle):
        hits = [v for kn, v in got[counter].items() if needle in kn.replace(" ", "")]
        return hits[0] if len(hits) == 1 else None

    res = {"method": "rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, one run each over a child process of this bench "
                     "(KiB per dispatch), each scaled by what the counter reads for a plain 1 GiB copy kernel"}
    scale = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        c = pick(counter, "nqkv::(anonymousnamespace)::copy_kernel")
        if not c:
            return "calibration copy not found in the %s pass" % counter
        scale[counter] = (CALIB_BYTES / 1024.0) / c
    res["scale_fetch"], res["scale_write"] = round(scale["FETCH_SIZE"], 4), round(scale["WRITE_SIZE"], 4)
    for name, needle in (("decode_step_fused", "decode_kernel<4,128,64,true,"), ("decode_attention", "decode_kernel<4,128,64,false,"),
                         ("quantize", "quantize_slab_kernel<4,128,64,")):
        f, w = pick("FETCH_SIZE", needle), pick("WRITE_SIZE", needle)
        if f is None or w is None:
            res[name] = None
            continue
        res[name] = {"read_bytes": int(f * scale["FETCH_SIZE"] * 1024), "written_bytes": int(w * scale["WRITE_SIZE"] * 1024)}
    return res


# ---------------------------------------------------------------------------------------------
def main():
    args = parse_args()
    if args.kernels_only:
        kernels_only([c for c in args.kernels_only.split(",") if c], not args.no_sweep)
        return
    if args.timeline:
        timeline_report(args.timeline.split(","))
        return
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards by batch/head with no "
              "exchange); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    traffic = measure_traffic_live() if args.traffic == "live" else "not requested (--traffic none)"

    import torch
    from paper_2505_16210_amd import benchaux, nqkv, workloads

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    n_launch = max(100, args.kernel_launches)

    def timed_graph(fn, n_nodes, min_launches=n_launch):
        """fn(i), i in [0, n_nodes), captured into one HIP graph; the replays are timed with events
        on the launch stream, so a figure holds no host launch overhead (several kernels here run
        3-50 us, about what one launch from Python costs).  -> (avg, median, min) milliseconds per
        launch over at least min_launches launches (median / min over replays)."""
        for i in range(min(n_nodes, 3)):
            fn(i)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            with torch.cuda.graph(gr, stream=side):
                for i in range(n_nodes):
                    fn(i)
        gr.replay()
        torch.cuda.synchronize()
        reps = max(2, -(-min_launches // n_nodes))
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        marks[0].record(stream)
        for r in range(reps):
            gr.replay()
            marks[r + 1].record(stream)
        torch.cuda.synchronize()
        per = sorted(marks[r].elapsed_time(marks[r + 1]) / n_nodes for r in range(reps))
        return marks[0].elapsed_time(marks[reps]) / (reps * n_nodes), per[len(per) // 2], per[0], reps * n_nodes

    def entry(config, kernel, nbytes, t, **extra):
        avg, med, mn, launches = t
        gbps = nbytes / (avg * 1e-3) / 1e9
        e = {"config": config, "kernel": kernel, "us": round(avg * 1e3, 2), "us_median": round(med * 1e3, 2),
             "us_min": round(mn * 1e3, 2), "launches": launches, "bytes": int(nbytes),
             "GBps": round(gbps, 1), "frac": round(gbps / HBM_PEAK_GBPS, 4)}
        e.update(extra)
        return e

    configs_out = []        # roofline.configs
    kern = {}               # further figures

    # ------------------------------------------------------------------ the step: C5, 4-bit, block 64
    cfg = workloads.C5
    B, H, D, S, k, blk = cfg.B, cfg.H, cfg.D, cfg.S, cfg.bits, cfg.block
    want_c5 = "C5" in args.configs.split(",")
    g = workloads.make_generator(cfg, dev)
    K5, V5 = workloads.make_kv(cfg, dev, g, n_tokens=S + 1)          # 7 GiB of fp16: larger than any cache (no rotation needed)
    q5 = workloads.make_q(cfg, dev, g)
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(B, H, D, k, blk, S + STEP_HEADROOM)
    kc, ks = nqkv.alloc_cache(desc, dev)
    vc, vs = nqkv.alloc_cache(desc, dev)
    out5 = torch.empty_like(q5)
    Kp, Vp, Kn, Vn = K5[:, :, :S], V5[:, :, :S], K5[:, :, S:], V5[:, :, S:]

    def step():
        nqkv.quantize_kv_pair(desc, lv, Kp, Vp, kc, ks, vc, vs, 0)
        nqkv.decode_step(desc, lv, q5, Kn, Vn, kc, ks, vc, vs, S, 1.0, out=out5)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_host0 = time.perf_counter()
    e0.record(stream)
    for s in range(args.steps):
        marks[s][0].record(stream)
        nqkv.quantize_kv_pair(desc, lv, Kp, Vp, kc, ks, vc, vs, 0)
        marks[s][1].record(stream)
        nqkv.decode_step(desc, lv, q5, Kn, Vn, kc, ks, vc, vs, S, 1.0, out=out5)
        marks[s][2].record(stream)
    e1.record(stream)
    torch.cuda.synchronize()
    host_ms = (time.perf_counter() - t_host0) * 1e3 / max(args.steps, 1)
    log("timed %d steps" % args.steps)
    ms_per_step = e0.elapsed_time(e1) / max(args.steps, 1)
    t_quant = sorted(m[0].elapsed_time(m[1]) for m in marks)
    t_dec = sorted(m[1].elapsed_time(m[2]) for m in marks)
    per_step = sorted(m[0].elapsed_time(m[2]) for m in marks)
    avg = lambda xs: sum(xs) / max(len(xs), 1)
    per_tok = workloads.decode_bytes_per_token_head(D, k, blk)
    qbytes = 2 * B * H * S * D * workloads.quantize_bytes_per_element(k, blk)
    # fused step: S cached token-heads read, the new token's fp16 rows in and its codes and scales out, q in, out out
    dbytes = B * H * (S * per_tok + 2 * D * 2 + per_tok + 4 * D)
    elems = 2 * B * H * D * S + 2 * B * H * D * (S + 1)               # K and V quantized + K and V attended over
    value = 2 * elems / (ms_per_step * 1e-3) / 1e9
    q_gbps = qbytes / (avg(t_quant) * 1e-3) / 1e9
    dec_gbps = dbytes / (avg(t_dec) * 1e-3) / 1e9
    # The dominant kernel of the step is the quantizer (about four fifths of the step time); the
    # fused decode kernel of the same step is described beside it.  Both are timed live, with
    # events on the launch stream between the launches of the timed steps.
    roofline = {"kernel": "quantize_slab_kernel<k=4, D=128, block=64>, K and V in one launch", "config": "C5 k4 b64",
                "bound": "hbm", "achieved": round(q_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(q_gbps / HBM_PEAK_GBPS, 4), "bytes_per_launch": int(qbytes),
                "avg_launch_us": round(avg(t_quant) * 1e3, 2), "median_launch_us": round(t_quant[len(t_quant) // 2] * 1e3, 2),
                "min_launch_us": round(t_quant[0] * 1e3, 2),
                "share_of_step_time": round(avg(t_quant) / max(avg(t_quant) + avg(t_dec), 1e-9), 3),
                "timing": "HIP events on the launch stream between the launches of the %d timed steps" % args.steps,
                "decode_step": {
                    "kernel": "decode_kernel<k=4, D=128, block=64, fused append>", "bytes_per_launch": int(dbytes),
                    "in_step": {"avg_launch_us": round(avg(t_dec) * 1e3, 2), "min_launch_us": round(t_dec[0] * 1e3, 2),
                                "achieved": round(dec_gbps, 1), "frac": round(dec_gbps / HBM_PEAK_GBPS, 4),
                                "note": "launched right behind the quantizer, which has just written 2 GB: this launch also "
                                        "pays for writing back the dirty lines that pass left in the memory-side last-level "
                                        "cache (measured: the cost follows recent writes of any kernel, survives 1 ms of "
                                        "streaming reads in between and is absent behind a read-only kernel)"}}}
    if isinstance(traffic, dict) and traffic.get("quantize"):
        tq = traffic["quantize"]
        roofline["traffic"] = tq["read_bytes"] + tq["written_bytes"]
        roofline["traffic_over_algorithmic"] = round(roofline["traffic"] / qbytes, 4)
        roofline["traffic_detail"] = traffic
        if traffic.get("decode_step_fused"):
            t_ = traffic["decode_step_fused"]
            roofline["decode_step"]["traffic"] = t_["read_bytes"] + t_["written_bytes"]
            roofline["decode_step"]["traffic_over_algorithmic"] = round((t_["read_bytes"] + t_["written_bytes"]) / dbytes, 4)
    else:
        roofline["traffic"] = None
        roofline["traffic_note"] = traffic if isinstance(traffic, str) else "kernel not found in the counter passes"
    del kc, ks, vc, vs

    # ------------------------------------------------------------------ per-config kernel figures
    names = [c for c in args.configs.split(",") if c]
    if want_c5:
        variants = [(4, 64)] if args.no_sweep else [(kb, bl) for kb in (4, 3, 2) for bl in (64, 128)]
        bench_config(nqkv, workloads, torch, dev, cfg, variants, configs_out, kern, timed_graph, entry, args.cold,
                     not args.no_extras, srcs=[(Kp, Vp)], q=q5)
    del K5, V5, Kp, Vp, Kn, Vn
    torch.cuda.empty_cache()
    for name in names:
        if name == "C5":
            continue
        base = workloads.CONFIGS[name]
        bench_config(nqkv, workloads, torch, dev, base, [(base.bits, base.block)], configs_out, kern, timed_graph, entry,
                     args.cold, not args.no_extras)
    order = {"C2": 0, "C3": 1, "C4": 2, "C5": 3}
    configs_out.sort(key=lambda e: order.get(e["config"].split()[0], 9))
    roofline["configs"] = configs_out
    for e in configs_out:
        if e["config"] == "C5 k4 b64" and "fused append" in e["kernel"]:
            roofline["decode_step"]["steady_state"] = {
                "us": e["us"], "achieved": e["GBps"], "frac": e["frac"],
                "note": "the same launch replayed back to back from a HIP graph (%d launches), the cache read from HBM each time" % e["launches"]}

    if not args.no_extras:
        c2_decode_loop(nqkv, benchaux, workloads, torch, dev, stream, kern, timed_graph, args.cold)
        # what this machine's memory system delivers to the simplest reader (2 GiB, 128-bit non-temporal loads)
        buf = torch.empty(1 << 29, dtype=torch.int32, device=dev).fill_(1)
        sums = torch.empty(benchaux.PROBE_WORKGROUPS, dtype=torch.int32, device=dev)
        t_rs = timed_graph(lambda i: benchaux.read_stream(buf, sums), 5, min_launches=20)
        stream_gbps = buf.numel() * 4 / (t_rs[0] * 1e-3) / 1e9
        del buf
        roofline["read_stream_GBps"] = round(stream_gbps, 1)
        roofline["frac_of_read_stream"] = round(roofline["achieved"] / stream_gbps, 4)
        for e in configs_out:
            e["frac_of_read_stream"] = round(e["GBps"] / stream_gbps, 4)
        # ... and to the simplest kernel with the quantizer's read : write mix (4 : 1; the quantizer's own is
        # 3.7 : 1) and the dequantizer's (1 : 4): a mixed stream runs well below a pure read stream on
        # this chip, so these are the yardsticks for those two kernels
        big = torch.empty(1 << 30, dtype=torch.int32, device=dev).fill_(3)          # 4 GiB
        small = torch.empty(1 << 28, dtype=torch.int32, device=dev)                 # 1 GiB
        mix = {}
        for label, (a_, b_, r_, w_) in {"4r:1w": (big, small, 4, 1), "1r:4w": (small, big, 1, 4)}.items():
            moved = benchaux.mix_stream(a_, b_, r_, w_)
            t_mx = timed_graph(lambda i: benchaux.mix_stream(a_, b_, r_, w_), 5, min_launches=20)
            mix[label] = round(moved / (t_mx[0] * 1e-3) / 1e9, 1)
        del big, small
        roofline["mix_stream_GBps"] = mix
        roofline["frac_of_mix_stream"] = round(roofline["achieved"] / mix["4r:1w"], 4)
        for e in configs_out:
            if e["kernel"].startswith("quantize"):
                e["frac_of_mix_stream"] = round(e["GBps"] / mix["4r:1w"], 4)
        for name_, e in kern.items():
            if name_.endswith(".dequantize") and "GBps" in e:
                e["frac_of_mix_stream"] = round(e["GBps"] / mix["1r:4w"], 4)

    result = {
        "metric": "effective KV GB/s (quantize + fused decode attn) & decode tokens/s/layer",
        "value": round(value, 1), "unit": "GB/s (fp16-equivalent KV bytes processed per second)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(per_step[len(per_step) // 2], 4),
        "ms_per_step_min": round(per_step[0], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "C5 OPT-30B-shaped layer: B16 H56 D128, 16384 cached tokens, 4-bit block 64; one step = "
                               "quantize the whole K and V prefill (one launch) + one fused decode step (append the new "
                               "token + dequantize-fused attention over 16385 tokens, one launch); cache capacity "
                               "%d tokens" % (S + STEP_HEADROOM),
                   "storage": "fp16 in/out, %d-bit codes, fp16 scales" % k,
                   "arithmetic": "fp32 accumulation, fp16 look-up table"},
        "decode_tokens_per_s_per_layer": round(B / (avg(t_dec) * 1e-3), 1),
        "decode_step_us": round(avg(t_dec) * 1e3, 2),
        "quantize_us": round(avg(t_quant) * 1e3, 2),
        "host_ms_per_step": round(host_ms, 4),
        "launch": "eager, two launches per step through the C ABI (each kernel runs >= 300 us: the host stays ahead)",
        "roofline": roofline,
    }
    if kern:
        result["kernels"] = kern
    if not args.no_cpu:
        log("cpu baseline (oracle on the host cores)")
        result["cpu_baseline"] = cpu_baseline(workloads, torch, dev)
    log("done")
    print(json.dumps(result))


def timeline_report(config_names):
    """Where the time of one decode launch goes, from inside the kernel: the measurement build of the
    library records the 100 MHz real-time counter in every wave at eight points of its item's life
    (paper_2505_16210_amd/csrc/decode_attention.hip, NQKV_TIMELINE).  One launch per rotating cache
    copy (reads come from HBM); the stamps of the last launch are reported."""
    import numpy as np
    import torch
    from paper_2505_16210_amd import build as lib_build, nqkv, workloads
    if not os.path.exists(lib_build.TIMELINE_LIB):
        sys.exit("bench.py --timeline: build the measurement library first (python paper_2505_16210_amd/build.py --timeline)")
    nqkv.use_library(lib_build.TIMELINE_LIB)
    dev = torch.device("cuda:0")
    tick_us = 0.01                            # s_memrealtime counts at 100 MHz
    names = ["wave running", "first loads issued", "table built", "trips begin", "trips end", "waves merged",
             "partial published, ticket taken", "result stored"]
    for cn in config_names:
        cfg = workloads.CONFIGS[cn]
        B, H, D, S, k, blk = cfg.B, cfg.H, cfg.D, cfg.S, cfg.bits, cfg.block
        g = workloads.make_generator(cfg, dev)
        K, V = workloads.make_kv(cfg, dev, g)
        q = workloads.make_q(cfg, dev, g)
        lv = nqkv.build_codebook(k)
        desc = nqkv.make_desc(B, H, D, k, blk, S)
        per_tok = workloads.decode_bytes_per_token_head(D, k, blk)
        copies = max(2, min(32, -(-(1 << 30) // (B * H * S * per_tok))))
        caches = []
        for r in range(copies):
            kc, ks = nqkv.alloc_cache(desc, dev)
            vc, vs = nqkv.alloc_cache(desc, dev)
            nqkv.quantize_kv_pair(desc, lv, K, V, kc, ks, vc, vs, 0)
            caches.append((kc, ks, vc, vs))
        out = torch.empty(B, H, D, dtype=torch.float16, device=dev)
        ws = torch.zeros(2 << 20, dtype=torch.uint8, device=dev)
        for fused in (False, True):
            splits = nqkv.decode_workspace_bytes(desc, S - 1 if fused else S, 0)[1]
            n_items = min(B * H * splits, 1024)
            for _ in range(2):
                for c in caches:
                    if fused:
                        nqkv.decode_step(desc, lv, q, K[:, :, S - 1:S], V[:, :, S - 1:S], *c, S - 1, 1.0, out=out, workspace=ws)
                    else:
                        nqkv.decode_attention(desc, lv, q, *c, S, 1.0, out=out, workspace=ws)
                torch.cuda.synchronize()
            d = ws[65536:65536 + n_items * 8 * 64].cpu().numpy().view(np.uint64).reshape(n_items, 8, 8).astype(np.int64)
            ws[:65536 + 1024 * 8 * 64].zero_()
            if splits == 1:
                d[:, :, 6] = d[:, :, 5]                                   # no ticket is taken without a split
            rel = (d - d[:, :, 0].min()) * tick_us
            what = "fused decode step" if fused else "decode attention"
            grid = "one workgroup per item" if S // splits >= 4096 else "persistent grid of at most 512 workgroups"
            print("== %s %s: B %d H %d D %d S %d, %d-bit block %d, %d pieces per sequence, %d work items (%s)"
                  % (cn, what, B, H, D, S, k, blk, splits, B * H * splits, grid))
            print("   span inside the kernel (first wave running -> last result stored): %.2f us" % rel[:, :, 7].max())
            print("   workgroup start   min %.2f  median %.2f  max %.2f us" % (rel[:, 0, 0].min(), float(np.median(rel[:, 0, 0])), rel[:, 0, 0].max()))
            for j in range(1, 8):
                x = (d[:, :, j] - d[:, :, j - 1]) * tick_us
                print("   %-32s -> %-32s mean %6.2f  min %6.2f  max %6.2f us" % (names[j - 1], names[j], x.mean(), x.min(), x.max()))
            ends = rel[:, :, 7].max(axis=1)
            print("   workgroup end percentiles 0/25/50/75/100: " + " ".join("%.2f" % v for v in np.percentile(ends, [0, 25, 50, 75, 100])))
            if B * H * splits > 1024 or S // splits < 4096:
                print("   (persistent grid: the stamps are those of each workgroup's items as it met them; 'wave running', 'first loads issued' "
                      "and 'table built' are the workgroup's own start-up and appear once)")
        del caches
        torch.cuda.empty_cache()


def bench_config(nqkv, workloads, torch, dev, base, variants, configs_out, kern, timed_graph, entry, cold, extras,
                 srcs=None, q=None):
    """quantize (K and V in one launch), decode attention and the fused decode step at full size ->
    configs_out; with `extras`, the other calls of the library -> kern."""
    B, H, D, S = base.B, base.H, base.D, base.S
    cname = base.name.split("-")[0]
    fp16_bytes = 2 * B * H * S * D * 2
    g = workloads.make_generator(base, dev)
    if srcs is None:
        # rotate so that copies x working set >= 1 GiB (sources) / packed caches likewise
        r_src = max(1, min(8, -(-(1 << 30) // fp16_bytes))) if cold else 1
        srcs = [workloads.make_kv(base, dev, g) for _ in range(r_src)]
        q = workloads.make_q(base, dev, g)
    r_src = len(srcs)
    out = torch.empty_like(q)
    for (kb, bl) in variants:
        lv = nqkv.build_codebook(kb)
        desc = nqkv.make_desc(B, H, D, kb, bl, S)
        per_tok = workloads.decode_bytes_per_token_head(D, kb, bl)
        packed = B * H * S * per_tok
        r_cache = max(1, min(32, -(-(1 << 30) // packed))) if cold else 1
        caches = []
        for r in range(r_cache):
            kc, ks = nqkv.alloc_cache(desc, dev)
            vc, vs = nqkv.alloc_cache(desc, dev)
            caches.append((kc, ks, vc, vs))
        ws_bytes, splits = nqkv.decode_workspace_bytes(desc, S, 0)
        ws_bytes_f, splits_f = nqkv.decode_workspace_bytes(desc, S - 1, 0)     # the fused step plans over S - 1
        ws = torch.zeros(max(ws_bytes, ws_bytes_f, 16), dtype=torch.uint8, device=dev)

        def quant(i):
            ksrc, vsrc = srcs[i % r_src]
            kc, ks, vc, vs = caches[i % r_cache]
            nqkv.quantize_kv_pair(desc, lv, ksrc, vsrc, kc, ks, vc, vs, 0)

        def attend(i):
            kc, ks, vc, vs = caches[i % r_cache]
            nqkv.decode_attention(desc, lv, q, kc, ks, vc, vs, S, 1.0, out=out, workspace=ws)

        def step_fused(i):
            # the decode step over the same cache: rows [0, S-1) are read, row S-1 is the new token
            kc, ks, vc, vs = caches[i % r_cache]
            ksrc, vsrc = srcs[i % r_src]
            nqkv.decode_step(desc, lv, q, ksrc[:, :, S - 1:S], vsrc[:, :, S - 1:S], kc, ks, vc, vs, S - 1, 1.0,
                             out=out, workspace=ws)

        for r in range(r_cache):
            quant(r)
        nodes = max(r_cache, r_src, 2)
        nodes_small = max(nodes, 40)                     # short kernels: more nodes per replay
        t_q = timed_graph(quant, nodes if fp16_bytes > (1 << 28) else nodes_small)
        t_a = timed_graph(attend, nodes_small)
        t_f = timed_graph(step_fused, nodes_small)
        label = "%s k%d b%d" % (cname, kb, bl)
        tag = "%s.k%d.b%d" % (cname, kb, bl)
        qbytes = 2 * B * H * S * D * workloads.quantize_bytes_per_element(kb, bl)
        part = lambda sp: (2 * B * H * sp * (D + 2) * 4 if sp > 1 else 0)      # partial results written and re-read
        dbytes = packed + B * H * 4 * D + part(splits)
        fbytes = B * H * ((S - 1) * per_tok + 2 * D * 2 + per_tok + 4 * D) + part(splits_f)
        configs_out.append(entry(label, "quantize_slab_kernel<%d,%d,%d> K+V" % (kb, D, bl), qbytes, t_q,
                                 src_copies=r_src, cache_copies=r_cache))
        configs_out.append(entry(label, "decode_kernel<%d,%d,%d> attention" % (kb, D, bl), dbytes, t_a, splits=splits,
                                 cache_copies=r_cache, tokens_per_s_per_layer=round(B / (t_a[0] * 1e-3), 1)))
        configs_out.append(entry(label, "decode_kernel<%d,%d,%d,fused append> decode step" % (kb, D, bl), fbytes, t_f,
                                 splits=splits_f, cache_copies=r_cache, tokens_per_s_per_layer=round(B / (t_f[0] * 1e-3), 1)))
        if r_cache > 1:
            # labelled cache-warm figure: the same launch over ONE cache copy, which then waits in the
            # 256 MB last-level cache (all of it at C2 and C4, most of it at C3) -- not an HBM figure
            def attend_warm(i):
                kc, ks, vc, vs = caches[0]
                nqkv.decode_attention(desc, lv, q, kc, ks, vc, vs, S, 1.0, out=out, workspace=ws)
            t_w = timed_graph(attend_warm, nodes_small)
            configs_out[-2]["cache_warm_us"] = round(t_w[0] * 1e3, 2)
        log("%s: quantize %.1f us, attention %.1f us, fused step %.1f us" % (label, t_q[0] * 1e3, t_a[0] * 1e3, t_f[0] * 1e3))
        if extras:
            bench_extras(nqkv, workloads, torch, dev, base, kb, bl, lv, desc, srcs, q, out, caches, ws, splits, packed, qbytes,
                         fp16_bytes, t_a, tag, kern, timed_graph, entry, g)
        del caches, ws
        torch.cuda.empty_cache()


def bench_extras(nqkv, workloads, torch, dev, base, kb, bl, lv, desc, srcs, q, out, caches, ws, splits, packed, qbytes, fp16_bytes,
                 t_a, tag, kern, timed_graph, entry, g):
    """The library's other calls at this configuration: dequantize, the paper's own decode flow,
    a length mix, the paged cache, several queries per step, the paper's block geometry."""
    B, H, D, S = base.B, base.H, base.D, base.S
    r_src, r_cache = len(srcs), len(caches)
    few = 24                                               # these figures: 24+ launches each
    ent = lambda nbytes, t, **kw: {k_: v for k_, v in entry("", "", nbytes, t, **kw).items() if k_ not in ("config", "kernel")}
    part = lambda sp, ql=1: (2 * B * H * sp * ql * (D + 2) * 4 if sp > 1 else 0)
    if fp16_bytes <= (8 << 30):
        k_full = torch.empty(B, H, S, D, dtype=torch.float16, device=dev)
        v_full = torch.empty_like(k_full)
        scores = torch.empty(B, H, 1, S, dtype=torch.float16, device=dev)
        probs32 = torch.empty(B, H, 1, S, dtype=torch.float32, device=dev)
        probs16 = torch.empty_like(scores)
        out_pf = torch.empty(B, H, 1, D, dtype=torch.float16, device=dev)

        def dequant_both(i):
            nqkv.dequantize_kv(desc, lv, *caches[i % r_cache][:2], 0, S, out=k_full)
            nqkv.dequantize_kv(desc, lv, *caches[i % r_cache][2:], 0, S, out=v_full)

        def paper_flow(i):
            # the decode flow as the paper runs it: restore the whole cache to fp16, then attention
            # as two batched matrix products around a softmax (library GEMMs; fp32 softmax)
            dequant_both(i)
            torch.matmul(q.unsqueeze(2), k_full.transpose(-1, -2), out=scores)
            torch.softmax(scores.float(), dim=-1, out=probs32)
            probs16.copy_(probs32)
            torch.matmul(probs16, v_full, out=out_pf)

        t_d = timed_graph(dequant_both, max(r_cache, 2), min_launches=few)
        kern[tag + ".dequantize"] = ent(packed + fp16_bytes, t_d, launches_per_call=2)
        # eager: library GEMMs inside a captured graph are not this build's business
        for i in range(2):
            paper_flow(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n_pf = 6
        e0.record()
        for i in range(n_pf):
            paper_flow(i)
        e1.record()
        torch.cuda.synchronize()
        t_p = e0.elapsed_time(e1) / n_pf
        # bytes this flow moves: packed cache in, fp16 cache out, fp16 cache back in
        kern[tag + ".paper_flow_decode"] = ent(packed + 2 * fp16_bytes, (t_p, t_p, t_p, n_pf), fused_speedup=round(t_p / t_a[0], 2))
        del k_full, v_full, scores, probs32, probs16, out_pf
    per_tok = workloads.decode_bytes_per_token_head(D, kb, bl)
    if B >= 8:
        # a length mix (continuous batching): sequence lengths spread evenly over [S/8, S], in a
        # seeded random order over the batch
        lens_host = torch.linspace(S / 8, S, B).round().to(torch.int32)
        lens_host = lens_host[torch.randperm(B, generator=torch.Generator().manual_seed(0))]
        lens_dev = lens_host.to(dev)

        def attend_varlen(i):
            kc, ks, vc, vs = caches[i % r_cache]
            nqkv.decode_attention_varlen(desc, lv, q, kc, ks, vc, vs, lens_dev, S, 1.0, out=out, workspace=ws)

        t_v = timed_graph(attend_varlen, max(r_cache, 8), min_launches=few)
        vbytes = int(lens_host.sum()) * H * per_tok + B * H * 4 * D + part(splits)
        kern[tag + ".decode_attention_varlen"] = ent(vbytes, t_v, splits=splits, lengths="%d..%d evenly spread" % (S // 8, S))
    if B >= 8 and packed <= (1 << 30) and S % 256 == 0:
        # the same cache as a shuffled pool of 256-token pages behind a block table
        P = 256
        n_pg = S // P
        perm = torch.randperm(B * n_pg, generator=torch.Generator().manual_seed(1)).to(dev)
        table = perm.reshape(B, n_pg).to(torch.int32)
        inv = torch.empty_like(perm)
        inv[perm] = torch.arange(B * n_pg, device=dev)

        def to_pool(t):      # [B,H,S,X] -> [B*n_pg,H,P,X], logical page (b, j) stored at page table[b, j]
            X = t.shape[-1]
            pages = t.reshape(B, H, n_pg, P, X).permute(0, 2, 1, 3, 4).reshape(B * n_pg, H, P, X)
            return pages.index_select(0, inv).contiguous()

        pools = [tuple(to_pool(t) for t in c) for c in caches]
        pdesc = nqkv.make_desc(B, H, D, kb, bl, P)
        pws_bytes, p_items = nqkv.decode_paged_workspace_bytes(pdesc, S)
        pws = torch.zeros(max(pws_bytes, 16), dtype=torch.uint8, device=dev)
        full = torch.full((B,), S, dtype=torch.int32, device=dev)

        def attend_paged(i):
            nqkv.decode_attention_paged(pdesc, lv, q, *pools[i % r_cache], table, full, S, 1.0, out=out, workspace=pws)

        def quant_paged(i):
            ksrc, vsrc = srcs[i % r_src]
            nqkv.quantize_kv_paged(pdesc, lv, ksrc, vsrc, *pools[i % r_cache], table, 0)

        kern[tag + ".quantize_paged"] = ent(qbytes, timed_graph(quant_paged, max(r_cache, r_src, 2), min_launches=few), page_tokens=P)
        kern[tag + ".decode_attention_paged"] = ent(packed + B * H * 4 * D + part(p_items),
                                                    timed_graph(attend_paged, max(r_cache, 8), min_launches=few),
                                                    page_tokens=P, pages_per_sequence=n_pg, items_per_sequence=p_items)
        del pools, pws
    # a step that appended q_len tokens (speculative / batched verify): their queries over the same
    # cache, each on its causal prefix, on the matrix cores
    for q_len in ((4, 16) if kb == 4 else (4,)):
        qm = (torch.randn(B, H, q_len, D, device=dev, generator=g) / D ** 0.5).to(torch.float16)
        outm = torch.empty_like(qm)
        mws_bytes, m_splits = nqkv.decode_multi_workspace_bytes(desc, S, q_len, 0)
        mws = torch.empty(max(mws_bytes, 16), dtype=torch.uint8, device=dev)

        def attend_multi(i):
            kc, ks, vc, vs = caches[i % r_cache]
            nqkv.decode_attention_multi(desc, lv, qm, kc, ks, vc, vs, S, 1.0, out=outm, workspace=mws)

        t_m = timed_graph(attend_multi, max(r_cache, 8), min_launches=few)
        mbytes = packed + B * H * q_len * 4 * D + part(m_splits, q_len)
        flops = 4.0 * B * H * S * D * 16                 # two products, 16 query columns issued whatever q_len is
        kern[tag + ".decode_attention_multi.q%d" % q_len] = ent(
            mbytes, t_m, splits=m_splits, q_len=q_len, vs_one_query=round(t_m[0] / t_a[0], 3),
            mfma_TFLOPs_issued=round(flops / (t_m[0] * 1e-3) / 1e12, 1))
        del qm, outm, mws
    if (H * D) % 256 == 0 and bl == 64:
        # the paper's own block geometry: 256 consecutive elements of the token's hidden vector,
        # read from token-major storage (the same bytes viewed as [B,S,H,D]); one scale per head
        desc_h = nqkv.make_desc(B, H, D, kb, D, S)
        caches_h = [nqkv.alloc_cache(desc_h, dev) + nqkv.alloc_cache(desc_h, dev) for _ in range(r_cache)]

        tm = [tuple(t.contiguous().view(B, S, H, D).transpose(1, 2) for t in pair) for pair in srcs]    # token-major views

        def quant_hidden(i):
            ksrc, vsrc = tm[i % r_src]
            kc, ks, vc, vs = caches_h[i % r_cache]
            nqkv.quantize_kv_hidden(desc_h, lv, ksrc, vsrc, kc, ks, vc, vs, 0, 256)

        t_h = timed_graph(quant_hidden, max(r_cache, r_src, 2), min_launches=few)
        kern[tag.rsplit(".", 1)[0] + ".hidden256.quantize"] = ent(2 * B * H * S * D * workloads.quantize_bytes_per_element(kb, D), t_h)
        del caches_h, tm


def c2_decode_loop(nqkv, benchaux, workloads, torch, dev, stream, kern, timed_graph, cold):
    """The OPT-1.3B-shaped decode loop (C2): quantize a 2048-token prefill, then 128 decode steps of
    one launch each, as one HIP graph of 129 kernel nodes over rotating cache copies; beside it the
    cost of an empty kernel node (the launch floor of this machine) and what a fused step takes above
    its ideal time plus that floor."""
    cfg = workloads.C2
    B, H, D, S, steps_dec = cfg.B, cfg.H, cfg.D, cfg.S, cfg.decode_steps
    k, blk, cap = cfg.bits, cfg.block, cfg.cap_tokens
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(B, H, D, k, blk, cap)
    R = 32 if cold else 1
    g = workloads.make_generator(cfg, dev)
    srcs = [workloads.make_kv(cfg, dev, g, n_tokens=S) for _ in range(8 if cold else 1)]
    Knew, Vnew = workloads.make_kv(cfg, dev, g, n_tokens=steps_dec)
    qs = [workloads.make_q(cfg, dev, g) for _ in range(steps_dec)]
    fill_k, fill_v = workloads.make_kv(cfg, dev, g, n_tokens=cap)
    caches = []
    for r in range(R):
        kc, ks = nqkv.alloc_cache(desc, dev)
        vc, vs = nqkv.alloc_cache(desc, dev)
        nqkv.quantize_kv_pair(desc, lv, fill_k.roll(r, 2), fill_v.roll(r, 2), kc, ks, vc, vs, 0)
        caches.append((kc, ks, vc, vs))
    del fill_k, fill_v
    out = torch.empty(B, H, D, dtype=torch.float16, device=dev)
    ws = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
    new_views = [(Knew[:, :, i:i + 1], Vnew[:, :, i:i + 1]) for i in range(steps_dec)]

    def loop(s):
        ksrc, vsrc = srcs[s % len(srcs)]
        kc, ks, vc, vs = caches[s % R]
        nqkv.quantize_kv_pair(desc, lv, ksrc, vsrc, kc, ks, vc, vs, 0)
        for i in range(steps_dec):
            kc, ks, vc, vs = caches[i % R]
            kn, vn = new_views[i]
            nqkv.decode_step(desc, lv, qs[i], kn, vn, kc, ks, vc, vs, S + i, 1.0, out=out, workspace=ws)

    def fused(i):
        kc, ks, vc, vs = caches[i % R]
        j = i % steps_dec
        nqkv.decode_step(desc, lv, qs[j], *new_views[j], kc, ks, vc, vs, S + j, 1.0, out=out, workspace=ws)

    def append(i):
        kc, ks, vc, vs = caches[i % R]
        nqkv.quantize_kv_pair(desc, lv, *new_views[i % steps_dec], kc, ks, vc, vs, S + (i % steps_dec))

    t_loop = timed_graph(lambda i: loop(i), 1, min_launches=20)
    t_fused = timed_graph(fused, steps_dec)
    t_app = timed_graph(append, steps_dec)
    t_empty = timed_graph(lambda i: benchaux.empty_launch(), steps_dec, min_launches=1000)
    per_tok = workloads.decode_bytes_per_token_head(D, k, blk)
    mean_cached = S + (steps_dec - 1) / 2.0
    fbytes = B * H * (mean_cached * per_tok + 2 * D * 2 + per_tok + 4 * D)
    ideal_us = fbytes / (HBM_PEAK_GBPS * 1e9) * 1e6
    elems = 2 * B * H * D * (S + steps_dec) + 2 * B * H * D * sum(S + i + 1 for i in range(steps_dec))
    kern["C2.decode_loop"] = {
        "what": "prefill quantize of 2048 tokens + 128 fused decode steps, one HIP graph of 129 kernel nodes, %d cache copies rotated" % R,
        "ms": round(t_loop[0], 4), "effective_fp16_GBps": round(2 * elems / (t_loop[0] * 1e-3) / 1e9, 1),
        "decode_tokens_per_s_per_layer": round(B / (t_fused[0] * 1e-3), 1)}
    kern["C2.decode_step_fused.in_loop"] = {
        "us": round(t_fused[0] * 1e3, 2), "us_min": round(t_fused[2] * 1e3, 2), "bytes": int(fbytes),
        "frac": round(fbytes / (t_fused[0] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "ideal_us_at_8TBps": round(ideal_us, 2), "empty_kernel_node_us": round(t_empty[0] * 1e3, 2),
        "us_above_ideal_plus_launch_floor": round(t_fused[0] * 1e3 - ideal_us - t_empty[0] * 1e3, 2)}
    kern["C2.quantize_append"] = {"us": round(t_app[0] * 1e3, 2), "note": "separate append launch (the two-launch form of a decode step)"}


def cpu_baseline(workloads, torch, dev):
    """The CPU oracle, as it stands, on half of the C5 workload (batch rows 0-7 of 16, all 56 heads,
    all 16384 tokens, 4-bit block 64): prefill quantize of K and V, then one decode step (quantize
    and append the new token, attention over 16385 tokens).  Inputs are copies of the very fp16
    bits the GPU step uses.  Same definition of effective GB/s as the GPU figure."""
    import numpy as np
    from oracle import nqkv_oracle as oracle

    cfg = workloads.C5
    rows = 8
    H, D, S, k, blk = cfg.H, cfg.D, cfg.S, cfg.bits, cfg.block
    g = workloads.make_generator(cfg, dev)
    Kd, Vd = workloads.make_kv(cfg, dev, g, n_tokens=S + 1)
    qd = workloads.make_q(cfg, dev, g)
    K = Kd[:rows].cpu().numpy().view(np.uint16)
    V = Vd[:rows].cpu().numpy().view(np.uint16)
    q = qd[:rows].cpu().numpy().view(np.uint16)
    del Kd, Vd, qd
    torch.cuda.empty_cache()
    _, lv, _ = oracle.codebook(k)
    threads = oracle.hardware_threads()
    kc, ks = oracle.new_cache(rows, H, D, k, blk, S + 1)
    vc, vs = oracle.new_cache(rows, H, D, k, blk, S + 1)
    t0 = time.perf_counter()
    oracle.quantize_kv(K[:, :, :S], k, blk, lv, kc, ks, 0, threads)
    oracle.quantize_kv(V[:, :, :S], k, blk, lv, vc, vs, 0, threads)
    t1 = time.perf_counter()
    oracle.quantize_kv(K[:, :, S:], k, blk, lv, kc, ks, S, threads)
    oracle.quantize_kv(V[:, :, S:], k, blk, lv, vc, vs, S, threads)
    oracle.decode_attention(q, kc, ks, vc, vs, k, blk, lv, S + 1, 1.0, threads)
    t2 = time.perf_counter()
    elems = 2 * rows * H * D * S + 2 * rows * H * D * (S + 1)
    return {"value": round(2 * elems / (t2 - t0) / 1e9, 4), "unit": "GB/s (fp16-equivalent KV bytes processed per second)",
            "cores": threads, "kind": "oracle",
            "sample": "half of the C5 step: batch rows 0-%d of 16, all %d heads, all %d tokens, the same fp16 bits as the GPU "
                      "step; prefill quantize %.2f s, decode step %.2f s" % (rows - 1, H, S, t1 - t0, t2 - t1),
            "quantize_Melem_per_s": round(2 * rows * H * D * S / (t1 - t0) / 1e6, 2),
            "decode_tokens_per_s_per_layer": round(rows / (t2 - t1), 3)}


if __name__ == "__main__":
    main()
