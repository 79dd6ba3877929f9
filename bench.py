#!/usr/bin/env python3
"""Benchmark of the NQKV hot path on one MI355X.

One "step" is one pass of the whole hot path over the OPT-1.3B-shaped workload
(batch 8, 32 heads, head_dim 64, 4-bit codes, block 64): quantize a 2048-token prefill
cache (K and V), then 128 decode steps, each appending one token (K and V, one launch) and
running the fused decode attention over everything cached so far.  Inputs are synthetic
(seeded, distributions of paper_2505_16210_amd/workloads.py) and resident in HBM before the
timed region.  To keep the 256 MB last-level cache from serving repeat reads, the step
rotates over 32 independent copies of the cache ("layers") and 8 copies of the fp16 prefill
source, so every launch streams from HBM.

Prints ONE JSON line.  `value` is effective fp16 KV GB/s: 2 bytes x (K and V elements
quantized + K and V elements attended over) per second of the step.  `roofline` describes the
dominant kernel of the step (the fused decode attention); `kernels` adds per-kernel figures
for the larger single-GPU configurations; `cpu_baseline` times the CPU oracle on a bounded
sample of the same workload on this machine's host cores.
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

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--configs", default="C2,C3,C4,C5",
                    help="configurations whose kernels are timed for the `kernels` section")
    ap.add_argument("--sweep", action="store_true", help="C5: also time k in {2,3} and block 128")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--kernel-iters", type=int, default=30)
    ap.add_argument("--cold", type=int, default=1, help="1: rotate buffers to defeat the last-level cache")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch the step's 257 kernels one by one from Python instead of replaying a HIP graph")
    ap.add_argument("--two-launch", action="store_true",
                    help="decode iteration as two launches (quantizer append, then attention) instead of "
                         "the fused single-launch step")
    ap.add_argument("--no-paper-flow", action="store_true",
                    help="skip the paper's own decode flow (dequantize the whole cache, then unfused attention)")
    ap.add_argument("--calib-copy", type=int, default=0,
                    help="with --skip-step: also run a torch copy of this many MiB (counter calibration)")
    ap.add_argument("--skip-step", action="store_true",
                    help="profiling aid: skip the timed C2 step, only run the kernels of --configs")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards by batch/head with no "
              "exchange); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_16210_amd import nqkv, workloads

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()

    def timed(fn, iters, warm=2):
        """average milliseconds per call of fn(i), events on the launch stream"""
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(iters):
            fn(warm + i)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    def timed_graph(fn, n_calls, reps=6):
        """average milliseconds per call of fn(i), i in [0, n_calls): the calls are captured into
        one HIP graph and the replays timed, so the figure holds no host launch overhead (the
        kernels here run 5-35 us, about what one launch from Python costs)"""
        for i in range(min(n_calls, 4)):
            fn(i)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            with torch.cuda.graph(gr, stream=side):
                for i in range(n_calls):
                    fn(i)
        for _ in range(2):
            gr.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            gr.replay()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * n_calls)

    def read_stream_ceiling():
        """GB/s of a plain 128-bit read stream over 2 GiB (the library's probe kernel): what this
        box's memory system delivers to the simplest reader, quoted beside the 8 TB/s peak"""
        buf = torch.empty(1 << 29, dtype=torch.int32, device=dev).fill_(1)
        sums = torch.empty(nqkv.PROBE_WORKGROUPS, dtype=torch.int32, device=dev)
        ms = timed(lambda i: nqkv.probe_read_stream(buf, sums), 10)
        return buf.numel() * 4 / (ms * 1e-3) / 1e9

    if args.skip_step:
        kern = {}
        if args.calib_copy:
            # plain device-to-device copy of known size: the yardstick for HBM byte counters
            # (bitwise_not: a one-read one-write elementwise kernel with a name of its own)
            a = torch.ones(args.calib_copy << 18, dtype=torch.int32, device=dev)
            b = torch.empty_like(a)
            for _ in range(3):
                torch.bitwise_not(a, out=b)
            torch.cuda.synchronize()
            kern["calibration_copy_bytes_each_way"] = a.numel() * 4
            del a, b
        for name in [c for c in args.configs.split(",") if c]:
            base = workloads.CONFIGS[name]
            variants = [(base.bits, base.block)]
            if name == "C5" and args.sweep:
                variants = [(kb, bl) for kb in (4, 3, 2) for bl in (64, 128)]
            bench_config(nqkv, workloads, torch, dev, stream, base, variants, kern, timed, args.kernel_iters, args.cold,
                         not args.no_paper_flow)
        print(json.dumps({"kernels": kern}))
        return

    # ------------------------------------------------------------------ the step (C2)
    cfg = workloads.C2
    B, H, D, S, steps_dec = cfg.B, cfg.H, cfg.D, cfg.S, cfg.decode_steps
    k, blk, cap = cfg.bits, cfg.block, cfg.cap_tokens
    lv = nqkv.build_codebook(k)
    desc = nqkv.make_desc(B, H, D, k, blk, cap)
    R_CACHE = 32 if args.cold else 1
    R_SRC = 8 if args.cold else 1
    g = workloads.make_generator(cfg, dev)
    srcs = [workloads.make_kv(cfg, dev, g, n_tokens=S) for _ in range(R_SRC)]
    Knew, Vnew = workloads.make_kv(cfg, dev, g, n_tokens=steps_dec)
    qs = [workloads.make_q(cfg, dev, g) for _ in range(steps_dec)]
    caches = []
    fill_k, fill_v = workloads.make_kv(cfg, dev, g, n_tokens=cap)
    for r in range(R_CACHE):
        kc, ks = nqkv.alloc_cache(desc, dev)
        vc, vs = nqkv.alloc_cache(desc, dev)
        # every copy starts fully populated so that any position read later holds valid codes
        nqkv.quantize_kv_pair(desc, lv, fill_k.roll(r, 2), fill_v.roll(r, 2), kc, ks, vc, vs, 0)
        caches.append((kc, ks, vc, vs))
    del fill_k, fill_v
    out = torch.empty(B, H, D, dtype=torch.float16, device=dev)
    ws_bytes, splits = nqkv.decode_workspace_bytes(desc, cap, 0)
    ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    new_views = [(Knew[:, :, i:i + 1], Vnew[:, :, i:i + 1]) for i in range(steps_dec)]

    def prefill(s):
        ksrc, vsrc = srcs[s % R_SRC]
        kc, ks, vc, vs = caches[s % R_CACHE]
        nqkv.quantize_kv_pair(desc, lv, ksrc, vsrc, kc, ks, vc, vs, 0)

    def append(i):
        kc, ks, vc, vs = caches[i % R_CACHE]
        kn, vn = new_views[i % steps_dec]
        nqkv.quantize_kv_pair(desc, lv, kn, vn, kc, ks, vc, vs, S + (i % steps_dec))

    def attend(i):
        kc, ks, vc, vs = caches[i % R_CACHE]
        j = i % steps_dec
        nqkv.decode_attention(desc, lv, qs[j], kc, ks, vc, vs, S + j + 1, 1.0, out=out, workspace=ws)

    def fused(i):
        kc, ks, vc, vs = caches[i % R_CACHE]
        j = i % steps_dec
        kn, vn = new_views[j]
        nqkv.decode_step(desc, lv, qs[j], kn, vn, kc, ks, vc, vs, S + j, 1.0, out=out, workspace=ws)

    def step(s):
        prefill(s)
        for i in range(steps_dec):
            if args.two_launch:
                append(i)
                attend(i)
            else:
                fused(i)

    # ------------------------------------------------------------------ per-kernel timings, C2
    it = args.kernel_iters
    kern = {}
    tk = timed if args.no_graph else (lambda fn, n, warm=0: timed_graph(fn, n))
    t_pre = tk(prefill, it)
    qb = workloads.quantize_bytes_per_element(k, blk)
    kern["C2.quantize_prefill"] = kernel_entry(2 * B * H * S * D * qb, t_pre)
    t_app = tk(append, steps_dec * 2)
    kern["C2.quantize_append"] = kernel_entry(2 * B * H * D * qb, t_app)
    t_att = tk(attend, steps_dec * 4, warm=steps_dec)
    mean_seq = S + (steps_dec + 1) / 2.0
    dec_bytes = B * H * (mean_seq * workloads.decode_bytes_per_token_head(D, k, blk) + 4 * D) \
        + (2 * B * H * splits * (D + 2) * 4 if splits > 1 else 0)      # partials written and re-read
    kern["C2.decode_attention"] = kernel_entry(dec_bytes, t_att, splits=splits)
    # fused step: the cached prefix is one token shorter, and the new token costs its fp16 rows
    # in plus its codes and scales out
    t_fused = tk(fused, steps_dec * 4, warm=steps_dec)
    per_tok = workloads.decode_bytes_per_token_head(D, k, blk)
    fused_bytes = dec_bytes - B * H * per_tok + B * H * (2 * D * 2 + per_tok)
    kern["C2.decode_step_fused"] = kernel_entry(fused_bytes, t_fused, splits=splits)
    if args.cold:
        # labelled cache-warm: the same launch over ONE cache copy, which the 256 MB last-level cache keeps
        t_warm = tk(lambda i: nqkv.decode_step(desc, lv, qs[i % steps_dec], *new_views[i % steps_dec], *caches[0],
                                               S + (i % steps_dec), 1.0, out=out, workspace=ws), steps_dec * 2)
        kern["C2.decode_step_fused.cache_warm"] = kernel_entry(fused_bytes, t_warm, splits=splits,
                                                                note="one cache copy, served from the last-level cache")
    if not args.two_launch:
        dec_bytes, t_att = fused_bytes, t_fused          # the dominant kernel of the timed step

    # The step is 1 + 2 * 128 kernel launches of 5-35 us each: issued one by one from Python the
    # host cannot keep up, so the step is captured once into a HIP graph (kernel nodes only) and
    # replayed.  Replays are checked against the eager result before timing.
    step(0)
    torch.cuda.synchronize()
    eager_out = out.clone()
    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step(0)
        for _ in range(3):
            out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager_out), "graph replay differs from eager step"
            prefill(1)                      # eager work between replays
            torch.cuda.synchronize()
        run_step = lambda s_: graph.replay()
    else:
        run_step = step

    for s in range(args.warmup):
        run_step(s)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_host0 = time.perf_counter()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]     # per-step marks: median, min
    e0.record(stream)
    marks[0].record(stream)
    for s in range(args.steps):
        run_step(args.warmup + s)
        marks[s + 1].record(stream)
    e1.record(stream)
    torch.cuda.synchronize()
    host_ms = (time.perf_counter() - t_host0) * 1e3 / args.steps
    ms_per_step = e0.elapsed_time(e1) / args.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    ms_median, ms_min = per_step[len(per_step) // 2], per_step[0]

    # decode-step time as it runs inside the step (graph: no launch gaps)
    t_decode_step = max(ms_per_step - t_pre, 0.0) / steps_dec
    tokens_per_s_layer = B / (t_decode_step * 1e-3)

    elems_quant = 2 * B * H * D * (S + steps_dec)                       # K and V, prefill + appended
    elems_attn = 2 * B * H * D * sum(S + i + 1 for i in range(steps_dec))
    eff_bytes = 2 * (elems_quant + elems_attn)
    value = eff_bytes / (ms_per_step * 1e-3) / 1e9

    traffic_ratio = 1.0032 if args.two_launch else 1.0062
    roofline = {"kernel": "decode_kernel<4,64,64,%s>" % ("false" if args.two_launch else "true"), "bound": "hbm",
                "achieved": round(dec_bytes / (t_att * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(dec_bytes / (t_att * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "bytes_per_launch": int(dec_bytes), "avg_launch_us": round(t_att * 1e3, 2),
                # HBM bytes of one launch from rocprofv3 FETCH_SIZE / WRITE_SIZE (scaled by a 1 GiB copy
                # kernel: x2.000 / x1.000), measured at 2048 tokens: 1.0062 x algorithmic for the fused
                # step, 1.0032 x for attention alone
                # (profiles/hbm_traffic_counters_c2_quantize_decode_fused_step.txt)
                "traffic": int(round(dec_bytes * traffic_ratio)),
                "traffic_source": "rocprofv3 pmc, separate run; ratio measured/algorithmic = %.4f" % traffic_ratio}

    # free the C2 buffers before the big configurations
    del srcs, caches, Knew, Vnew, qs, new_views
    torch.cuda.empty_cache()

    # ------------------------------------------------------------------ larger configurations
    for name in [c for c in args.configs.split(",") if c]:
        base = workloads.CONFIGS[name]
        variants = [(base.bits, base.block)]
        if name == "C5" and args.sweep:
            variants = [(kb, bl) for kb in (4, 3, 2) for bl in (64, 128)]
        bench_config(nqkv, workloads, torch, dev, stream, base, variants, kern, timed, it, args.cold, not args.no_paper_flow,
                     timed_kernels=tk if name == "C2" else None)

    stream_gbps = read_stream_ceiling()
    for e in kern.values():
        e["frac_of_read_stream"] = round(e["GBps"] / stream_gbps, 4)
    roofline["read_stream_GBps"] = round(stream_gbps, 1)
    roofline["frac_of_read_stream"] = round(roofline["achieved"] / stream_gbps, 4)

    result = {
        "metric": "effective KV GB/s (quantize + fused decode attn) & decode tokens/s/layer",
        "value": round(value, 1), "unit": "GB/s (fp16-equivalent KV bytes processed per second)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(ms_median, 4),
        "ms_per_step_min": round(ms_min, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "C2 OPT-1.3B-shaped layer: B8 H32 D64, 4-bit block 64, quantize 2048-token "
                               "prefill + 128 x (append 1 token + fused decode attention, %s); "
                               "%d cache copies rotated" % ("two launches" if args.two_launch else "one launch", R_CACHE),
                   "storage": "fp16 in/out, %d-bit codes, fp16 scales" % k},
        "decode_tokens_per_s_per_layer": round(tokens_per_s_layer, 1),
        "decode_step_us": round(t_decode_step * 1e3, 2),
        "host_ms_per_step": round(host_ms, 4),
        "launch": "eager (Python, one call per kernel)" if args.no_graph else "HIP graph replay (%d kernel nodes per step)" % (1 + steps_dec * (2 if args.two_launch else 1)),
        "roofline": roofline,
        "kernels": kern,
    }
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(workloads)
    print(json.dumps(result))


def kernel_entry(nbytes, ms, **extra):
    gbps = nbytes / (ms * 1e-3) / 1e9
    e = {"us": round(ms * 1e3, 2), "algorithmic_bytes": int(nbytes), "GBps": round(gbps, 1),
         "frac_of_8TBps": round(gbps / HBM_PEAK_GBPS, 4)}
    e.update(extra)
    return e


def bench_config(nqkv, workloads, torch, dev, stream, base, variants, kern, timed, iters, cold, paper_flow_on=True,
                 timed_kernels=None):
    """quantize (K and V in one launch), decode attention, and the fused decode step at full size."""
    B, H, D, S = base.B, base.H, base.D, base.S
    fp16_bytes = 2 * B * H * S * D * 2
    # rotate so that copies x working set >= 1 GiB (sources) / packed caches likewise
    r_src = max(1, min(8, -(-(1 << 30) // fp16_bytes))) if cold else 1
    g = workloads.make_generator(base, dev)
    srcs = [workloads.make_kv(base, dev, g) for _ in range(r_src)]
    q = workloads.make_q(base, dev, g)
    out = torch.empty_like(q)
    for (kb, bl) in variants:
        lv = nqkv.build_codebook(kb)
        desc = nqkv.make_desc(B, H, D, kb, bl, S)
        packed = B * H * S * workloads.decode_bytes_per_token_head(D, kb, bl)
        r_cache = max(1, min(16, -(-(1 << 30) // packed))) if cold else 1
        caches = []
        for r in range(r_cache):
            kc, ks = nqkv.alloc_cache(desc, dev)
            vc, vs = nqkv.alloc_cache(desc, dev)
            caches.append((kc, ks, vc, vs))
        ws_bytes, splits = nqkv.decode_workspace_bytes(desc, S, 0)
        ws_bytes = max(ws_bytes, nqkv.decode_workspace_bytes(desc, S - 1, 0)[0])     # the fused step plans over S - 1
        ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

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

        def paper_flow(i):
            # the decode flow as the paper runs it: restore the whole cache to fp16, then attention
            # as two batched matrix products around a softmax (library GEMMs; fp32 softmax)
            kc, ks, vc, vs = caches[i % r_cache]
            nqkv.dequantize_kv(desc, lv, kc, ks, 0, S, out=k_full)
            nqkv.dequantize_kv(desc, lv, vc, vs, 0, S, out=v_full)
            torch.matmul(q.unsqueeze(2), k_full.transpose(-1, -2), out=scores)
            torch.softmax(scores.float(), dim=-1, out=probs32)
            probs16.copy_(probs32)
            torch.matmul(probs16, v_full, out=out_pf)

        for r in range(r_cache):
            quant(r)
        n_it = max(5, min(iters, int(2000.0 / max(1.0, fp16_bytes / 1e9 * 0.4))))
        tk = timed_kernels or timed       # short kernels: timed through graph replays, without launch gaps
        t_q = tk(quant, n_it, warm=max(2, r_cache))
        t_a = tk(attend, n_it * 2, warm=max(2, r_cache))
        t_f = tk(step_fused, n_it * 2, warm=max(2, r_cache))
        tag = "%s.k%d.b%d" % (base.name.split("-")[0], kb, bl)
        qbytes = 2 * B * H * S * D * workloads.quantize_bytes_per_element(kb, bl)
        dbytes = packed + B * H * 4 * D + (2 * B * H * splits * (D + 2) * 4 if splits > 1 else 0)
        kern[tag + ".quantize"] = kernel_entry(qbytes, t_q, src_copies=r_src)
        kern[tag + ".decode_attention"] = kernel_entry(dbytes, t_a, splits=splits, cache_copies=r_cache,
                                                       tokens_per_s_per_layer=round(B / (t_a * 1e-3), 1))
        if paper_flow_on and fp16_bytes <= (8 << 30):
            k_full = torch.empty(B, H, S, D, dtype=torch.float16, device=dev)
            v_full = torch.empty_like(k_full)
            scores = torch.empty(B, H, 1, S, dtype=torch.float16, device=dev)
            probs32 = torch.empty(B, H, 1, S, dtype=torch.float32, device=dev)
            probs16 = torch.empty_like(scores)
            out_pf = torch.empty(B, H, 1, D, dtype=torch.float16, device=dev)
            t_p = timed(paper_flow, max(3, n_it // 2), warm=2)
            # nqkv_dequantize_kv by itself, K and V of one cache copy per call pair (packed codes and
            # scales in, fp16 out)
            t_d = timed(lambda i: (nqkv.dequantize_kv(desc, lv, *caches[i % r_cache][:2], 0, S, out=k_full),
                                   nqkv.dequantize_kv(desc, lv, *caches[i % r_cache][2:], 0, S, out=v_full)),
                        max(3, n_it // 2), warm=2)
            kern[tag + ".dequantize"] = kernel_entry(packed + fp16_bytes, t_d, launches=2)
            # bytes this flow moves: packed cache in, fp16 cache out, fp16 cache back in
            kern[tag + ".paper_flow_decode"] = kernel_entry(packed + 2 * fp16_bytes, t_p, fused_speedup=round(t_p / t_a, 2))
            del k_full, v_full, scores, probs32, probs16, out_pf
        if B >= 8:
            # a length mix (continuous batching): sequence lengths spread evenly over [S/8, S], in a
            # seeded random order over the batch
            lens_host = torch.linspace(S / 8, S, B).round().to(torch.int32)
            lens_host = lens_host[torch.randperm(B, generator=torch.Generator().manual_seed(0))]
            lens_dev = lens_host.to(dev)

            def attend_varlen(i):
                kc, ks, vc, vs = caches[i % r_cache]
                nqkv.decode_attention_varlen(desc, lv, q, kc, ks, vc, vs, lens_dev, S, 1.0, out=out, workspace=ws)

            t_v = tk(attend_varlen, n_it * 2, warm=max(2, r_cache))
            vbytes = int(lens_host.sum()) * H * workloads.decode_bytes_per_token_head(D, kb, bl) + B * H * 4 * D \
                + (2 * B * H * splits * (D + 2) * 4 if splits > 1 else 0)
            kern[tag + ".decode_attention_varlen"] = kernel_entry(vbytes, t_v, splits=splits,
                                                                  lengths="%d..%d evenly spread" % (S // 8, S))
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

            t_qp = tk(quant_paged, n_it, warm=max(2, r_cache))
            kern[tag + ".quantize_paged"] = kernel_entry(qbytes, t_qp, page_tokens=P)
            t_pg = tk(attend_paged, n_it * 2, warm=max(2, r_cache))
            kern[tag + ".decode_attention_paged"] = kernel_entry(
                packed + B * H * 4 * D + (2 * B * H * p_items * (D + 2) * 4 if p_items > 1 else 0), t_pg,
                page_tokens=P, pages_per_sequence=n_pg, items_per_sequence=p_items)
            if kb == 4:
                qmp = (torch.randn(B, H, 4, D, device=dev, generator=g) / D ** 0.5).to(torch.float16)
                outmp = torch.empty_like(qmp)
                mpws_bytes, mp_splits = nqkv.decode_multi_paged_workspace_bytes(pdesc, S, 4, 0)
                mpws = torch.empty(max(mpws_bytes, 16), dtype=torch.uint8, device=dev)

                def attend_multi_paged(i):
                    nqkv.decode_attention_multi_paged(pdesc, lv, qmp, *pools[i % r_cache], table, full, S, 1.0, out=outmp,
                                                      workspace=mpws)

                t_mp = tk(attend_multi_paged, n_it * 2, warm=max(2, r_cache))
                kern[tag + ".decode_attention_multi_paged.q4"] = kernel_entry(
                    packed + B * H * 4 * 4 * D + (2 * B * H * mp_splits * 4 * (D + 2) * 4 if mp_splits > 1 else 0), t_mp,
                    page_tokens=P, splits=mp_splits, q_len=4)
                del qmp, outmp, mpws
            del pools, pws
        if True:     # (every code width)
            # a step that appended q_len tokens (speculative / batched verify): their queries over the
            # same cache, each on its causal prefix, on the matrix cores
            for q_len in ((4, 16) if kb == 4 else (4,)):
                qm = (torch.randn(B, H, q_len, D, device=dev, generator=g) / D ** 0.5).to(torch.float16)
                outm = torch.empty_like(qm)
                mws_bytes, m_splits = nqkv.decode_multi_workspace_bytes(desc, S, q_len, 0)
                mws = torch.empty(max(mws_bytes, 16), dtype=torch.uint8, device=dev)

                def attend_multi(i):
                    kc, ks, vc, vs = caches[i % r_cache]
                    nqkv.decode_attention_multi(desc, lv, qm, kc, ks, vc, vs, S, 1.0, out=outm, workspace=mws)

                t_m = tk(attend_multi, n_it * 2, warm=max(2, r_cache))
                mbytes = packed + B * H * q_len * 4 * D + (2 * B * H * m_splits * q_len * (D + 2) * 4 if m_splits > 1 else 0)
                flops = 4.0 * B * H * S * D * 16                 # two products, 16 query columns issued whatever q_len is
                kern[tag + ".decode_attention_multi.q%d" % q_len] = kernel_entry(
                    mbytes, t_m, splits=m_splits, q_len=q_len, vs_one_query=round(t_m / t_a, 3),
                    mfma_TFLOPs_issued=round(flops / (t_m * 1e-3) / 1e12, 1))
                if B >= 8 and q_len == 4 and kb == 4:
                    # the same step for the length mix of the per-sequence-length entry
                    mlens_host = torch.linspace(S / 8, S, B).round().to(torch.int32)
                    mlens_host = mlens_host[torch.randperm(B, generator=torch.Generator().manual_seed(0))]
                    mlens = mlens_host.to(dev)

                    def attend_multi_varlen(i):
                        kc, ks, vc, vs = caches[i % r_cache]
                        nqkv.decode_attention_multi_varlen(desc, lv, qm, kc, ks, vc, vs, mlens, S, 1.0, out=outm, workspace=mws)

                    t_mv = tk(attend_multi_varlen, n_it * 2, warm=max(2, r_cache))
                    mvbytes = int(mlens_host.sum()) * H * workloads.decode_bytes_per_token_head(D, kb, bl) \
                        + B * H * q_len * 4 * D + (2 * B * H * m_splits * q_len * (D + 2) * 4 if m_splits > 1 else 0)
                    kern[tag + ".decode_attention_multi_varlen.q%d" % q_len] = kernel_entry(
                        mvbytes, t_mv, splits=m_splits, q_len=q_len, lengths="%d..%d evenly spread" % (S // 8, S))
                del qm, outm, mws
        if (H * D) % 256 == 0:
            # the paper's own block geometry: 256 consecutive elements of the token's hidden vector,
            # read from token-major storage (the same bytes viewed as [B,S,H,D]); one scale per head
            desc_h = nqkv.make_desc(B, H, D, kb, D, S)
            caches_h = [nqkv.alloc_cache(desc_h, dev) + nqkv.alloc_cache(desc_h, dev) for _ in range(r_cache)]

            def quant_hidden(i):
                ksrc, vsrc = srcs[i % r_src]
                kc, ks, vc, vs = caches_h[i % r_cache]
                nqkv.quantize_kv_hidden(desc_h, lv, ksrc.view(B, S, H, D).transpose(1, 2),
                                        vsrc.view(B, S, H, D).transpose(1, 2), kc, ks, vc, vs, 0, 256)

            t_h = tk(quant_hidden, n_it, warm=max(2, r_cache))
            kern[tag.rsplit(".", 1)[0] + ".hidden256.quantize"] = kernel_entry(
                2 * B * H * S * D * workloads.quantize_bytes_per_element(kb, D), t_h, src_copies=r_src)
            del caches_h
        per_tok = workloads.decode_bytes_per_token_head(D, kb, bl)
        kern[tag + ".decode_step_fused"] = kernel_entry(dbytes - B * H * per_tok + B * H * (2 * D * 2 + per_tok), t_f,
                                                        splits=nqkv.decode_workspace_bytes(desc, S - 1, 0)[1])
        del caches, ws
        torch.cuda.empty_cache()


def cpu_baseline(workloads):
    """The CPU oracle, as it stands, on the C2 workload: the full B8 x H32 prefill quantize (K and
    V, 2048 tokens), then all 128 decode steps (append + attention).  Same definition of effective GB/s as the GPU figure."""
    import numpy as np
    from oracle import nqkv_oracle as oracle

    cfg = workloads.C2
    B, H, D, S, k, blk = cfg.B, cfg.H, cfg.D, cfg.S, cfg.bits, cfg.block
    n_steps = 128
    cap = S + n_steps
    rng = np.random.default_rng(0)
    K = rng.standard_normal((B, H, cap, D)).astype(np.float16)
    V = rng.standard_normal((B, H, cap, D)).astype(np.float16)
    q = (rng.standard_normal((n_steps, B, H, D)) / np.sqrt(D)).astype(np.float16)
    _, lv, _ = oracle.codebook(k)
    threads = oracle.hardware_threads()
    kc, ks = oracle.new_cache(B, H, D, k, blk, cap)
    vc, vs = oracle.new_cache(B, H, D, k, blk, cap)
    t0 = time.perf_counter()
    oracle.quantize_kv(K[:, :, :S], k, blk, lv, kc, ks, 0, threads)
    oracle.quantize_kv(V[:, :, :S], k, blk, lv, vc, vs, 0, threads)
    t1 = time.perf_counter()
    for i in range(n_steps):
        oracle.quantize_kv(K[:, :, S + i:S + i + 1], k, blk, lv, kc, ks, S + i, threads)
        oracle.quantize_kv(V[:, :, S + i:S + i + 1], k, blk, lv, vc, vs, S + i, threads)
        oracle.decode_attention(q[i], kc, ks, vc, vs, k, blk, lv, S + i + 1, 1.0, threads)
    t2 = time.perf_counter()
    elems = 2 * B * H * D * (S + n_steps) + 2 * B * H * D * sum(S + i + 1 for i in range(n_steps))
    return {"value": round(2 * elems / (t2 - t0) / 1e9, 4), "unit": "GB/s (fp16-equivalent KV bytes processed per second)",
            "cores": threads, "kind": "oracle",
            "sample": "C2 (B8 H32 D64): prefill quantize of 2048 tokens + all %d decode steps; "
                      "quantize %.2fs, decode %.2fs" % (n_steps, t1 - t0, t2 - t1),
            "quantize_Melem_per_s": round(2 * B * H * D * S / (t1 - t0) / 1e6, 2),
            "decode_tokens_per_s_per_layer": round(B * n_steps / (t2 - t1), 3)}


if __name__ == "__main__":
    main()
