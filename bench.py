#!/usr/bin/env python3
"""Benchmark of the Sali-Cache pre-attention filter on one MI355X.

One step = one frame through the whole hot path: sali_step (gray + pyramid + polynomial
expansion + flow + per-patch motion + gate; saliency + pooling; tiers + compaction; K/V pack)
followed by sali_kv_decompress of that frame (dequantise-on-read).  Inputs (all frames and all
K/V tensors of the workload) are resident in HBM before the timed region starts.

Prints one JSON line: frames/s, the HBM roofline of the dominant kernel (k_pack, timed with HIP
events around every launch inside the timed region) and the CPU oracle timed on a bounded sample.
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

HBM_PEAK = 8.0e12
TIER_W = (2.0, 1.0 + 4.0 / 32.0, 0.5 + 4.0 / 32.0 + 2.0 / 32.0)      # bytes written per element: fp16, int8, int4


def algorithmic_bytes(wl, row):
    """Bytes the method must move for one frame (none for a pointer frame beyond the image work)."""
    e = wl.elems_per_token
    image = 5 * wl.height * wl.width + 7 * 1024
    if not row.stored:
        return image, 0, 0
    kept = (row.n16, row.n8, row.n4)
    pack = sum(n * e * (2.0 + w) for n, w in zip(kept, TIER_W))
    unpack = sum(n * e * w for n, w in zip(kept, TIER_W)) + 576 * e * 2.0
    return image, pack, unpack


def cpu_baseline(wl, video, max_frames=16, budget_s=12.0):
    """The oracle, as it stands, on the host cores of this machine: the leading frames of the workload
    at its full K/V shape through step + dequantise-on-read, as many as fit in about `budget_s`
    seconds (at least 2, at most `max_frames`).  Single thread."""
    from threadpoolctl import threadpool_limits
    from oracle.cache import OracleConfig, SaliCacheOracle
    from paper_2602_14236_amd import synth

    frames = max_frames
    cap = lambda k: max(1, (k if wl.tier_mode == 1 else 576) * frames)
    oc = OracleConfig(src_h=wl.height, src_w=wl.width, flow_levels=wl.flow_levels, tier_mode=wl.tier_mode,
                      k_fp16=wl.k_fp16, k_int8=wl.k_int8, k_int4=wl.k_int4, n_layers=wl.n_layers, n_heads=wl.n_heads,
                      cap_fp16=cap(wl.k_fp16), cap_int8=cap(wl.k_int8), cap_int4=cap(wl.k_int4), max_frames=frames)
    scale = synth.kv_channel_scale(wl)
    total = 0.0
    done = 0
    with threadpool_limits(limits=1):
        orc = SaliCacheOracle(oc)
        for t in range(frames):
            if done >= 2 and total >= budget_s:
                break
            rgb = video.frame(t)
            kv = synth.kv_frame(wl, t, scale=scale).numpy()
            a = time.perf_counter()
            orc.step(rgb, kv, t)
            orc.kv_decompress(t)
            total += time.perf_counter() - a
            done += 1
            del kv
    frames = done
    return {"value": frames / total, "unit": "frames/s", "cores": 1, "kind": "oracle",
            "sample": f"first {frames} frames of {wl.name} at the full K/V shape, step + dequantise-on-read, "
                      f"{total:.1f} s of CPU work, one thread"}


def image_only(args, wl):
    """The image side alone: `steps` frames through sali_analyze_batch, four per call, one stream,
    an idle GPU otherwise (K/V shape cut to one plane: the K/V side is not run)."""
    import torch
    from paper_2602_14236_amd import binding, synth
    batch = int(os.environ.get("SALI_BENCH_BATCH", "4"))
    n = max(args.steps, batch)
    cfg = binding.make_config(wl.height, wl.width, flow_levels=wl.flow_levels, tier_mode=wl.tier_mode,
                              k_fp16=wl.k_fp16, k_int8=wl.k_int8, k_int4=wl.k_int4, n_layers=1, n_heads=1,
                              cap_fp16=576 * n, cap_int8=576 * n, cap_int4=576 * n, max_frames=n)
    ctx = binding.SaliContext(cfg, "cuda:0")
    n_src = min(16, n)
    video = synth.video(args.config, n_src)
    rgbs = [torch.from_numpy(video.frame(t)).to("cuda:0") for t in range(n_src)]

    def run():
        ctx.reset()
        for first in range(0, n, batch):
            frames = range(first, min(n, first + batch))
            ctx.analyze_batch([rgbs[t % n_src] for t in frames], first)

    run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.close()
    print(json.dumps({"what": "image side alone (sali_analyze_batch, one stream, idle GPU)", "workload": wl.name,
                      "source": f"{wl.width}x{wl.height}", "frames": n, "frames_per_call": batch,
                      "us_per_frame": dt / n * 1e6}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=64,
                    help="untimed steps before the timed ones; one pass over the 64-frame workload, so that every scratch "
                         "copy, pool region and clock is warm")
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (BASELINE configs); 2 is the metric's")
    ap.add_argument("--layers", type=int, default=None, help="cut the K/V down to this many layers (not a valid bench)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--extras", action="store_true",
                    help="also time the path without the read-back and the one-stream frame-by-frame path")
    ap.add_argument("--image-only", action="store_true",
                    help="time only the image side (sali_analyze_batch on one stream, nothing else on the GPU) and "
                         "print its cost per frame; not the benchmark, a reference figure for profiling")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy three times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (the method has no cross-GPU step); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_14236_amd import binding, synth

    wl = synth.WORKLOADS[args.config]
    if args.image_only:
        image_only(args, wl)
        return
    n_layers = wl.n_layers if args.layers is None else args.layers
    steps, warmup = args.steps, args.warmup
    n_src = min(wl.frames, max(steps, warmup))          # distinct input frames kept resident
    if args.config == 4:
        n_src = min(n_src, 8)                           # 13B-shaped K/V: 472 MB per frame; cycle a ring > the 256 MB cache
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cap = lambda k: max(1, (k if wl.tier_mode == 1 else 576) * steps)
    cfg = binding.make_config(wl.height, wl.width, flow_levels=wl.flow_levels, tier_mode=wl.tier_mode,
                              k_fp16=wl.k_fp16, k_int8=wl.k_int8, k_int4=wl.k_int4, n_layers=n_layers,
                              n_heads=wl.n_heads, cap_fp16=cap(wl.k_fp16), cap_int8=cap(wl.k_int8),
                              cap_int4=cap(wl.k_int4), max_frames=max(steps, warmup))
    ctx = binding.SaliContext(cfg, dev)

    # resident inputs
    video = synth.video(args.config, n_src)
    scale = synth.kv_channel_scale(wl, n_layers)
    rgbs = [torch.from_numpy(video.frame(t)).to(dev) for t in range(n_src)]
    kvs = [synth.kv_frame(wl, t, device=dev, n_layers=n_layers, scale=scale) for t in range(n_src)]
    # frames per launch: 4 where the K/V side bounds the path (a batch of 8 costs more pipeline fill
    # than it saves in a 64-step run), 8 where the image side does (configs 1 and 3: +30 % / +8 %)
    BATCH = int(os.environ.get("SALI_BENCH_BATCH", "8" if args.config in (1, 3) else "4"))
    outs = [torch.empty((n_layers, 2, wl.n_heads, 576, 128), dtype=torch.float16, device=dev)
            for _ in range(max(1, BATCH))]
    out = outs[0]
    torch.cuda.synchronize()

    def make_events(n):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in evs:            # a first record creates the HIP handles
            a.record()
            b.record()
        torch.cuda.synchronize()
        return evs

    # image-side analysis runs ahead of the K/V store: BATCH frames per sali_analyze_batch call, the
    # next batch being analysed on an image stream while the current one is stored on s_kv
    # (BATCH = 1: sali_step_pipelined with LOOKAHEAD single-frame analyses in flight)
    LOOKAHEAD = int(os.environ.get("SALI_BENCH_LOOKAHEAD", "2"))
    AHEAD = int(os.environ.get("SALI_BENCH_AHEAD", "1"))          # batches analysed ahead of the store
    s_imgs = [torch.cuda.Stream() for _ in range(max(2, LOOKAHEAD, AHEAD))]
    s_kv = torch.cuda.Stream()
    # a stream gets its hardware queue on first use (milliseconds): use each once before any timing
    for st in s_imgs + [s_kv]:
        with torch.cuda.stream(st):
            torch.zeros(1, device=dev)
    torch.cuda.synchronize()

    def run(n, with_unpack, pack_events=None, unpack_events=None):
        """Frames are analysed ahead on the image streams while frame t is stored (and read back)
        on s_kv.  Same kernels and same results as sali_step frame by frame."""
        def analyze(b):
            frames = range(b * BATCH, min(n, (b + 1) * BATCH))
            if len(frames) > 0:
                ctx.analyze_batch([rgbs[t % n_src] for t in frames], frames[0], s_imgs[b % len(s_imgs)])

        if BATCH > 1:
            # batch b + 1 is analysed while batch b is stored and read back, each in one launch
            for b in range(AHEAD):
                analyze(b)
            for b in range((n + BATCH - 1) // BATCH):
                frames = range(b * BATCH, min(n, (b + 1) * BATCH))
                analyze(b + AHEAD)
                if pack_events is not None:
                    ctx.set_profile_events(0, *pack_events[b])
                ctx.store_batch([kvs[t % n_src] for t in frames], frames[0], s_kv)
                if with_unpack:
                    if unpack_events is not None:
                        ctx.set_profile_events(1, *unpack_events[b])
                    ctx.kv_decompress_batch(frames[0], outs[:len(frames)], None, s_kv)
            return
        for t in range(min(LOOKAHEAD, n)):
            ctx.step_pipelined(rgbs[t % n_src], t, None, -1, s_imgs[t % LOOKAHEAD], s_kv)
        for t in range(n):
            if pack_events is not None:
                ctx.set_profile_events(0, *pack_events[t])
            a = t + LOOKAHEAD
            nxt = rgbs[a % n_src] if a < n else None
            ctx.step_pipelined(nxt, a, kvs[t % n_src], t, s_imgs[a % LOOKAHEAD], s_kv)
            if with_unpack:
                if unpack_events is not None:
                    ctx.set_profile_events(1, *unpack_events[t])
                with torch.cuda.stream(s_kv):
                    ctx.kv_decompress(t, out)

    def run_serial(n, with_unpack):
        for t in range(n):
            ctx.step(rgbs[t % n_src], kvs[t % n_src], t)
            if with_unpack:
                ctx.kv_decompress(t, out)

    host_enqueue = {}

    def timed(fn, *a):
        ctx.reset()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn(*a)
        host_enqueue[(fn.__name__,) + a] = time.perf_counter() - t0      # host time to enqueue everything
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # warm-up, then forget it
    run(warmup, True)
    torch.cuda.synchronize()

    # timed region: exactly `steps` steps, nothing else on the streams
    elapsed = timed(run, steps, True)
    rows = ctx.read_frame_table(0, steps)
    status = ctx.get_status()

    # the same `steps` steps again with a pair of HIP events around every k_pack / k_unpack launch
    # (recorded by the library on the launch stream).  Kept out of the region above because each
    # event record costs several microseconds of stream time.
    ctx.reset()
    n_launch = (steps + BATCH - 1) // BATCH if BATCH > 1 else steps      # launches of each K/V kernel
    pack_ev, unpack_ev = make_events(n_launch), make_events(n_launch)
    torch.cuda.synchronize()
    run(steps, True, pack_ev, unpack_ev)
    torch.cuda.synchronize()
    pack_ms = [a.elapsed_time(b) for a, b in pack_ev]
    unpack_ms = [a.elapsed_time(b) for a, b in unpack_ev]

    # reference figures: without the read-back, and the one-stream frame-by-frame path
    if args.extras:
        elapsed_step_only = timed(run, steps, False)
        elapsed_serial = timed(run_serial, steps, True)
        elapsed_serial_step_only = timed(run_serial, steps, False)

    wl_eff = wl if n_layers == wl.n_layers else type(wl)(**{**wl.__dict__, "n_layers": n_layers})
    img_b = pack_b = unpack_b = 0.0
    for r in rows:
        i, p, u = algorithmic_bytes(wl_eff, r)
        img_b += i
        pack_b += p
        # dequantise-on-read of a pointer frame reads its source frame
        if not r.stored and r.src >= 0:
            u = algorithmic_bytes(wl_eff, rows[r.src])[2]
        unpack_b += u
    n_stored = sum(1 for r in rows if r.stored)
    pack_s = sum(pack_ms) / 1e3
    unpack_s = sum(unpack_ms) / 1e3
    pack_gbps = pack_b / pack_s / 1e9 if pack_s > 0 else 0.0
    unpack_gbps = unpack_b / unpack_s / 1e9 if unpack_s > 0 else 0.0

    # HBM bytes per k_pack launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE runs, scaled
    # by a plain copy of known size); recorded in profiles/ because counters cannot be read in-process
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"k_pack_{wl.name}_pmc.txt")
    if os.path.exists(tpath) and args.layers is None:
        for line in open(tpath):
            if line.startswith("hbm_bytes_per_launch:"):
                traffic = float(line.split(":")[1])

    result = {
        "metric": "frames/s through sali_step + KV compress GB/s (% of HBM peak), 1 MI355X",
        "value": steps / elapsed,
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": elapsed / steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": wl.name, "frames": steps, "source": f"{wl.width}x{wl.height}",
                   "kv_shape": [n_layers, 2, wl.n_heads, 576, 128], "tier_mode": wl.tier_mode,
                   "k": [wl.k_fp16, wl.k_int8, wl.k_int4], "step": (f"sali_analyze_batch ({BATCH} frames per call, {AHEAD} batch(es) ahead of the K/V side) + sali_store_batch"
                            if BATCH > 1 else
                            f"sali_step_pipelined (image analysis runs {LOOKAHEAD} frames ahead of the K/V store)")
                   + (" + sali_kv_decompress_batch" if BATCH > 1 else " + sali_kv_decompress"),
                   "stored_frames": n_stored, "status_word": status},
        "roofline": {"bound": "hbm", "kernel": "k_pack", "achieved": pack_gbps, "peak": HBM_PEAK / 1e9,
                     "unit": "GB/s", "frac": pack_gbps / (HBM_PEAK / 1e9), "traffic": traffic,
                     "avg_launch_us": pack_s / n_launch * 1e6, "algorithmic_bytes_per_launch": pack_b / n_launch,
                     "frames_per_launch": max(1, BATCH),
                     "timing": "HIP events around each k_pack launch, second pass over the same steps"},
        "kv_compress_gbps": pack_gbps,
        "kv_compress_pct_of_hbm_peak": 100.0 * pack_gbps / (HBM_PEAK / 1e9),
        "kv_decompress_gbps": unpack_gbps,
        "kv_decompress_avg_launch_us": unpack_s / n_launch * 1e6,
        "step_hbm_frac": (img_b + pack_b + unpack_b) / elapsed / HBM_PEAK,
        "host_enqueue_us_per_step": host_enqueue[("run", steps, True)] / steps * 1e6,
    }
    if args.extras:
        result["extras"] = {
            "sali_step_only_fps": steps / elapsed_step_only,
            "sali_step_only_hbm_frac": (img_b + pack_b) / elapsed_step_only / HBM_PEAK,
            "host_enqueue_us_per_step_sali_step_only": host_enqueue[("run", steps, False)] / steps * 1e6,
            "one_stream_fps": steps / elapsed_serial,
            "one_stream_sali_step_only_fps": steps / elapsed_serial_step_only,
            "one_stream_sali_step_only_hbm_frac": (img_b + pack_b) / elapsed_serial_step_only / HBM_PEAK,
        }
    # Just-In-Time Dequantization fused with attention: one decode step = sali_attend_decode of every
    # layer over all cached frames (the state the last pass left in the pools), HIP events around the
    # main kernel of each call.  Algorithmic bytes = the compressed K and V rows of the layer, once.
    attn_ev = make_events(n_layers)
    q = torch.randn((wl.n_heads, 128), device=dev).to(torch.float16)
    attn_out = torch.empty((wl.n_heads, 128), dtype=torch.float32, device=dev)
    attn_lse = torch.empty((wl.n_heads,), dtype=torch.float32, device=dev)
    sm_scale = 1.0 / 128.0 ** 0.5
    for rep in range(2):                    # the first repetition warms up
        torch.cuda.synchronize()
        t_attn = time.perf_counter()
        for layer in range(n_layers):
            if rep == 1:
                ctx.set_profile_events(2, *attn_ev[layer])
            ctx.attend_decode(layer, q, 0, steps, sm_scale, attn_out, attn_lse, s_kv)
        torch.cuda.synchronize()
        t_attn = time.perf_counter() - t_attn
    attn_ms = [a.elapsed_time(b) for a, b in attn_ev]
    row_bytes = (256.0, 144.0, 88.0)        # fp16 row; int8 codes + scales; int4 codes + scales + zero-points
    attn_b = sum(2.0 * wl.n_heads * sum(n * b for n, b in zip((r.n16, r.n8, r.n4), row_bytes)) for r in rows if r.stored)
    attn_s = sum(attn_ms) / 1e3 / n_layers
    result["attend_decode"] = {
        "bound": "hbm", "kernel": "k_attn_partial", "avg_launch_us": attn_s * 1e6,
        "algorithmic_bytes_per_launch": attn_b, "achieved": attn_b / attn_s / 1e9 if attn_s > 0 else 0.0,
        "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": attn_b / attn_s / HBM_PEAK if attn_s > 0 else 0.0,
        "decode_step_ms_all_layers": t_attn * 1e3, "frames": steps,
        "what": "single-query attention of one layer over all cached frames, pools read directly",
    }
    # the same with 32 queries per K/V head (a prompt's tokens against the cached video): matrix-core kernel
    NQ = 32
    q32 = torch.randn((wl.n_heads * NQ, 128), device=dev).to(torch.float16)
    out32 = torch.empty((wl.n_heads * NQ, 128), dtype=torch.float32, device=dev)
    lse32 = torch.empty((wl.n_heads * NQ,), dtype=torch.float32, device=dev)
    pf_ev = make_events(n_layers)
    for rep in range(2):
        torch.cuda.synchronize()
        for layer in range(n_layers):
            if rep == 1:
                ctx.set_profile_events(2, *pf_ev[layer])
            ctx.attend_decode_gqa(layer, q32, NQ, 0, steps, sm_scale, out32, lse32, s_kv)
        torch.cuda.synchronize()
    pf_s = sum(a.elapsed_time(b) for a, b in pf_ev) / 1e3 / n_layers
    pf_flops = 4.0 * 128.0 * NQ * wl.n_heads * sum(r.n16 + r.n8 + r.n4 for r in rows if r.stored)    # Q K^T and P V
    result["attend_32_queries"] = {
        "kernel": "k_attn_prefill", "queries_per_kv_head": NQ, "avg_launch_us": pf_s * 1e6,
        "algorithmic_bytes_per_launch": attn_b, "achieved_gbps": attn_b / pf_s / 1e9 if pf_s > 0 else 0.0,
        "hbm_frac": attn_b / pf_s / HBM_PEAK if pf_s > 0 else 0.0,
        "mfma_tflops_f16": pf_flops / pf_s / 1e12 if pf_s > 0 else 0.0,
        "what": "32 queries per K/V head, one layer over all cached frames, v_mfma_f32_32x32x16_f16 on fp16 operands",
    }
    del q32, out32, lse32
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)              # one elementwise copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        result["calibration_copy_bytes"] = 1 << 30
        del src, dst
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl_eff, synth.video(args.config, 16))
    ctx.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
