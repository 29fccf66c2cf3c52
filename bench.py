#!/usr/bin/env python3
"""Benchmark of the Sali-Cache pre-attention filter on one MI355X.

One step = one frame through the whole hot path: the image side (gray + pyramid + polynomial
expansion + flow + per-patch motion + gate; saliency + pooling; tiers + compaction), the K/V pack,
and the dequantise-on-read of that frame.  All inputs (frames and K/V tensors) are resident in HBM
before a timed region starts; a timed region is bracketed by device synchronisations and holds
exactly `--steps` steps.  Every figure is the median of at least PASSES (5) such regions (up to 25
when a region is shorter than 50 ms).

The JSON line carries
  value / ms_per_step        frames/s of the whole path (analysis + store + read-back), workload 2
  sali_step_only             the same steps without the read-back: frames/s and the HBM fraction
                             sum_t bytes(t) / time / 8e12 with bytes(t) = 5 H W + 7 KB + (stored frame)
                             sum over kept tokens of E (2 + w_tier); no unpack term
  roofline                   the dominant kernel (k_pack): algorithmic bytes per launch / average
                             launch duration from HIP events the library records around each launch
                             on the launch stream, in a separate pass over the same steps (an event
                             record costs microseconds of stream time)
  configs                    a short run of workloads 1, 3, 4, 5 with the same quantities
  cpu_baseline               the CPU oracle on a bounded sample
The calls timed are sali_analyze_batch (image side, a batch ahead on two image streams) and
sali_store_batch / sali_kv_decompress_batch (third stream): the batched, overlapped form of
sali_step, identical in results; the one-stream frame-by-frame sali_step is reported beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12
TIER_W = (2.0, 1.0 + 4.0 / 32.0, 0.5 + 4.0 / 32.0 + 2.0 / 32.0)      # bytes written per element: fp16, int8, int4
PASSES = 5
MIN_REGION_S = 0.05          # regions shorter than this are repeated more often (up to 25 regions)


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
    times = []
    for _ in range(PASSES):
        t0 = time.perf_counter()
        run()
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
    rows = ctx.read_frame_table(0, n)
    ctx.close()
    print(json.dumps({"what": "image side alone (sali_analyze_batch, one stream, idle GPU)", "workload": wl.name,
                      "source": f"{wl.width}x{wl.height}", "frames": n, "frames_per_call": batch,
                      "pointer_frames": sum(1 for r in rows if not r.stored),
                      "us_per_frame": statistics.median(times) / n * 1e6,
                      "us_per_frame_passes": [t / n * 1e6 for t in times]}))


class Runner:
    """One workload set up on the GPU: context, resident inputs, streams; runs passes of `steps` steps."""

    def __init__(self, config, steps, n_layers=None, batch=None):
        import torch
        from paper_2602_14236_amd import binding, synth
        self.torch, self.binding = torch, binding
        self.wl = wl = synth.WORKLOADS[config]
        self.config = config
        self.steps = steps
        self.n_layers = wl.n_layers if n_layers is None else n_layers
        self.wl_eff = wl if self.n_layers == wl.n_layers else type(wl)(**{**wl.__dict__, "n_layers": self.n_layers})
        dev = self.dev = torch.device("cuda:0")
        n_src = min(wl.frames, steps)                    # distinct input frames kept resident
        if config == 4:
            n_src = min(n_src, 8)                        # 13B-shaped K/V: 472 MB per frame; a ring > the 256 MB cache
        self.n_src = n_src
        cap = lambda k: max(1, (k if wl.tier_mode == 1 else 576) * steps)
        cfg = binding.make_config(wl.height, wl.width, flow_levels=wl.flow_levels, tier_mode=wl.tier_mode,
                                  k_fp16=wl.k_fp16, k_int8=wl.k_int8, k_int4=wl.k_int4, n_layers=self.n_layers,
                                  n_heads=wl.n_heads, cap_fp16=cap(wl.k_fp16), cap_int8=cap(wl.k_int8),
                                  cap_int4=cap(wl.k_int4), max_frames=steps)
        self.ctx = binding.SaliContext(cfg, dev)
        video = synth.video(config, n_src)
        scale = synth.kv_channel_scale(wl, self.n_layers)
        self.rgbs = [torch.from_numpy(video.frame(t)).to(dev) for t in range(n_src)]
        self.kvs = [synth.kv_frame(wl, t, device=dev, n_layers=self.n_layers, scale=scale) for t in range(n_src)]
        # frames per launch: 4 where the K/V side bounds the path (a larger batch costs more pipeline fill
        # than it saves in a 64-step run), 16 where the image side does (workloads 1, 3 and 5)
        self.batch = batch if batch is not None else int(os.environ.get("SALI_BENCH_BATCH", "16" if config in (1, 3, 5) else "4"))
        self.outs = [torch.empty((self.n_layers, 2, wl.n_heads, 576, 128), dtype=torch.float16, device=dev)
                     for _ in range(max(1, self.batch))]
        # workload 5 is the one with large batches that the K/V side bounds: there a short first call (4, 8, 16, 16, ...)
        # lets the K/V side start earlier; where the image side bounds the path it only costs (measured: -5 to -12 %)
        self.ramp = int(os.environ.get("SALI_BENCH_RAMP", "4" if config == 5 else "0"))
        self.lookahead = int(os.environ.get("SALI_BENCH_LOOKAHEAD", "2"))
        self.ahead = int(os.environ.get("SALI_BENCH_AHEAD", "1"))          # batches analysed ahead of the store
        self.s_imgs = [torch.cuda.Stream() for _ in range(max(2, self.lookahead, self.ahead))]
        self.s_kv = torch.cuda.Stream()
        # a stream gets its hardware queue on first use (milliseconds): use each once before any timing
        for st in self.s_imgs + [self.s_kv]:
            with torch.cuda.stream(st):
                torch.zeros(1, device=dev)
        torch.cuda.synchronize()
        self.host_enqueue = {}

    def close(self):
        self.ctx.close()
        del self.rgbs, self.kvs, self.outs
        self.torch.cuda.empty_cache()

    def make_events(self, n):
        torch = self.torch
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in evs:            # a first record creates the HIP handles
            a.record()
            b.record()
        torch.cuda.synchronize()
        return evs

    def schedule(self, n):
        """Frame ranges of the calls of one pass over n frames: `batch` frames per call, after a ramp from
        `ramp` frames that doubles (a stream's first calls are small, so that the K/V side starts early;
        a long stream does not notice, a short timed region does)."""
        out, t, size = [], 0, min(self.ramp, self.batch) if self.ramp > 0 else self.batch
        while t < n:
            out.append(range(t, min(n, t + size)))
            t += size
            size = min(self.batch, 2 * size)
        return out

    def run(self, n, with_unpack, pack_events=None, unpack_events=None):
        """Frames are analysed ahead on the image streams while frame t is stored (and read back)
        on s_kv.  Same kernels and same results as sali_step frame by frame."""
        ctx, torch, B, n_src = self.ctx, self.torch, self.batch, self.n_src
        rgbs, kvs, outs, s_imgs, s_kv = self.rgbs, self.kvs, self.outs, self.s_imgs, self.s_kv

        sched = self.schedule(n)

        def analyze(b):
            if b < len(sched):
                frames = sched[b]
                ctx.analyze_batch([rgbs[t % n_src] for t in frames], frames[0], s_imgs[b % len(s_imgs)])

        if B > 1:
            # batch b + 1 is analysed while batch b is stored and read back, each in one launch
            for b in range(self.ahead):
                analyze(b)
            for b, frames in enumerate(sched):
                analyze(b + self.ahead)
                if pack_events is not None:
                    ctx.set_profile_events(0, *pack_events[b])
                ctx.store_batch([kvs[t % n_src] for t in frames], frames[0], s_kv)
                if with_unpack:
                    if unpack_events is not None:
                        ctx.set_profile_events(1, *unpack_events[b])
                    ctx.kv_decompress_batch(frames[0], outs[:len(frames)], None, s_kv)
            return
        L = self.lookahead
        for t in range(min(L, n)):
            ctx.step_pipelined(rgbs[t % n_src], t, None, -1, s_imgs[t % L], s_kv)
        for t in range(n):
            if pack_events is not None:
                ctx.set_profile_events(0, *pack_events[t])
            a = t + L
            nxt = rgbs[a % n_src] if a < n else None
            ctx.step_pipelined(nxt, a, kvs[t % n_src], t, s_imgs[a % L], s_kv)
            if with_unpack:
                if unpack_events is not None:
                    ctx.set_profile_events(1, *unpack_events[t])
                with torch.cuda.stream(s_kv):
                    ctx.kv_decompress(t, outs[0])

    def run_serial(self, n, with_unpack):
        """sali_step (+ sali_kv_decompress) frame by frame on one stream."""
        for t in range(n):
            self.ctx.step(self.rgbs[t % self.n_src], self.kvs[t % self.n_src], t)
            if with_unpack:
                self.ctx.kv_decompress(t, self.outs[0])

    def timed(self, fn, *a):
        """Median over timed regions of exactly `steps` steps each, every region bracketed by device
        synchronisations: PASSES regions, more (up to 25) while they add up to less than 5 x MIN_REGION_S,
        after one untimed region."""
        torch, ctx = self.torch, self.ctx
        times = []
        p = 0
        while True:
            ctx.reset()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn(*a)
            enq = time.perf_counter() - t0
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            p += 1
            if p == 1:
                continue                                   # untimed
            times.append(dt)
            self.host_enqueue[(fn.__name__,) + a] = enq
            if len(times) >= PASSES and (sum(times) >= PASSES * MIN_REGION_S or len(times) >= 25):
                break
        return statistics.median(times), times

    def measure(self, full_detail, serial=True):
        """-> dict of this workload's figures."""
        torch, ctx, wl, steps, B = self.torch, self.ctx, self.wl, self.steps, self.batch
        elapsed, passes = self.timed(self.run, steps, True)
        rows = ctx.read_frame_table(0, steps)
        status = ctx.get_status()
        elapsed_step_only, passes_step_only = self.timed(self.run, steps, False)

        # the same steps again with a pair of HIP events around every k_pack / k_unpack launch
        ctx.reset()
        n_launch = len(self.schedule(steps)) if B > 1 else steps
        pack_ev, unpack_ev = self.make_events(n_launch), self.make_events(n_launch)
        pack_ms, unpack_ms = [], []
        for _ in range(2 if full_detail else 1):
            ctx.reset()
            torch.cuda.synchronize()
            self.run(steps, True, pack_ev, unpack_ev)
            torch.cuda.synchronize()
            pack_ms += [a.elapsed_time(b) for a, b in pack_ev]
            unpack_ms += [a.elapsed_time(b) for a, b in unpack_ev]
        n_ev_passes = len(pack_ms) // n_launch

        img_b = pack_b = unpack_b = 0.0
        for r in rows:
            i, p, u = algorithmic_bytes(self.wl_eff, r)
            img_b += i
            pack_b += p
            if not r.stored and r.src >= 0:          # dequantise-on-read of a pointer frame reads its source frame
                u = algorithmic_bytes(self.wl_eff, rows[r.src])[2]
            unpack_b += u
        n_stored = sum(1 for r in rows if r.stored)
        pack_s = sum(pack_ms) / 1e3 / n_ev_passes
        unpack_s = sum(unpack_ms) / 1e3 / n_ev_passes
        pack_gbps = pack_b / pack_s / 1e9 if pack_s > 0 and pack_b > 0 else 0.0
        unpack_gbps = unpack_b / unpack_s / 1e9 if unpack_s > 0 and unpack_b > 0 else 0.0
        ramp = f", the first calls {[len(r) for r in self.schedule(steps)[:3]]}" if self.ramp > 0 and B > self.ramp else ""
        step_call = (f"sali_analyze_batch ({B} frames per call{ramp}, {self.ahead} batch(es) ahead of the K/V side) + "
                     f"sali_store_batch" if B > 1 else
                     f"sali_step_pipelined (image analysis runs {self.lookahead} frames ahead of the K/V store)")
        out = {
            "workload": wl.name, "frames": steps, "source": f"{wl.width}x{wl.height}",
            "kv_shape": [self.n_layers, 2, wl.n_heads, 576, 128], "tier_mode": wl.tier_mode,
            "k": [wl.k_fp16, wl.k_int8, wl.k_int4],
            "stored_frames": n_stored, "pointer_frames": steps - n_stored, "status_word": status,
            "calls": step_call + (" + sali_kv_decompress_batch" if B > 1 else " + sali_kv_decompress"),
            "fps": steps / elapsed, "ms_per_step": elapsed / steps * 1e3,
            "fps_passes": [steps / t for t in passes],
            "step_with_readback_hbm_frac": (img_b + pack_b + unpack_b) / elapsed / HBM_PEAK,
            "sali_step_only": {
                "fps": steps / elapsed_step_only, "ms_per_step": elapsed_step_only / steps * 1e3,
                "hbm_frac": (img_b + pack_b) / elapsed_step_only / HBM_PEAK,
                "algorithmic_bytes_per_step": (img_b + pack_b) / steps,
                "fps_passes": [steps / t for t in passes_step_only],
                "what": "the same calls without the read-back: analysis + store, the sali_step of Algorithm 1",
            },
            "k_pack": {"achieved_gbps": pack_gbps, "hbm_frac": pack_gbps / (HBM_PEAK / 1e9),
                       "avg_launch_us": pack_s / n_launch * 1e6, "algorithmic_bytes_per_launch": pack_b / n_launch,
                       "frames_per_launch": max(1, B)},
            "k_unpack": {"achieved_gbps": unpack_gbps, "hbm_frac": unpack_gbps / (HBM_PEAK / 1e9),
                         "avg_launch_us": unpack_s / n_launch * 1e6},
            "host_enqueue_us_per_step": self.host_enqueue[("run", steps, True)] / steps * 1e6,
        }
        if full_detail and serial:
            e_serial, _ = self.timed(self.run_serial, steps, True)
            e_serial_only, _ = self.timed(self.run_serial, steps, False)
            out["one_stream_sali_step"] = {
                "fps_with_readback": steps / e_serial, "fps": steps / e_serial_only,
                "hbm_frac": (img_b + pack_b) / e_serial_only / HBM_PEAK,
                "what": "sali_step frame by frame on one stream (no overlap of image side and K/V side)",
            }
        self._rows = rows
        return out


def attention_figures(rn, result):
    """Just-In-Time Dequantization fused with attention: one decode step = sali_attend_decode of every
    layer over all cached frames (the state the last pass left in the pools), HIP events around the
    main kernel of each call.  Algorithmic bytes = the compressed K and V rows of the layer, once."""
    torch, ctx, wl, steps, n_layers, dev = rn.torch, rn.ctx, rn.wl, rn.steps, rn.n_layers, rn.dev
    rows = rn._rows
    attn_ev = rn.make_events(n_layers)
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
            ctx.attend_decode(layer, q, 0, steps, sm_scale, attn_out, attn_lse, rn.s_kv)
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
    pf_ev = rn.make_events(n_layers)
    for rep in range(2):
        torch.cuda.synchronize()
        for layer in range(n_layers):
            if rep == 1:
                ctx.set_profile_events(2, *pf_ev[layer])
            ctx.attend_decode_gqa(layer, q32, NQ, 0, steps, sm_scale, out32, lse32, rn.s_kv)
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


def recorded_traffic(wl_name):
    """HBM bytes per k_pack launch from rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE runs scaled by a plain
    copy of known size).  Counters cannot be read in-process: the value is the one recorded in
    profiles/ (the file names its command and the code it was taken on), not measured by this run."""
    tpath = os.path.join(ROOT, "profiles", f"k_pack_{wl_name}_pmc.txt")
    if not os.path.exists(tpath):
        return None, None
    for line in open(tpath):
        if line.startswith("hbm_bytes_per_launch:"):
            return float(line.split(":")[1]), os.path.relpath(tpath, ROOT)
    return None, None


# runs of the other workloads: leading frames (workload 5: all of them; workload 1: its 8 frames cycled 8 times)
OTHER_CONFIGS = {1: 64, 3: 128, 4: 32, 5: 128}


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
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--no-attention", action="store_true", help="skip the attention-over-the-cache figures")
    ap.add_argument("--no-serial", action="store_true",
                    help="skip the one-stream frame-by-frame sali_step figures (under a profiler: every dispatch of the "
                         "run then covers the same number of frames)")
    ap.add_argument("--image-only", action="store_true",
                    help="time only the image side (sali_analyze_batch on one stream, nothing else on the GPU) and "
                         "print its cost per frame; not the benchmark, a reference figure for profiling")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy three times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (the method has no cross-GPU step); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_14236_amd import synth

    wl = synth.WORKLOADS[args.config]
    if args.image_only:
        image_only(args, wl)
        return
    torch.cuda.set_device(0)
    steps, warmup = args.steps, args.warmup

    rn = Runner(args.config, steps, args.layers)
    # warm-up: `warmup` untimed steps (in passes of at most `steps`), then forget them
    left = warmup
    while left > 0:
        rn.ctx.reset()
        rn.run(min(left, steps), True)
        left -= min(left, steps)
    torch.cuda.synchronize()
    m = rn.measure(full_detail=True, serial=not args.no_serial)

    traffic, traffic_src = recorded_traffic(wl.name) if args.layers is None else (None, None)
    result = {
        "metric": "frames/s through sali_step + KV compress GB/s (% of HBM peak), 1 MI355X",
        "value": m["fps"],
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": m["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "timing": f"median of {len(m['fps_passes'])} timed regions of exactly {steps} steps each, device-synchronised on both sides",
        "value_is": "whole path per frame: image side + K/V pack + dequantise-on-read (all resident in HBM)",
        "config": {"workload": m["workload"], "frames": steps, "source": m["source"], "kv_shape": m["kv_shape"],
                   "tier_mode": m["tier_mode"], "k": m["k"], "step": m["calls"],
                   "stored_frames": m["stored_frames"], "pointer_frames": m["pointer_frames"],
                   "status_word": m["status_word"]},
        "fps_passes": m["fps_passes"],
        "sali_step_only": m["sali_step_only"],
        "one_stream_sali_step": m.get("one_stream_sali_step"),
        "roofline": {"bound": "hbm", "kernel": "k_pack", "achieved": m["k_pack"]["achieved_gbps"], "peak": HBM_PEAK / 1e9,
                     "unit": "GB/s", "frac": m["k_pack"]["hbm_frac"], "traffic": traffic,
                     "traffic_is": (f"recorded value from {traffic_src} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE), "
                                    "not measured in this run" if traffic is not None else None),
                     "avg_launch_us": m["k_pack"]["avg_launch_us"],
                     "algorithmic_bytes_per_launch": m["k_pack"]["algorithmic_bytes_per_launch"],
                     "frames_per_launch": m["k_pack"]["frames_per_launch"],
                     "timing": "HIP events recorded by the library around each k_pack launch on its stream, "
                               "two further passes over the same steps"},
        "kv_compress_gbps": m["k_pack"]["achieved_gbps"],
        "kv_compress_pct_of_hbm_peak": 100.0 * m["k_pack"]["hbm_frac"],
        "kv_decompress_gbps": m["k_unpack"]["achieved_gbps"],
        "kv_decompress_avg_launch_us": m["k_unpack"]["avg_launch_us"],
        "step_with_readback_hbm_frac": m["step_with_readback_hbm_frac"],
        "host_enqueue_us_per_step": m["host_enqueue_us_per_step"],
    }
    if not args.no_attention:
        attention_figures(rn, result)
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=rn.dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)              # one elementwise copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        result["calibration_copy_bytes"] = 1 << 30
        del src, dst
    wl_eff = rn.wl_eff
    rn.close()

    if not args.no_others and args.layers is None:
        others = {}
        for cid, n in OTHER_CONFIGS.items():
            if cid == args.config:
                continue
            r2 = Runner(cid, n)
            r2.ctx.reset()
            r2.run(n, True)                  # warm-up pass
            torch.cuda.synchronize()
            o = r2.measure(full_detail=False)
            r2.close()
            keep = ("workload", "frames", "source", "kv_shape", "stored_frames", "pointer_frames", "status_word", "calls",
                    "fps", "ms_per_step", "step_with_readback_hbm_frac", "sali_step_only", "k_pack", "k_unpack")
            others[f"cfg{cid}"] = {k: o[k] for k in keep}
        result["configs"] = others
        result["configs_note"] = ("the leading frames of each workload (5: the whole workload; 1: its 8 frames cycled 8 times), same calls, same timing protocol; "
                                  "workloads 1 and 3 move a few MB per step and are bound by the latency of the image "
                                  "side's launch chain, not by HBM")
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl_eff, synth.video(args.config, 16))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
