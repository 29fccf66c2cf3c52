"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(sali_analyze_batch of four frames one batch ahead on two image streams; sali_store_batch and
sali_kv_decompress_batch on a third).

The oracle cannot hold the full pools, so it runs the image side in full (flow, gate, saliency,
tiers, slots: bit-exact rows / tiers / slots) and quantises a random sample of (layer, K|V, head)
planes, which are compared row by row with the pools and with the dequantised frame."""
import numpy as np
import pytest
import torch

from oracle import flow as oflow
from oracle import quant as oq
from oracle import saliency as osal
from paper_2602_14236_amd import synth

from _util import FLOW_ATOL, FLOW_RTOL, assert_same, close, lib_config, workload_params

pytestmark = pytest.mark.gpu


def _oracle_image_side(wl, p, video, n):
    """Algorithm 1 without the K/V: per frame (stored?, tier, slot, counts, dp, gate)."""
    out = []
    prev = None
    for t in range(n):
        rgb = video.frame(t)
        gray = oflow.gray_float(rgb)
        redundant, dp, gate = False, None, None
        if prev is not None:
            d = oflow.flow_from_gray(prev, gray, p["flow_levels"], p["flow_iters"])
            dp = oflow.patch_motion(d)
            gate = oflow.gate(dp, p["tau_t"], p["theta_r"])
            redundant = gate[2]
        prev = gray
        if redundant:
            out.append(dict(stored=0, dp=dp, gate=gate))
            continue
        scores, _ = osal.saliency_pool(rgb, 24, p["canny_lo"], p["canny_hi"])
        if p["tier_mode"] == 0:
            tier = oq.tiers_threshold(scores, p["tau_high"], p["tau_med"], p["tau_low"])
        else:
            tier = oq.tiers_topk(scores, p["k_fp16"], p["k_int8"], p["k_int4"])
        slot, cnt = oq.slots(tier)
        out.append(dict(stored=1, tier=tier, slot=slot, cnt=cnt, dp=dp, gate=gate, scores=scores))
    return out


def _run_fullsize(cfg_id, n_frames, n_sample_planes, seed):
    from paper_2602_14236_amd import binding
    wl = synth.WORKLOADS[cfg_id]
    p = workload_params(wl, frames=n_frames)
    video = synth.video(cfg_id, n_frames)
    print(f"{wl.name}: oracle image side for {n_frames} frames", flush=True)
    ora = _oracle_image_side(wl, p, video, n_frames)

    ctx = binding.SaliContext(lib_config(p))
    scale = synth.kv_channel_scale(wl)
    rgbs = [torch.from_numpy(video.frame(t)).cuda() for t in range(n_frames)]
    kvs = [synth.kv_frame(wl, t, device="cuda", scale=scale) for t in range(n_frames)]
    outs = [torch.empty_like(kvs[0]) for _ in range(n_frames)]
    batch = 4
    s_imgs = [torch.cuda.Stream(), torch.cuda.Stream()]
    s_kv = torch.cuda.Stream()
    torch.cuda.synchronize()
    print(f"{wl.name}: GPU run, {batch} frames per launch, analysis one batch ahead", flush=True)
    n_batches = (n_frames + batch - 1) // batch

    def analyze(b):
        if b < n_batches:
            ctx.analyze_batch(rgbs[b * batch:(b + 1) * batch], b * batch, s_imgs[b % 2])

    analyze(0)
    for b in range(n_batches):
        analyze(b + 1)
        ctx.store_batch(kvs[b * batch:(b + 1) * batch], b * batch, s_kv)
        ctx.kv_decompress_batch(b * batch, outs[b * batch:(b + 1) * batch], None, s_kv)
    torch.cuda.synchronize()
    assert ctx.get_status() == 0

    rows = ctx.read_frame_table(0, n_frames)
    n_planes = wl.n_layers * 2 * wl.n_heads
    rng = np.random.default_rng(seed)
    planes = sorted(rng.choice(n_planes, n_sample_planes, replace=False).tolist())
    pv = ctx.pool_views(planes)          # the sampled planes' rows, regrouped per plane
    base = [0, 0, 0]
    last_src = -1
    for t in range(n_frames):
        o = ora[t]
        r = rows[t]
        if not o["stored"]:
            assert (r.stored, r.src) == (0, last_src), f"frame {t} should be a pointer"
            continue
        cnt = o["cnt"]
        assert r.as_tuple() == (t, t, 1, base[0], base[1], base[2], int(cnt[0]), int(cnt[1]), int(cnt[2]), int(cnt[3])), \
            f"row {t}: {r.as_tuple()}"
        tier, slot = ctx.read_frame_tiers(t)
        assert_same(tier, o["tier"], f"tier {t}")
        assert_same(slot.astype(np.int32), o["slot"], f"slot {t}")
        kv_planes = kvs[t].view(n_planes, 576, 128)[planes].cpu().numpy()
        out_planes = outs[t].view(n_planes, 576, 128)[planes].cpu().numpy()
        i16 = np.nonzero(tier == 0)[0]
        i8 = np.nonzero(tier == 1)[0]
        i4 = np.nonzero(tier == 2)[0]
        ip = np.nonzero(tier == 3)[0]
        exp_out = np.zeros_like(kv_planes)
        if i16.size:
            got = pv["fp16"][:, base[0]:base[0] + i16.size].cpu().numpy()
            assert_same(got, kv_planes[:, i16], f"frame {t} fp16 pool rows")
            exp_out[:, i16] = kv_planes[:, i16]
        if i8.size:
            q, s = oq.quant_int8(kv_planes[:, i8])
            assert_same(pv["codes8"][:, base[1]:base[1] + i8.size].cpu().numpy(), q, f"frame {t} int8 codes")
            assert_same(pv["scale8"][:, base[1]:base[1] + i8.size].cpu().numpy(), s, f"frame {t} int8 scales")
            exp_out[:, i8] = oq.dequant_int8(q, s)
        if i4.size:
            q, s, z = oq.quant_int4(kv_planes[:, i4])
            assert_same(pv["codes4"][:, base[2]:base[2] + i4.size].cpu().numpy(), oq.pack_nibbles(q), f"frame {t} int4 codes")
            assert_same(pv["scale4"][:, base[2]:base[2] + i4.size].cpu().numpy(), s, f"frame {t} int4 scales")
            assert_same(pv["zero4"][:, base[2]:base[2] + i4.size].cpu().numpy(), z, f"frame {t} int4 zero-points")
            exp_out[:, i4] = oq.dequant_int4(q, s, z)
        assert_same(out_planes, exp_out, f"frame {t} dequantised planes")
        assert not out_planes[:, ip].any()
        base = [base[0] + int(cnt[0]), base[1] + int(cnt[1]), base[2] + int(cnt[2])]
        last_src = t
    # properties that hold for every plane: FP16-tier rows of the read-back equal the input bit for bit,
    # pruned rows are zero (checked on the whole tensor of the last stored frame)
    t = max(i for i in range(n_frames) if ora[i]["stored"])
    tier = torch.from_numpy(ora[t]["tier"]).cuda()
    full_in = kvs[t].view(n_planes, 576, 128)
    full_out = outs[t].view(n_planes, 576, 128)
    assert bool((full_in[:, tier == 0].view(torch.int16) == full_out[:, tier == 0].view(torch.int16)).all())
    assert not bool(full_out[:, tier == 3].any())
    kept = tier != 3
    err = (full_in[:, kept].float() - full_out[:, kept].float()).abs().amax(dim=(0, 2))
    assert bool(torch.isfinite(err).all())
    ctx.close()
    return ora, rows


def test_config2_full_shape_sampled_planes():
    """64-frame workload's shape: 336x336, 32 x 2 x 32 planes, top-k 173 fp16 / 403 int8; 6 frames (a batch of four and one of two)."""
    ora, rows = _run_fullsize(2, 6, 12, seed=1)
    assert all(o["stored"] for o in ora)


def test_config4_full_shape_sampled_planes():
    """1920x1080 source, 5 pyramid levels, 40 x 2 x 40 planes, top-k 173 fp16 / 403 int4; 2 frames."""
    ora, rows = _run_fullsize(4, 2, 8, seed=2)
    assert all(o["stored"] for o in ora)
    assert ora[1]["gate"][3] > 10 * (FLOW_ATOL + FLOW_RTOL * 0.5)      # gate margin far from the tolerance


def test_config5_full_shape_duplicate_run():
    """7B shape with Student-t K/V and outlier channels; frames 4..8 hold a duplicate run (pointer rows)."""
    ora, rows = _run_fullsize(5, 8, 8, seed=3)
    assert [o["stored"] for o in ora] == [1, 1, 1, 1, 1, 0, 0, 0]


def test_config4_flow_field_1080p():
    """Flow field, per-patch motion and gate of one 1920x1080 frame pair (5 levels, sub-pixel velocities up
    to 12 px/frame; the 32x32-tile variant of the update kernel and the per-level pyramid path)."""
    from paper_2602_14236_amd import binding
    wl = synth.WORKLOADS[4]
    p = workload_params(wl, frames=2, n_layers=1, n_heads=1)
    video = synth.video(4, 2)
    prev, cur = video.frame(0), video.frame(1)
    print("oracle flow 1080p", flush=True)
    d = oflow.flow(prev, cur, 5)
    edp = oflow.patch_motion(d)
    n, r, red, margin = oflow.gate(edp, 0.5, 0.9)
    ctx = binding.SaliContext(lib_config(p))
    uv = torch.empty((2, wl.height, wl.width), dtype=torch.float32, device="cuda")
    dp = torch.empty(576, dtype=torch.float32, device="cuda")
    gate = torch.zeros(4, dtype=torch.int32, device="cuda")
    print("GPU flow 1080p", flush=True)
    ctx.flow_score(torch.from_numpy(prev).cuda(), torch.from_numpy(cur).cuda(), uv, dp, gate)
    torch.cuda.synchronize()
    uv = uv.cpu().numpy()
    err = max(np.abs(uv[0] - d[..., 0]).max(), np.abs(uv[1] - d[..., 1]).max())
    print(f"max |flow err| {err:.3e}, max |flow| {np.abs(d).max():.2f}, gate margin {margin:.3e}", flush=True)
    bad = (~close(uv[0], d[..., 0])).sum() + (~close(uv[1], d[..., 1])).sum()
    assert bad == 0, f"{bad} flow values out of tolerance (max err {err})"
    assert close(dp.cpu().numpy(), edp).all()
    g = gate.cpu().numpy()
    assert (int(g[0]), int(g[2])) == (n, int(red))
    ctx.close()
