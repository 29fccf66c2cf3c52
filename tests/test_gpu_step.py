"""GPU parity of the chained per-frame path (Algorithm 1) against the oracle, through the C ABI.
Rows, tiers, slots, pool contents and dequantised frames are bit-exact; Delta P within the flow
tolerance; gate decisions equal wherever the oracle's margin to tau_t exceeds that tolerance (the
minimum margin met is printed)."""
import numpy as np
import pytest
import torch

from oracle.cache import SaliCacheOracle
from paper_2602_14236_amd import synth

from _util import FLOW_ATOL, FLOW_RTOL, assert_same, close, lib_config, oracle_config, pool_arrays, workload_params

pytestmark = pytest.mark.gpu


def _run_sequence(p, wl, frames, video):
    from paper_2602_14236_amd import binding
    ctx = binding.SaliContext(lib_config(p))
    orc = SaliCacheOracle(oracle_config(p))
    min_margin = np.inf
    nl, nh = p["n_layers"], p["n_heads"]
    kv_scale = synth.kv_channel_scale(wl, nl, nh)
    for t in frames:
        print(f"{wl.name} frame {t} ({video.kind(t)})", flush=True)
        rgb = video.frame(t)
        kv = synth.kv_frame(wl, t, device="cuda", n_layers=nl, n_heads=nh, scale=kv_scale)
        ctx.step(torch.from_numpy(rgb).cuda(), kv, t)
        dp, gate, scores = ctx.read_last_step()
        row = orc.step(rgb, kv.cpu().numpy(), t)
        if orc.last_gate is not None:
            n, r, red, margin = orc.last_gate
            tau = p["tau_t"]
            fragile = int(np.count_nonzero(np.abs(orc.last_dp - tau) <= FLOW_ATOL + FLOW_RTOL * tau))
            min_margin = min(min_margin, margin)
            assert close(dp, orc.last_dp).all(), f"frame {t}: Delta P out of tolerance"
            assert abs(gate.n_static - n) <= fragile
            assert fragile == 0, "seeded input sits on the threshold: pick another seed"
            assert (gate.n_static, gate.r_frame, gate.redundant) == (n, float(r), int(red)), f"gate of frame {t}"
        if row.stored:
            assert_same(scores, orc.last_scores, f"scores of frame {t}")
    torch.cuda.synchronize()
    print(f"{wl.name}: minimum gate margin {min_margin:.3e}", flush=True)
    return ctx, orc


def _compare_all(ctx, orc, frames):
    rows = ctx.read_frame_table(0, ctx.cfg.max_frames)
    for f in frames:
        assert rows[f].as_tuple() == orc.rows[f].as_tuple(), f"row {f}: {rows[f].as_tuple()} vs {orc.rows[f].as_tuple()}"
        if orc.rows[f].stored:
            tier, slot = ctx.read_frame_tiers(f)
            assert_same(tier, orc.tier[f], f"tier {f}")
            assert_same(slot.astype(np.int32), orc.slot[f], f"slot {f}")
    pa = pool_arrays(ctx)
    c16, c8, c4 = orc.cursor
    assert_same(pa["fp16"][..., :c16, :], orc.pool16[..., :c16, :], "fp16 pool")
    assert_same(pa["codes8"][..., :c8, :], orc.codes8[..., :c8, :], "int8 codes")
    assert_same(pa["scale8"][..., :c8, :], orc.scale8[..., :c8, :], "int8 scales")
    assert_same(pa["codes4"][..., :c4, :], orc.codes4[..., :c4, :], "int4 codes")
    assert_same(pa["scale4"][..., :c4, :], orc.scale4[..., :c4, :], "int4 scales")
    assert_same(pa["zero4"][..., :c4, :], orc.zero4[..., :c4, :], "int4 zero-points")
    c = ctx.cfg
    out = torch.empty((c.n_layers, 2, c.n_heads, 576, 128), dtype=torch.float16, device="cuda")
    valid = torch.empty(576, dtype=torch.uint8, device="cuda")
    for f in frames:
        if orc.rows[f].src < 0:
            continue
        ctx.kv_decompress(f, out, valid)
        torch.cuda.synchronize()
        exp, exp_valid = orc.kv_decompress(f)
        assert_same(out.cpu().numpy(), exp, f"decompressed frame {f}")
        assert_same(valid.cpu().numpy(), exp_valid, f"valid mask {f}")
    assert ctx.get_status() == 0


def test_config1_whole():
    """8 frames 336x336, 1 layer x 32 heads, threshold tiers; frame 3 (0-based) is a byte copy of frame 2."""
    wl = synth.WORKLOADS[1]
    p = workload_params(wl)
    v = synth.video(1)
    ctx, orc = _run_sequence(p, wl, range(8), v)
    assert [orc.rows[t].stored for t in range(8)] == [1, 1, 1, 0, 1, 1, 1, 1]
    assert orc.rows[3].src == 2
    _compare_all(ctx, orc, range(8))
    ctx.close()


def test_slow_drift_reference_is_the_adjacent_frame():
    """A pan of 0.3 px per frame (tau_t = 0.5): measured against the adjacent frame every drifting
    frame is redundant and points at frame 0, measured against the last stored frame the third would
    be stored (the CPU pin of the oracle shows both).  Same frames through sali_step."""
    from paper_2602_14236_amd import binding
    from _util import DRIFT_SHIFTS, drift_frame, params
    p = params(96, 96, flow_levels=2, n_layers=1, n_heads=1, cap_fp16=4000, cap_int8=4000, cap_int4=4000, max_frames=8)
    ctx = binding.SaliContext(lib_config(p))
    orc = SaliCacheOracle(oracle_config(p))
    g = torch.Generator().manual_seed(3)
    for t, s in enumerate(DRIFT_SHIFTS):
        rgb = drift_frame(s)
        kv = torch.randn((1, 2, 1, 576, 128), generator=g).to(torch.float16)
        ctx.step(torch.from_numpy(rgb).cuda(), kv.cuda(), t)
        dp, gate, _ = ctx.read_last_step()
        orc.step(rgb, kv.numpy(), t)
        if t > 0:
            n, r, red, margin = orc.last_gate
            print(f"frame {t}: n_static {n} (device {gate.n_static}), gate margin {margin:.3e}", flush=True)
            assert close(dp, orc.last_dp).all(), f"frame {t}: Delta P out of tolerance"
            fragile = int(np.count_nonzero(np.abs(orc.last_dp - 0.5) <= FLOW_ATOL + FLOW_RTOL * 0.5))
            assert abs(gate.n_static - n) <= fragile and gate.redundant == int(red)
    assert [orc.rows[t].stored for t in range(5)] == [1, 0, 0, 0, 1]
    assert [orc.rows[t].src for t in range(5)] == [0, 0, 0, 0, 4]
    _compare_all(ctx, orc, range(5))
    ctx.close()


def test_tier_params_changed_between_frames():
    """sali_set_tier_params: thresholds -> top-k counts -> other thresholds while the video runs; the
    oracle's configuration is changed at the same frames.  Pool capacities are sized for any mix."""
    from paper_2602_14236_amd import binding
    wl = synth.WORKLOADS[1]
    p = workload_params(wl, n_layers=1, n_heads=3)
    v = synth.video(1)
    ctx = binding.SaliContext(lib_config(p))
    orc = SaliCacheOracle(oracle_config(p))
    kv_scale = synth.kv_channel_scale(wl, 1, 3)
    changes = {3: dict(tier_mode=1, k_fp16=100, k_int8=200, k_int4=150),
               5: dict(tier_mode=0, tau_high=0.5, tau_med=0.2, tau_low=0.1),
               7: dict(tier_mode=1, k_fp16=0, k_int8=0, k_int4=576)}
    for t in range(8):
        if t in changes:
            c = dict(tier_mode=0, tau_high=0.30, tau_med=0.15, tau_low=0.03, k_fp16=0, k_int8=0, k_int4=0)
            c.update(changes[t])
            ctx.set_tier_params(**c)
            for k, val in c.items():
                setattr(orc.cfg, k, val)
        rgb = v.frame(t)
        kv = synth.kv_frame(wl, t, device="cuda", n_layers=1, n_heads=3, scale=kv_scale)
        ctx.step(torch.from_numpy(rgb).cuda(), kv, t)
        orc.step(rgb, kv.cpu().numpy(), t)
    torch.cuda.synchronize()
    rows = {t: orc.rows[t] for t in range(8)}
    assert (rows[4].n16, rows[4].n8, rows[4].n4) == (100, 200, 150) and rows[7].n4 == 576
    assert (rows[5].n16, rows[5].n8, rows[5].n4) != (rows[2].n16, rows[2].n8, rows[2].n4)
    _compare_all(ctx, orc, range(8))
    # an inconsistent set is refused and changes nothing
    with pytest.raises(binding.SaliError) as e:
        ctx.set_tier_params(0, tau_high=0.1, tau_med=0.2, tau_low=0.05)
    assert e.value.code == -4
    with pytest.raises(binding.SaliError) as e:
        ctx.set_tier_params(1, k_fp16=300, k_int8=300, k_int4=1)
    assert e.value.code == -4
    ctx.close()


def test_config3_prefix_near_static_runs():
    """640x360 source, paper-mix top-k tiers; a prefix long enough to hold moving and near-static frames."""
    wl = synth.WORKLOADS[3]
    v = synth.video(3, 100)
    frames = list(range(76, 88))             # crosses from a moving run into a near-static run
    p = workload_params(wl, frames=100, n_layers=1, n_heads=4,
                        cap_fp16=249 * 12, cap_int8=56 * 12, cap_int4=168 * 12)
    ctx, orc = _run_sequence(p, wl, frames, v)
    flags = [orc.rows[t].stored for t in frames]
    assert 0 in flags[1:] and 1 in flags[1:]
    _compare_all(ctx, orc, frames)
    ctx.close()


def test_config5_adversarial_prefix():
    """Scene cuts, duplicate runs, uniform-noise frames; Student-t K/V with outlier channels."""
    wl = synth.WORKLOADS[5]
    v = synth.video(5, 32)
    frames = list(range(0, 24))              # cut at 16, duplicates 5..8, noise at 21, 22
    p = workload_params(wl, frames=32, n_layers=1, n_heads=2)
    ctx, orc = _run_sequence(p, wl, frames, v)
    assert [orc.rows[t].stored for t in (5, 6, 7, 8)] == [0, 0, 0, 0]
    assert orc.rows[16].stored == 1 and orc.rows[21].stored == 1
    _compare_all(ctx, orc, frames)
    ctx.close()


def test_read_analysis_of_recent_frames_only():
    """sali_read_analysis returns a frame's own Delta P / gate / scores while its scratch copy is still its
    own (the 32 most recent analyses) and refuses older or unknown frames."""
    from paper_2602_14236_amd import binding
    from _util import params
    p = params(96, 96, flow_levels=2, n_layers=1, n_heads=1, max_frames=48, cap_fp16=576 * 48, cap_int8=576 * 48,
               cap_int4=576 * 48)
    ctx = binding.SaliContext(lib_config(p))
    rng = np.random.default_rng(0)
    frames = [torch.from_numpy(rng.integers(0, 256, (96, 96, 3), dtype=np.uint8)).cuda() for _ in range(4)]
    seen = {}
    for t in range(40):
        ctx.analyze(frames[t % 4], t)
        seen[t] = ctx.read_analysis(t)
    for t in range(8, 40):                      # still in their scratch copies: identical to what was read at the time
        dp, gate, sc = ctx.read_analysis(t)
        assert np.array_equal(dp, seen[t][0]) and np.array_equal(sc, seen[t][2]) and gate.n_static == seen[t][1].n_static
    assert not np.array_equal(seen[5][2], seen[6][2])
    for bad in (0, 7, 45):
        with pytest.raises(binding.SaliError) as e:
            ctx.read_analysis(bad)
        assert e.value.code == -5
    ctx.close()


def test_reset_forgets_history():
    from paper_2602_14236_amd import binding
    wl = synth.WORKLOADS[1]
    p = workload_params(wl, n_heads=1)
    v = synth.video(1)
    ctx = binding.SaliContext(lib_config(p))
    rgb = torch.from_numpy(v.frame(0)).cuda()
    kv = synth.kv_frame(wl, 0, device="cuda", n_heads=1)
    ctx.step(rgb, kv, 0)
    ctx.step(rgb, kv, 1)                     # identical frame: pointer
    rows = ctx.read_frame_table(0, 2)
    assert (rows[0].stored, rows[1].stored, rows[1].src) == (1, 0, 0)
    ctx.reset()
    ctx.step(rgb, kv, 0)                     # first frame again: stored, cursors restart at 0
    rows = ctx.read_frame_table(0, 2)
    assert rows[0].stored == 1 and rows[0].base16 == 0 and rows[1].src == -1
    ctx.close()


@pytest.mark.parametrize("lookahead", [1, 2, 3])
def test_pipelined_step_matches_oracle(lookahead):
    """sali_step_pipelined (image analysis of later frames on other streams while frame t is stored)
    must leave exactly the state the frame-by-frame path leaves."""
    from paper_2602_14236_amd import binding
    wl = synth.WORKLOADS[1]
    p = workload_params(wl, n_heads=4)
    v = synth.video(1)
    n = 8
    scale = synth.kv_channel_scale(wl, 1, 4)
    rgbs = [torch.from_numpy(v.frame(t)).cuda() for t in range(n)]
    kvs = [synth.kv_frame(wl, t, device="cuda", n_layers=1, n_heads=4, scale=scale) for t in range(n)]
    orc = SaliCacheOracle(oracle_config(p))
    for t in range(n):
        orc.step(v.frame(t), kvs[t].cpu().numpy(), t)
    ctx = binding.SaliContext(lib_config(p))
    s_imgs = [torch.cuda.Stream() for _ in range(lookahead)]
    s_kv = torch.cuda.Stream()
    torch.cuda.synchronize()
    for rep in range(2):                     # twice: the second pass reuses every scratch copy and event
        print(f"pipelined lookahead={lookahead} pass {rep}", flush=True)
        for t in range(min(lookahead, n)):
            ctx.step_pipelined(rgbs[t], t, None, -1, s_imgs[t % lookahead], s_kv)
        for t in range(n):
            a = t + lookahead
            ctx.step_pipelined(rgbs[a] if a < n else None, a, kvs[t], t, s_imgs[a % lookahead], s_kv)
        torch.cuda.synchronize()
        _compare_all(ctx, orc, range(n))
        ctx.reset()
        torch.cuda.synchronize()
    # storing a frame that was never analysed is a synchronous error
    with pytest.raises(binding.SaliError) as e:
        ctx.store(kvs[0], 3, s_kv)
    assert e.value.code == -5
    ctx.close()


def test_batched_analysis_matches_oracle():
    """sali_analyze_batch (the frame is a grid dimension of every image kernel) with batches of mixed
    sizes on two alternating streams, more frames than scratch copies, must leave exactly the state
    the frame-by-frame path leaves: scene cuts, duplicate runs and noise frames included."""
    from paper_2602_14236_amd import binding
    wl = synth.WORKLOADS[5]
    n = 36
    v = synth.video(5, n)
    p = workload_params(wl, frames=n, n_layers=1, n_heads=1)
    scale = synth.kv_channel_scale(wl, 1, 1)
    rgbs = [torch.from_numpy(v.frame(t)).cuda() for t in range(n)]
    kvs = [synth.kv_frame(wl, t, device="cuda", n_layers=1, n_heads=1, scale=scale) for t in range(n)]
    orc = SaliCacheOracle(oracle_config(p))
    for t in range(n):
        orc.step(v.frame(t), kvs[t].cpu().numpy(), t)
    print("oracle done", flush=True)
    assert binding.MAX_BATCH == 16
    sizes = [16, 8, 4, 3, 1, 4]
    assert sum(sizes) == n
    ctx = binding.SaliContext(lib_config(p))
    s_imgs = [torch.cuda.Stream(), torch.cuda.Stream()]
    s_kv = torch.cuda.Stream()
    torch.cuda.synchronize()
    first = 0
    pending = []                             # frames analysed but not yet stored
    for b, size in enumerate(sizes):
        print(f"batch {b}: frames {first}..{first + size - 1}", flush=True)
        ctx.analyze_batch(rgbs[first:first + size], first, s_imgs[b % 2])
        if pending:
            ctx.store_batch([kvs[t] for t in pending], pending[0], s_kv)
        pending = list(range(first, first + size))
        first += size
    for t in pending:                        # the last batch frame by frame
        ctx.store(kvs[t], t, s_kv)
    torch.cuda.synchronize()
    _compare_all(ctx, orc, range(n))
    # batched read-back (pointer frames and scene cuts inside the range) against the oracle
    outs = [torch.empty_like(kvs[0]) for _ in range(8)]
    valid = torch.empty(8 * 576, dtype=torch.uint8, device="cuda")
    ctx.kv_decompress_batch(2, outs, valid, s_kv)
    torch.cuda.synchronize()
    for i in range(8):
        exp, exp_valid = orc.kv_decompress(2 + i)
        assert_same(outs[i].cpu().numpy(), exp, f"batched read-back of frame {2 + i}")
        assert_same(valid[576 * i:576 * (i + 1)].cpu().numpy(), exp_valid, f"batched valid mask {2 + i}")
    # argument checks
    with pytest.raises(binding.SaliError) as e:
        ctx.analyze_batch(rgbs[:17], 0, s_imgs[0])
    assert e.value.code == -2
    with pytest.raises(binding.SaliError) as e:
        ctx.analyze_batch(rgbs[:4], n - 2, s_imgs[0])
    assert e.value.code == -2
    ctx.close()


def test_step_batch_matches_oracle():
    """sali_step_batch: config 1 (one duplicate frame) in two calls of five and three frames."""
    from paper_2602_14236_amd import binding
    wl = synth.WORKLOADS[1]
    p = workload_params(wl, n_heads=2)
    v = synth.video(1)
    n = 8
    scale = synth.kv_channel_scale(wl, 1, 2)
    rgbs = [torch.from_numpy(v.frame(t)).cuda() for t in range(n)]
    kvs = [synth.kv_frame(wl, t, device="cuda", n_layers=1, n_heads=2, scale=scale) for t in range(n)]
    orc = SaliCacheOracle(oracle_config(p))
    for t in range(n):
        orc.step(v.frame(t), kvs[t].cpu().numpy(), t)
    ctx = binding.SaliContext(lib_config(p))
    ctx.step_batch(rgbs[:5], kvs[:5], 0)
    ctx.step_batch(rgbs[5:], kvs[5:], 5)
    torch.cuda.synchronize()
    assert sum(1 for t in range(n) if not orc.rows[t].stored) == 1
    _compare_all(ctx, orc, range(n))
    # a frame that was never analysed cannot be stored
    with pytest.raises(binding.SaliError) as e:
        ctx.store_batch(kvs[:2], 20)
    assert e.value.code in (-2, -5)
    ctx.close()


def test_random_batch_schedules_equal_the_one_stream_path():
    """Property test of the scheduling layer: 120 frames (config 5's scene cuts, duplicate runs and
    noise frames, cycled) analysed in batches of random size 1..8 on three alternating image
    streams, stored in batches of other random sizes on a fourth stream with the analysis up to two
    batches ahead, must leave the frame table, tier tables and pools of the one-stream
    frame-by-frame path (which the other tests tie to the oracle).  More frames than scratch copies
    and ring entries, so every reuse wait is exercised."""
    from paper_2602_14236_amd import binding
    wl = synth.WORKLOADS[5]
    n, n_src = 120, 24
    v = synth.video(5, 32)
    p = workload_params(wl, frames=n, n_layers=1, n_heads=1)
    scale = synth.kv_channel_scale(wl, 1, 1)
    rgbs = [torch.from_numpy(v.frame(t)).cuda() for t in range(n_src)]
    kvs = [synth.kv_frame(wl, t, device="cuda", n_layers=1, n_heads=1, scale=scale) for t in range(n_src)]

    ref = binding.SaliContext(lib_config(p))
    for t in range(n):
        ref.step(rgbs[t % n_src], kvs[t % n_src], t)
    torch.cuda.synchronize()
    ref_rows = [r.as_tuple() for r in ref.read_frame_table(0, n)]
    ref_pools = {k: a.clone() for k, a in ref.pool_views().items()}
    assert 0 < sum(1 for r in ref_rows if r[2] == 0) < n          # some pointer frames, not all

    for seed in (1, 2):
        rng = np.random.default_rng(seed)
        ctx = binding.SaliContext(lib_config(p))
        s_imgs = [torch.cuda.Stream() for _ in range(3)]
        s_kv = torch.cuda.Stream()
        torch.cuda.synchronize()
        analysed = stored = 0
        b = 0
        while stored < n:
            # keep the analysis between 1 and 16 frames ahead of the store
            while analysed < n and analysed - stored < 9:
                size = int(min(rng.integers(1, 9), n - analysed))
                ctx.analyze_batch([rgbs[t % n_src] for t in range(analysed, analysed + size)], analysed, s_imgs[b % 3])
                analysed += size
                b += 1
            size = int(min(rng.integers(1, 9), analysed - stored))
            ctx.store_batch([kvs[t % n_src] for t in range(stored, stored + size)], stored, s_kv)
            stored += size
        torch.cuda.synchronize()
        print(f"schedule {seed}: {b} analysis batches", flush=True)
        assert ctx.get_status() == 0
        rows = [r.as_tuple() for r in ctx.read_frame_table(0, n)]
        assert rows == ref_rows
        for t in range(n):
            if ref_rows[t][2]:
                a, c = ctx.read_frame_tiers(t), ref.read_frame_tiers(t)
                assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1]), f"tiers of frame {t}"
        pools = ctx.pool_views()
        used = {"fp16": sum(r[6] for r in ref_rows if r[2]), "codes8": sum(r[7] for r in ref_rows if r[2]),
                "codes4": sum(r[8] for r in ref_rows if r[2])}
        used.update(scale8=used["codes8"], scale4=used["codes4"], zero4=used["codes4"])
        for k in ref_pools:                  # rows behind the cursors are unwritten memory
            assert torch.equal(pools[k][:, :used[k]], ref_pools[k][:, :used[k]]), f"pool {k}"
        ctx.close()
    ref.close()
