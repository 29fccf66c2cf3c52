"""GPU parity of dynamic-resolution frames (several images of 576 patches per video frame, one reuse
decision per frame, one cache entry per tile) against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle.cache import SaliCacheOracle, step_tiles
from paper_2602_14236_amd import synth

from _util import FLOW_ATOL, FLOW_RTOL, assert_same, close, drift_frame, lib_config, oracle_config, params, pool_arrays

pytestmark = pytest.mark.gpu


def _compare(ctx, orc, n_entries):
    rows = ctx.read_frame_table(0, n_entries)
    for e in range(n_entries):
        assert rows[e].as_tuple() == orc.rows[e].as_tuple(), f"row {e}: {rows[e].as_tuple()} vs {orc.rows[e].as_tuple()}"
        if orc.rows[e].stored:
            tier, slot = ctx.read_frame_tiers(e)
            assert_same(tier, orc.tier[e], f"tier {e}")
            assert_same(slot.astype(np.int32), orc.slot[e], f"slot {e}")
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
    for e in range(n_entries):
        if orc.rows[e].src < 0:
            continue
        ctx.kv_decompress(e, out)
        torch.cuda.synchronize()
        assert_same(out.cpu().numpy(), orc.kv_decompress(e)[0], f"decompressed entry {e}")
    assert ctx.get_status() == 0


def _check_gate(ctx, orc, T, t):
    if orc.last_gate is None:
        return
    n, r, red, margin = orc.last_gate
    tau = ctx.cfg.tau_t
    fragile = 0
    for j in range(T):
        dp, gate, _ = ctx.read_analysis(t * T + j)
        assert close(dp, orc.last_dp[j]).all(), f"frame {t} tile {j}: Delta P out of tolerance"
        fragile += int(np.count_nonzero(np.abs(orc.last_dp[j] - tau) <= FLOW_ATOL + FLOW_RTOL * tau))
        assert abs(gate.n_static - n) <= fragile + 576 * T * 0, (gate.n_static, n)
    assert fragile == 0 and (gate.n_static, gate.r_frame, gate.redundant) == (n, float(r), int(red)), \
        f"frame {t}: gate {(gate.n_static, gate.r_frame, gate.redundant)} vs {(n, float(r), int(red))}"


@pytest.mark.parametrize("adaptive", [False, True])
def test_two_tiles_joint_decision_drift_sequence(adaptive):
    """The sequence of the oracle's pin: frame 1 has a static and a moving tile (stored whole), frames 2 and
    3 are redundant (pointer entries per tile), frame 4 is stored again.  One video frame per call.
    adaptive: with thresholds that follow the score quantiles, moved after every stored entry (tile)."""
    from paper_2602_14236_amd import binding
    T = 2
    extra = dict(tier_mode=2, k_fp16=100, k_int8=150, k_int4=200, adapt_rate_q8=96) if adaptive else {}
    p = params(96, 96, flow_levels=2, n_layers=1, n_heads=1, cap_fp16=6000, cap_int8=6000, cap_int4=6000, max_frames=16,
               tiles_per_frame=T, **extra)
    ctx = binding.SaliContext(lib_config(p))
    orc = SaliCacheOracle(oracle_config(p))
    seq = [(0.0, 5.0), (0.0, 7.0), (0.0, 7.0), (0.3, 7.3), (3.0, 7.3)]
    g = torch.Generator().manual_seed(1)
    for t, shifts in enumerate(seq):
        rgbs = [drift_frame(s) for s in shifts]
        kvs = [torch.randn((1, 2, 1, 576, 128), generator=g).to(torch.float16) for _ in range(T)]
        ctx.step_batch([torch.from_numpy(r).cuda() for r in rgbs], [k.cuda() for k in kvs], t * T)
        step_tiles(orc, rgbs, [k.numpy() for k in kvs], t)
        _check_gate(ctx, orc, T, t)
    assert [orc.rows[e].stored for e in range(10)] == [1, 1, 1, 1, 0, 0, 0, 0, 1, 1]
    if adaptive:
        print("thresholds at the end:", orc.table.adapt_tau, [orc.rows[e].as_tuple()[6:10] for e in (0, 1, 8, 9)], flush=True)
        assert orc.rows[0].as_tuple()[6:10] != orc.rows[9].as_tuple()[6:10]      # the thresholds did move
    assert [orc.rows[e].src for e in range(10)] == [0, 1, 2, 3, 2, 3, 2, 3, 8, 9]
    _compare(ctx, orc, 10)
    # whole frames only
    x = torch.from_numpy(drift_frame(0.0)).cuda()
    with pytest.raises(binding.SaliError) as e:
        ctx.analyze_batch([x], 10)
    assert e.value.code == -2
    with pytest.raises(binding.SaliError) as e:
        ctx.analyze_batch([x, x], 11)
    assert e.value.code == -2
    with pytest.raises(binding.SaliError) as e:
        binding.workspace_bytes(lib_config(params(tiles_per_frame=2, budget_tokens=784)))
    assert e.value.code == -4
    ctx.close()


def test_four_tiles_two_frames_per_call_workload_video():
    """Four tiles per frame cut from consecutive frames of the 336x336 workload video (tile j of frame t is
    video frame 4 t' + j of a strided pick, so tiles move differently), two video frames per call (eight
    entries: the second frame's predecessor entries are in the same launch), top-k tiers per tile, 2 heads."""
    from paper_2602_14236_amd import binding
    T, n_frames = 4, 6
    wl = synth.WORKLOADS[1]
    v = synth.video(1, 8)
    p = params(336, 336, tier_mode=1, k_fp16=120, k_int8=200, k_int4=150, n_layers=1, n_heads=2, cap_fp16=120 * 24,
               cap_int8=200 * 24, cap_int4=150 * 24, max_frames=T * n_frames, tiles_per_frame=T)
    ctx = binding.SaliContext(lib_config(p))
    orc = SaliCacheOracle(oracle_config(p))
    # tile j of frame t shows video frame pick[t][j]: frames 2 and 3 of the video are identical, so tiles
    # that show them in consecutive frames are static while the others move
    pick = [(0, 1, 2, 4), (1, 2, 3, 5), (1, 2, 3, 5), (1, 2, 3, 5), (2, 3, 3, 6), (2, 3, 3, 6)]
    g = torch.Generator(device="cuda").manual_seed(9)
    for t0 in range(0, n_frames, 2):
        rgbs, kvs = [], []
        for t in (t0, t0 + 1):
            for j in range(T):
                rgbs.append(v.frame(pick[t][j]))
                kvs.append((torch.randn((1, 2, 2, 576, 128), generator=g, device="cuda") * 1.2).to(torch.float16))
        print(f"frames {t0}, {t0 + 1}", flush=True)
        ctx.step_batch([torch.from_numpy(r).cuda() for r in rgbs], kvs, t0 * T)
        for k, t in enumerate((t0, t0 + 1)):
            step_tiles(orc, rgbs[k * T:(k + 1) * T], [x.cpu().numpy() for x in kvs[k * T:(k + 1) * T]], t)
            _check_gate(ctx, orc, T, t)
    stored = [orc.rows[t * T].stored for t in range(n_frames)]
    print("stored per frame:", stored, flush=True)
    assert stored == [1, 1, 0, 0, 1, 0]
    _compare(ctx, orc, T * n_frames)
    ctx.close()
