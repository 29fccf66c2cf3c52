"""GPU parity of the adaptive-threshold mode (tier_mode 2: Eq. 8 with thresholds that follow the score
quantiles of the stored frames) against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle.cache import SaliCacheOracle
from paper_2602_14236_amd import synth

from _util import assert_same, lib_config, oracle_config, params, pool_arrays, workload_params

pytestmark = pytest.mark.gpu


def _compare(ctx, orc, frames):
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
    assert_same(pa["codes4"][..., :c4, :], orc.codes4[..., :c4, :], "int4 codes")
    assert ctx.get_status() == 0


@pytest.mark.parametrize("rate", [0, 77, 256])
def test_adaptive_thresholds_kv_compress(rate):
    """Twelve frames of scores from any source (lattice values with ties, arbitrary floats, values outside
    [0, 1], a frame of zeros) through sali_kv_compress: rows, tiers and slots of every frame."""
    from paper_2602_14236_amd import binding
    n = 12
    p = params(tier_mode=2, k_fp16=100, k_int8=150, k_int4=200, adapt_rate_q8=rate, n_layers=1, n_heads=1,
               cap_fp16=576 * n, cap_int8=576 * n, cap_int4=576 * n, max_frames=n)
    ctx = binding.SaliContext(lib_config(p))
    orc = SaliCacheOracle(oracle_config(p))
    rng = np.random.default_rng(rate)
    g = torch.Generator(device="cuda").manual_seed(rate)
    for f in range(n):
        kind = f % 4
        if kind == 0:
            scores = (rng.integers(0, 2000, 576) * 32 / 65536.0).astype(np.float32)        # lattice, many ties
        elif kind == 1:
            scores = rng.uniform(0, 1, 576).astype(np.float32)                              # off the lattice
        elif kind == 2:
            scores = rng.normal(0.3, 0.5, 576).astype(np.float32)                           # some outside [0, 1]
        else:
            scores = np.zeros(576, dtype=np.float32) if f == 3 else rng.uniform(0, 0.05, 576).astype(np.float32)
        kv = torch.randn((1, 2, 1, 576, 128), generator=g, device="cuda").to(torch.float16)
        ctx.kv_compress(kv, torch.from_numpy(scores).cuda(), f)
        orc.kv_compress(kv.cpu().numpy(), scores, f)
        row = ctx.read_frame_table(f, 1)[0]
        assert row.as_tuple() == orc.rows[f].as_tuple(), f"frame {f}: {row.as_tuple()} vs {orc.rows[f].as_tuple()}"
    print(f"rate {rate}: thresholds at the end {orc.table.adapt_tau}, counts {[orc.rows[f].as_tuple()[6:10] for f in range(n)]}",
          flush=True)
    _compare(ctx, orc, range(n))
    ctx.close()


def test_adaptive_thresholds_chained_batches():
    """The 336x336 workload video (8 frames, one duplicate = a pointer frame in the middle of a batch) through
    sali_step_batch in batches of 3, 4 and 1 frames, then frame by frame after a reset: the same rows, tiers
    and pools as the oracle's frame-by-frame walk.  In a batch the frames are ranked in parallel and tiered in
    order by the last block, each with the thresholds its predecessor left."""
    from paper_2602_14236_amd import binding
    wl = synth.WORKLOADS[1]
    v = synth.video(1)
    nl, nh = 1, 2
    p = workload_params(wl, n_layers=nl, n_heads=nh, tier_mode=2, k_fp16=150, k_int8=150, k_int4=150, adapt_rate_q8=96,
                        tau_high=0.5, tau_med=0.25, tau_low=0.05)
    ctx = binding.SaliContext(lib_config(p))
    orc = SaliCacheOracle(oracle_config(p))
    scale = synth.kv_channel_scale(wl, nl, nh)
    kvs = [synth.kv_frame(wl, t, device="cuda", n_layers=nl, n_heads=nh, scale=scale) for t in range(8)]
    rgbs = [torch.from_numpy(v.frame(t)).cuda() for t in range(8)]
    taus = []
    for t in range(8):
        orc.step(v.frame(t), kvs[t].cpu().numpy(), t)
        taus.append(list(orc.table.adapt_tau))
    print("thresholds after each frame:", taus, flush=True)
    assert orc.rows[3].stored == 0 and taus[3] == taus[2] and taus[7] != taus[0]
    for lo, hi in ((0, 3), (3, 7), (7, 8)):
        ctx.step_batch(rgbs[lo:hi], kvs[lo:hi], lo)
    torch.cuda.synchronize()
    _compare(ctx, orc, range(8))
    ctx.reset()
    for t in range(8):
        ctx.step(rgbs[t], kvs[t], t)
    torch.cuda.synchronize()
    _compare(ctx, orc, range(8))
    ctx.close()
