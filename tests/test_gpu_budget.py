"""GPU parity of the memory-budget mode (whole frames evicted oldest first, ring-shaped pools) against
the oracle, through the C ABI: frame-table rows of every frame after every step, pool rows and
dequantised contents of the frames still held, evicted frames reading as no data."""
import math

import numpy as np
import pytest
import torch

from oracle.attention import attend_decode
from oracle.cache import SaliCacheOracle
from paper_2602_14236_amd import synth

from _util import assert_same, lib_config, oracle_config, params, workload_params

pytestmark = pytest.mark.gpu


def _check_rows(ctx, orc, n):
    rows = ctx.read_frame_table(0, n)
    for f in range(n):
        exp = orc.rows[f].as_tuple() if f in orc.rows else None
        if exp is not None:
            assert rows[f].as_tuple() == exp, f"row {f}: {rows[f].as_tuple()} vs {exp}"


def _check_contents(ctx, orc, n, expect_no_data_bit=True):
    """Every frame so far: held frames (and pointer entries to them) read back bit-identically, the
    others as zeros; pool rows of the held frames equal the oracle's."""
    from paper_2602_14236_amd import binding
    c = ctx.cfg
    out = torch.empty((c.n_layers, 2, c.n_heads, 576, 128), dtype=torch.float16, device="cuda")
    valid = torch.empty(576, dtype=torch.uint8, device="cuda")
    flat = ctx.pool_views_flat()
    P = ctx.n_planes
    shp = (c.n_layers, 2, c.n_heads)
    any_dead = False
    for f in range(n):
        if f not in orc.rows:
            continue
        r = orc.rows[f]
        out.fill_(1.0)
        ctx.kv_decompress(f, out, valid)
        torch.cuda.synchronize()
        if r.src < 0:
            any_dead = True
            assert not out.any() and not valid.any(), f"frame {f} holds no data"
            continue
        exp, exp_valid = orc.kv_decompress(f)
        assert_same(out.cpu().numpy(), exp, f"decompressed frame {f}")
        assert_same(valid.cpu().numpy(), exp_valid, f"valid mask {f}")
        if r.stored:
            for name, ref, base, cnt in (("fp16", orc.pool16, r.base16, r.n16), ("codes8", orc.codes8, r.base8, r.n8),
                                         ("scale8", orc.scale8, r.base8, r.n8), ("codes4", orc.codes4, r.base4, r.n4),
                                         ("scale4", orc.scale4, r.base4, r.n4), ("zero4", orc.zero4, r.base4, r.n4)):
                if cnt == 0:
                    continue
                got = flat[name][base * P:(base + cnt) * P].view(P, cnt, -1).cpu().numpy().reshape(shp + (cnt, -1))
                assert_same(got, ref[..., base:base + cnt, :], f"frame {f} {name} rows")
    status = ctx.get_status()
    assert status & ~binding.FAULT_NO_DATA == 0, status
    if expect_no_data_bit and any_dead:
        assert status & binding.FAULT_NO_DATA


def test_budget_kv_compress_random_sequence():
    """sali_kv_compress with varying tier mixes into small ring pools under a budget of 1000 tokens."""
    from paper_2602_14236_amd import binding
    n = 36
    p = params(n_layers=1, n_heads=2, cap_fp16=700, cap_int8=650, cap_int4=600, max_frames=n, budget_tokens=1000)
    ctx = binding.SaliContext(lib_config(p))
    orc = SaliCacheOracle(oracle_config(p))
    rng = np.random.default_rng(7)
    g = torch.Generator(device="cuda").manual_seed(3)
    for f in range(n):
        scores = (rng.integers(0, int(rng.integers(8, 40)), 576) / 64.0).astype(np.float32)
        kv = (torch.randn((1, 2, 2, 576, 128), generator=g, device="cuda") * 1.5).to(torch.float16)
        ctx.kv_compress(kv, torch.from_numpy(scores).cuda(), f)
        orc.kv_compress(kv.cpu().numpy(), scores, f)
        _check_rows(ctx, orc, f + 1)
        if f % 6 == 5 or f == n - 1:
            print(f"frame {f}: held {orc.table.held}", flush=True)
            _check_contents(ctx, orc, f + 1)
    assert len(orc.table.held) < n and not orc.overflow
    # ids must increase in this mode; a budget below one frame is refused
    with pytest.raises(binding.SaliError) as e:
        ctx.kv_compress(kv, torch.from_numpy(scores).cuda(), 5)
    assert e.value.code == -5
    with pytest.raises(binding.SaliError) as e:
        binding.workspace_bytes(lib_config(params(budget_tokens=500)))
    assert e.value.code == -4
    ctx.close()


def test_budget_with_adaptive_thresholds():
    """The two optional modes together: thresholds that follow the score quantiles decide how many tokens a
    frame keeps, the budget decides how many frames stay."""
    from paper_2602_14236_amd import binding
    n = 24
    p = params(n_layers=1, n_heads=1, cap_fp16=600, cap_int8=600, cap_int4=600, max_frames=n, budget_tokens=900,
               tier_mode=2, k_fp16=60, k_int8=90, k_int4=120, adapt_rate_q8=160)
    ctx = binding.SaliContext(lib_config(p))
    orc = SaliCacheOracle(oracle_config(p))
    rng = np.random.default_rng(17)
    g = torch.Generator(device="cuda").manual_seed(4)
    for f in range(n):
        scores = (rng.integers(0, 65537, 576) / 65536.0 * rng.uniform(0.2, 1.0)).astype(np.float32)
        kv = torch.randn((1, 2, 1, 576, 128), generator=g, device="cuda").to(torch.float16)
        ctx.kv_compress(kv, torch.from_numpy(scores).cuda(), f)
        orc.kv_compress(kv.cpu().numpy(), scores, f)
        _check_rows(ctx, orc, f + 1)
    print(f"held {orc.table.held}, thresholds {orc.table.adapt_tau}", flush=True)
    assert 1 <= len(orc.table.held) < n
    _check_contents(ctx, orc, n)
    ctx.close()


def test_budget_wrap_and_oversized_frame():
    """Frames that keep 200 fp16 tokens in a pool of 500 rows: two fit, every further one evicts the oldest
    and goes to row 0 or behind the cursor in turn; then a frame whose rows no empty pool can hold."""
    from paper_2602_14236_amd import binding
    p = params(tier_mode=1, k_fp16=200, k_int8=0, k_int4=0, n_layers=1, n_heads=1, cap_fp16=500, cap_int8=8,
               cap_int4=8, max_frames=8, budget_tokens=5000)
    ctx = binding.SaliContext(lib_config(p))
    orc = SaliCacheOracle(oracle_config(p))
    g = torch.Generator(device="cuda").manual_seed(5)
    scores = torch.rand(576, generator=torch.Generator().manual_seed(1))
    for f in range(5):
        kv = torch.randn((1, 2, 1, 576, 128), generator=g, device="cuda").to(torch.float16)
        ctx.kv_compress(kv, scores.cuda(), f)
        orc.kv_compress(kv.cpu().numpy(), scores.numpy(), f)
    assert [orc.rows[f].base16 for f in range(5) if orc.rows[f].stored] == [200, 0]      # frames 3 and 4 (the ring has wrapped twice)
    assert [orc.rows[f].stored for f in range(5)] == [0, 0, 0, 1, 1]
    _check_rows(ctx, orc, 5)
    _check_contents(ctx, orc, 5)
    ctx.set_tier_params(1, k_fp16=501, k_int8=0, k_int4=0)
    orc.cfg.k_fp16 = 501
    kv = torch.randn((1, 2, 1, 576, 128), generator=g, device="cuda").to(torch.float16)
    ctx.kv_compress(kv, scores.cuda(), 5)
    orc.kv_compress(kv.cpu().numpy(), scores.numpy(), 5)
    assert orc.overflow and orc.table.held == []
    _check_rows(ctx, orc, 6)
    assert ctx.get_status() & binding.FAULT_OVERFLOW
    ctx.close()


def _run_config5(budget, n, batched):
    from paper_2602_14236_amd import binding
    wl = synth.WORKLOADS[5]
    v = synth.video(5, 32)
    nl, nh = 1, 2
    p = workload_params(wl, frames=n, n_layers=nl, n_heads=nh, cap_fp16=900, cap_int8=900, cap_int4=900,
                        budget_tokens=budget)
    ctx = binding.SaliContext(lib_config(p))
    scale = synth.kv_channel_scale(wl, nl, nh)
    kvs = [synth.kv_frame(wl, t, device="cuda", n_layers=nl, n_heads=nh, scale=scale) for t in range(n)]
    rgbs = [torch.from_numpy(v.frame(t)).cuda() for t in range(n)]
    if batched:
        for lo in range(0, n, 4):
            ctx.step_batch(rgbs[lo:lo + 4], kvs[lo:lo + 4], lo)
    else:
        for t in range(n):
            ctx.step(rgbs[t], kvs[t], t)
    torch.cuda.synchronize()
    return ctx, p, v, kvs


def test_budget_784_patches_chained_step_with_pointer_frames():
    """The paper's budget of 784 patches on the adversarial workload's first 14 frames (duplicates 5..8 are
    pointer entries): sali_step frame by frame and sali_step_batch four at a time against the oracle; the
    final cache state is the same in both (a frame evicted by a later frame of its own batch is simply
    never written)."""
    n = 14
    ctx, p, v, kvs = _run_config5(784, n, batched=False)
    orc = SaliCacheOracle(oracle_config(p))
    for t in range(n):
        orc.step(v.frame(t), kvs[t].cpu().numpy(), t)
    held = orc.table.held
    print(f"held at the end: {held}; rows {[orc.rows[t].as_tuple()[:3] for t in range(n)]}", flush=True)
    assert len(held) >= 1 and held[-1] == max(t for t in range(n) if orc.rows[t].stored)
    assert sum(orc.rows[g].n16 + orc.rows[g].n8 + orc.rows[g].n4 for g in held) <= 784
    assert any(orc.rows[t].stored == 0 and orc.rows[t].src == -1 for t in range(5, 9)) or orc.rows[8].src >= 0
    _check_rows(ctx, orc, n)
    _check_contents(ctx, orc, n)
    # attention over the whole range reads only what is still held
    q = torch.randn((2, 128), generator=torch.Generator().manual_seed(2)).to(torch.float16).cuda()
    out = torch.empty((2, 128), dtype=torch.float32, device="cuda")
    lse = torch.empty(2, dtype=torch.float32, device="cuda")
    sm = 1.0 / math.sqrt(128.0)
    ctx.attend_decode(0, q, 0, n, sm, out, lse)
    torch.cuda.synchronize()
    exp_out, exp_lse = attend_decode(orc, 0, q.cpu().numpy(), 0, n, sm)
    assert np.all(np.abs(out.cpu().numpy() - exp_out) <= 1e-4 + 1e-3 * np.abs(exp_out))
    assert np.all(np.abs(lse.cpu().numpy() - exp_lse) <= 1e-4 + 1e-3 * np.abs(exp_lse))
    ctx.close()
    ctx2, _, _, _ = _run_config5(784, n, batched=True)
    _check_rows(ctx2, orc, n)
    _check_contents(ctx2, orc, n)
    ctx2.close()
