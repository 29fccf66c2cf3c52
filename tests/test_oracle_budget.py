"""Pins of the oracle's memory-budget mode (CPU only).

Reading pinned (Experimental Setup names a strict budget of 784 patches and no eviction rule): whole
frames are evicted oldest first until the new frame's kept tokens fit the budget and its rows fit the
ring-shaped pools; evicted frames and the pointer entries that referred to them hold no data."""
import numpy as np
import pytest

from oracle import quant as oq
from oracle.cache import OracleConfig, SaliCacheOracle, _FrameTable


def _cfg(**kw):
    base = dict(src_h=96, src_w=96, n_layers=1, n_heads=1, cap_fp16=2000, cap_int8=2000, cap_int4=2000, max_frames=64)
    base.update(kw)
    return OracleConfig(**base)


def _kv(seed):
    return (np.random.default_rng(seed).standard_normal((1, 2, 1, 576, 128)) * 1.5).astype(np.float16)


def _held(table):
    return [f for f, r in sorted(table.rows.items()) if r.stored]


def test_ring_placement_worked_example():
    """A pool of 10 rows, frames of 4 rows each (traced by hand): bases 0, 4; the third does not fit
    behind row 8, and row 0 is free only once frame 0 is gone; the fourth finds the cursor at 4 blocked
    by frame 1, whose eviction frees it."""
    t = _FrameTable(_cfg(cap_fp16=10, cap_int8=10, cap_int4=10, budget_tokens=1000))
    cnt = (4, 0, 0, 572)
    assert t.store(0, cnt).as_tuple()[:7] == (0, 0, 1, 0, 0, 0, 4)
    assert t.store(1, cnt).base16 == 4 and _held(t) == [0, 1]
    r2 = t.store(2, cnt)
    assert (r2.base16, r2.stored) == (0, 1) and _held(t) == [1, 2] and t.rows[0].as_tuple()[:3] == (0, -1, 0)
    r3 = t.store(3, cnt)
    assert r3.base16 == 4 and _held(t) == [2, 3]
    r4 = t.store(4, (6, 0, 0, 570))           # 6 rows: behind row 8 no room, row 0..5 needs frames 2 and 3 gone
    assert r4.base16 == 0 and _held(t) == [4]
    assert not t.overflow
    r5 = t.store(5, (11, 0, 0, 565))          # larger than the pool: cannot be held at all
    assert r5.stored == 0 and r5.src == -1 and t.overflow and _held(t) == []


def test_token_budget_closed_form():
    """Top-k tiers keep k tokens per frame: with roomy pools exactly floor(budget / k) newest frames are held."""
    for budget, k in ((784, 576), (1200, 576), (2000, 300), (576, 576)):
        cfg = _cfg(tier_mode=1, k_fp16=k // 3, k_int8=k // 3, k_int4=k - 2 * (k // 3), budget_tokens=budget,
                   cap_fp16=3000, cap_int8=3000, cap_int4=3000)
        t = _FrameTable(cfg)
        for f in range(12):
            t.store(f, (cfg.k_fp16, cfg.k_int8, cfg.k_int4, 576 - k))
            held = _held(t)
            assert held == list(range(max(0, f + 1 - budget // k), f + 1)), (budget, k, f, held)
            assert sum(t.rows[g].n16 + t.rows[g].n8 + t.rows[g].n4 for g in held) <= budget


def test_budget_invariants_and_contents_random_sequence():
    """Random tier mixes, pointer frames, small pools: after every frame the held frames are the newest
    stored ones, within budget, with pairwise disjoint row runs inside the pools; pointer entries follow
    their source out of the cache; and every held frame reads back exactly what a cache without budget
    (large pools) returns for it."""
    rng = np.random.default_rng(7)
    budget = 1000
    cfg = _cfg(budget_tokens=budget, cap_fp16=700, cap_int8=650, cap_int4=600)
    ref_cfg = _cfg(cap_fp16=20000, cap_int8=20000, cap_int4=20000)
    o, ref = SaliCacheOracle(cfg), SaliCacheOracle(ref_cfg)
    stored_order = []
    for f in range(40):
        if f > 0 and rng.random() < 0.25:                 # a redundant frame: pointer entry
            o.table.pointer(f)
            ref.table.pointer(f)
        else:
            # thresholds 0.30 / 0.15 / 0.03 on coarse scores: every tier populated, counts vary per frame
            scores = (rng.integers(0, int(rng.integers(8, 40)), 576) / 64.0).astype(np.float32)
            kv = _kv(100 + f)
            row = o.kv_compress(kv, scores, f)
            ref.kv_compress(kv, scores, f)
            assert row.stored == 1
            stored_order.append(f)
        held = _held(o.table)
        assert held == o.table.held and held == stored_order[len(stored_order) - len(held):]      # newest, FIFO
        assert sum(o.rows[g].n16 + o.rows[g].n8 + o.rows[g].n4 for g in held) <= budget
        assert stored_order[-1] in held
        for pool, cap in enumerate((cfg.cap_fp16, cfg.cap_int8, cfg.cap_int4)):
            runs = sorted(((o.rows[g].base16, o.rows[g].base8, o.rows[g].base4)[pool],
                           (o.rows[g].n16, o.rows[g].n8, o.rows[g].n4)[pool]) for g in held)
            runs = [r for r in runs if r[1] > 0]
            assert all(b >= 0 and b + n <= cap for b, n in runs)
            assert all(runs[i][0] + runs[i][1] <= runs[i + 1][0] for i in range(len(runs) - 1))
        for g in range(f + 1):
            r, rr = o.rows[g], ref.rows[g]
            if rr.stored:
                assert r.stored == (1 if g in held else 0)
            else:                                          # pointer entry: alive iff its source is
                assert r.stored == 0 and r.src == (rr.src if rr.src in held else -1)
            if r.src >= 0:
                got, gv = o.kv_decompress(g)
                exp, ev = ref.kv_decompress(g)
                assert np.array_equal(got.view(np.uint16), exp.view(np.uint16)) and np.array_equal(gv, ev)
            else:
                with pytest.raises(KeyError):
                    o.kv_decompress(g)
    assert len(_held(o.table)) < len(stored_order)         # something was evicted
    assert not o.overflow


def test_without_budget_nothing_changes():
    cfg = _cfg(cap_fp16=700, cap_int8=700, cap_int4=700)
    o = SaliCacheOracle(cfg)
    scores = np.linspace(0, 1, 576).astype(np.float32)
    assert o.kv_compress(_kv(1), scores, 0).stored == 1
    tier = oq.tiers_threshold(scores, 0.30, 0.15, 0.03)
    assert o.kv_compress(_kv(2), scores, 1).stored == (1 if 2 * np.bincount(tier, minlength=4)[:3].max() <= 700 else 0)
    assert o.table.held == []
