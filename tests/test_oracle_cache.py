"""Pins of the chained oracle (Algorithm 1) and of the input generators (CPU only)."""
import numpy as np
import pytest

from oracle import quant as oq
from oracle.cache import OracleConfig, SaliCacheOracle
from paper_2602_14236_amd import synth


def _kv(seed, nl=1, nh=2, n=576, d=128):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((nl, 2, nh, n, d)) * 1.5).astype(np.float16)


def _cfg(**kw):
    base = dict(src_h=96, src_w=96, n_layers=1, n_heads=2, cap_fp16=2000, cap_int8=2000, cap_int4=2000, max_frames=16)
    base.update(kw)
    return OracleConfig(**base)


def test_compress_decompress_layout_and_roundtrip():
    o = SaliCacheOracle(_cfg())
    rng = np.random.default_rng(0)
    scores = (rng.integers(0, 40, 576) / 64.0).astype(np.float32)
    kv = _kv(1)
    row = o.kv_compress(kv, scores, 0)
    tier = oq.tiers_threshold(scores, 0.30, 0.15, 0.03)
    cnt = np.bincount(tier, minlength=4)
    assert row.as_tuple() == (0, 0, 1, 0, 0, 0, cnt[0], cnt[1], cnt[2], cnt[3])
    assert cnt.min() > 0
    out, valid = o.kv_decompress(0)
    assert np.array_equal(valid, (tier != 3).astype(np.uint8))
    assert np.array_equal(out[:, :, :, tier == 0].view(np.uint16), kv[:, :, :, tier == 0].view(np.uint16))  # bitwise
    assert not out[:, :, :, tier == 3].any()
    # int8 / int4 rows obey the error bound through the pools
    q8, s8 = oq.quant_int8(kv[:, :, :, tier == 1])
    err = np.abs(out[:, :, :, tier == 1].astype(np.float64) - kv[:, :, :, tier == 1].astype(np.float64))
    bound = np.repeat(s8, 32, axis=-1).astype(np.float64) * 0.51 + 2.0 ** -10 * np.abs(kv[:, :, :, tier == 1].astype(np.float64))
    assert np.all(err <= bound + 1e-7)
    # a second frame lands behind the first in every pool
    row2 = o.kv_compress(_kv(2), scores, 1)
    assert (row2.base16, row2.base8, row2.base4) == (cnt[0], cnt[1], cnt[2])
    assert o.cursor == [2 * cnt[0], 2 * cnt[1], 2 * cnt[2]]
    # the pool slot of token i is base + (number of earlier tokens of its tier)
    i8 = np.nonzero(tier == 1)[0]
    assert np.array_equal(o.codes8[0, 1, 1, :cnt[1]], q8[0, 1, 1])
    assert np.array_equal(o.codes8[0, 0, 0, 3], oq.quant_int8(kv[0, 0, 0, i8[3]][None])[0][0])


def test_pool_overflow_marks_frame_and_keeps_cursors():
    o = SaliCacheOracle(_cfg(tier_mode=1, k_fp16=100, k_int8=100, k_int4=100, cap_fp16=150, cap_int8=150, cap_int4=150))
    scores = np.linspace(0, 1, 576).astype(np.float32)
    assert o.kv_compress(_kv(3), scores, 0).stored == 1
    row = o.kv_compress(_kv(4), scores, 1)
    assert row.stored == 0 and row.src == -1 and o.overflow and o.cursor == [100, 100, 100]


def test_algorithm1_pointer_chain_and_first_frame():
    v = synth.video(1, 6)
    wl = synth.WORKLOADS[1]
    o = SaliCacheOracle(OracleConfig(src_h=336, src_w=336, n_layers=1, n_heads=1, cap_fp16=4000, cap_int8=4000,
                                     cap_int4=4000, max_frames=8))
    kvs = [_kv(10 + t, 1, 1) for t in range(5)]
    f = [v.frame(0), v.frame(0), v.frame(0), v.frame(1), v.frame(1)]
    rows = [o.step(f[t], kvs[t], t) for t in range(5)]
    # frame 0 is stored although nothing precedes it; byte-identical followers are pointers to it
    assert [r.stored for r in rows] == [1, 0, 0, 1, 0]
    assert [r.src for r in rows] == [0, 0, 0, 3, 3]
    out1, _ = o.kv_decompress(2)
    out0, _ = o.kv_decompress(0)
    assert np.array_equal(out1.view(np.uint16), out0.view(np.uint16))
    assert o.cursor[0] == rows[0].n16 + rows[3].n16


def test_config1_generator_properties():
    v = synth.video(1)
    assert len(v) == 8 and v.frame(0).shape == (336, 336, 3) and v.frame(0).dtype == np.uint8
    assert np.array_equal(v.frame(3), v.frame(2))                 # 1-based frames 3 and 4 are identical
    assert not np.array_equal(v.frame(1), v.frame(2))
    assert np.array_equal(synth.video(1).frame(5), v.frame(5))    # deterministic
    # noise sigma ~ 2 on the static background: difference of two frames has std ~ 2 * sqrt(2) where nothing moves
    d = v.frame(1).astype(np.int64) - v.frame(0).astype(np.int64)
    assert 2.0 < np.median(np.abs(d)) * 1.4826 < 6.0


def test_kv_generator_shape_and_determinism():
    wl = synth.WORKLOADS[1]
    a = synth.kv_frame(wl, 3)
    b = synth.kv_frame(wl, 3)
    assert tuple(a.shape) == (1, 2, 32, 576, 128) and str(a.dtype) == "torch.float16"
    assert bool((a == b).all()) and not bool((a == synth.kv_frame(wl, 4)).all())
    import torch
    assert bool(torch.isfinite(a.float()).all())
    wl5 = synth.WORKLOADS[5]
    c = synth.kv_frame(wl5, 0, n_layers=1).float()
    ch = c.abs().amax(dim=(0, 1, 3))                              # [heads, D]
    assert bool(((ch > 8 * ch.median(dim=1, keepdim=True).values).sum(dim=1) >= 3).all())    # outlier channels


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_other_generators_render(cfg):
    wl = synth.WORKLOADS[cfg]
    v = synth.video(cfg, 3)
    f = v.frame(2)
    assert f.shape == (wl.height, wl.width, 3)
    assert wl.elems_per_token == wl.n_layers * 2 * wl.n_heads * 128
