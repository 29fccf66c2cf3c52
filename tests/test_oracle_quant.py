"""Pins of the quantisation / tiering oracle (CPU only).

Each test fixes a property that follows from the stated operation sequence or from plain
arithmetic, chosen so that a dropped term, a wrong rounding mode, a swapped nibble or an
off-by-one in the ranks fails at least one of them.
"""
import os

import numpy as np
import pytest

from oracle import quant as oq

RNG = np.random.default_rng(12345)


def _rand_fp16(shape, scale=1.0):
    return (RNG.standard_normal(shape) * scale).astype(np.float16)


# ---- round trip within scale/2 ---------------------------------------------------------------
@pytest.mark.parametrize("scale", [1e-3, 1.0, 300.0])
def test_int8_roundtrip_error_bound(scale):
    x = _rand_fp16((64, 128), scale)
    q, s = oq.quant_int8(x)
    xg = x.astype(np.float64).reshape(64, 4, 32)
    xh32 = q.reshape(64, 4, 32).astype(np.float64) * s[..., None].astype(np.float64)
    # rounding of inv, of x*inv (|x*inv| <= 127) and of scale each move the result by at most
    # 127 * 2^-24 code units: |x - q*scale| <= scale * (1/2 + 3 * 127 * 2^-24) < scale * (1/2 + 2^-15)
    bound = s[..., None].astype(np.float64) * (0.5 + 2.0 ** -15)
    assert np.all(np.abs(xg - xh32) <= bound + 1e-30)
    xh16 = oq.dequant_int8(q, s).astype(np.float64).reshape(64, 4, 32)
    assert np.all(np.abs(xg - xh16) <= bound + 2.0 ** -11 * np.abs(xh32) + 2.0 ** -25)


@pytest.mark.parametrize("scale", [1e-3, 1.0, 300.0])
def test_int4_roundtrip_error_bound(scale):
    x = _rand_fp16((64, 128), scale)
    q, s, z = oq.quant_int4(x)
    xg = x.astype(np.float64).reshape(64, 4, 32)
    xh = q.reshape(64, 4, 32).astype(np.float64) * s[..., None].astype(np.float64) + z[..., None].astype(np.float64)
    bound = s[..., None].astype(np.float64) * (0.5 + 2.0 ** -15)        # as for int8, codes <= 15
    assert np.all(np.abs(xg - xh) <= bound + 1e-30)
    xh16 = oq.dequant_int4(q, s, z).astype(np.float64).reshape(64, 4, 32)
    assert np.all(np.abs(xg - xh16) <= bound + 2.0 ** -11 * np.abs(xh) + 2.0 ** -25)


# ---- extreme codes, zero-point, scale definition ------------------------------------------------
def test_int8_extremes_and_scale_value():
    x = _rand_fp16((32, 128))
    q, s = oq.quant_int8(x)
    xg = x.astype(np.float32).reshape(32, 4, 32)
    qg = q.reshape(32, 4, 32)
    m = np.abs(xg).max(-1)
    assert np.array_equal(s, (m / np.float32(127)).astype(np.float32))
    arg = np.abs(xg).argmax(-1)
    top = np.take_along_axis(qg, arg[..., None], -1)[..., 0]
    assert np.all(np.abs(top) == 127)
    assert qg.min() >= -127 and qg.max() <= 127


def test_int4_extremes_and_zero_point():
    x = _rand_fp16((32, 128))
    q, s, z = oq.quant_int4(x)
    xg = x.reshape(32, 4, 32)
    qg = q.reshape(32, 4, 32)
    assert np.array_equal(z, xg.min(-1))
    assert np.all(np.take_along_axis(qg, xg.argmin(-1)[..., None], -1) == 0)
    assert np.all(np.take_along_axis(qg, xg.argmax(-1)[..., None], -1) == 15)
    rng32 = xg.max(-1).astype(np.float32) - xg.min(-1).astype(np.float32)
    assert np.array_equal(s, (rng32 / np.float32(15)).astype(np.float32))


def test_int8_negation_negates_codes():
    x = _rand_fp16((16, 128))
    q1, s1 = oq.quant_int8(x)
    q2, s2 = oq.quant_int8(-x)
    assert np.array_equal(q2, -q1) and np.array_equal(s1, s2)


@pytest.mark.parametrize("k", [-6, -1, 3, 5])
def test_power_of_two_scaling_leaves_codes(k):
    # x * 2^k is exact in fp16 as long as nothing leaves the normal range
    x = (RNG.uniform(0.25, 4.0, (16, 128)) * RNG.choice([-1, 1], (16, 128))).astype(np.float16)
    y = (x.astype(np.float32) * np.float32(2.0 ** k)).astype(np.float16)
    assert np.array_equal(y.astype(np.float32), x.astype(np.float32) * np.float32(2.0 ** k))
    q1, s1 = oq.quant_int8(x)
    q2, s2 = oq.quant_int8(y)
    assert np.array_equal(q1, q2)
    assert np.array_equal(s2, s1 * np.float32(2.0 ** k))
    p1, t1, z1 = oq.quant_int4(x)
    p2, t2, z2 = oq.quant_int4(y)
    assert np.array_equal(p1, p2)
    assert np.array_equal(t2, t1 * np.float32(2.0 ** k))
    assert np.array_equal(z2.astype(np.float32), z1.astype(np.float32) * np.float32(2.0 ** k))


def test_round_half_to_even_is_used():
    # group max 127 => inv = 1 exactly, so x*inv = x; halves must go to the even neighbour
    x = np.zeros((1, 32), dtype=np.float16)
    x[0, 0] = 127.0
    x[0, 1:7] = [0.5, 1.5, 2.5, -0.5, -1.5, -2.5]
    q, s = oq.quant_int8(x)
    assert s[0, 0] == np.float32(1.0)
    assert q[0, :7].tolist() == [127, 0, 2, 2, 0, -2, -2]
    # int4: min 0, max 15 => inv = 1
    y = np.zeros((1, 32), dtype=np.float16)
    y[0, 0] = 15.0
    y[0, 1:5] = [0.5, 1.5, 2.5, 3.5]
    p, t, z = oq.quant_int4(y)
    assert p[0, :5].tolist() == [15, 0, 2, 2, 4] and z[0, 0] == 0


def test_constant_and_zero_groups():
    x = np.full((2, 128), 3.25, dtype=np.float16)
    p, t, z = oq.quant_int4(x)
    assert not p.any() and not t.any() and np.all(z == np.float16(3.25))
    assert np.array_equal(oq.dequant_int4(p, t, z), x)
    zero = np.zeros((2, 128), dtype=np.float16)
    q, s = oq.quant_int8(zero)
    assert not q.any() and not s.any()
    assert np.array_equal(oq.dequant_int8(q, s), zero)


def test_fp16_subnormal_inputs_stay_finite():
    x = np.zeros((1, 32), dtype=np.float16)
    x[0, 0] = np.float16(6e-8)          # smallest fp16 subnormal
    x[0, 1] = -np.float16(6e-8)
    q, s = oq.quant_int8(x)
    assert np.isfinite(s).all() and s[0, 0] > 0
    assert q[0, 0] == 127 and q[0, 1] == -127
    p, t, z = oq.quant_int4(x)
    assert p[0, 0] == 15 and p[0, 1] == 0 and np.isfinite(t).all()


def test_fma_dequant_is_single_rounding():
    # find a case where fl(fl(q*scale) + zero) differs from the fused result, and check we return the fused one
    rng = np.random.default_rng(7)
    found = 0
    for _ in range(4000):
        x = (rng.standard_normal((1, 32)) * 3).astype(np.float16)
        q, s, z = oq.quant_int4(x)
        prod = (q.astype(np.float32) * s[0, 0]).astype(np.float32)
        two_step = (prod + z[0, 0].astype(np.float32)).astype(np.float32)
        exact = q.astype(np.float64) * float(s[0, 0]) + float(z[0, 0])
        fused = exact.astype(np.float32)
        if not np.array_equal(two_step, fused):
            found += 1
        assert np.array_equal(oq.dequant_int4(q, s, z), fused.astype(np.float16))
    assert found > 0        # the distinction is real, so the test above can fail


def test_nibble_order_and_roundtrip():
    c = np.arange(32, dtype=np.uint8).reshape(1, 32) % 16
    p = oq.pack_nibbles(c)
    assert p.shape == (1, 16)
    assert p[0, 0] == (c[0, 0] | (c[0, 1] << 4))        # element 0 low nibble, element 1 high nibble
    assert p[0, 3] == 0x76
    assert np.array_equal(oq.unpack_nibbles(p), c)


# ---- tiers -----------------------------------------------------------------------------------------
def test_threshold_tiers_inequalities_as_printed():
    s = np.array([0.31, 0.30, 0.299, 0.15, 0.151, 0.03, 0.031, 0.0], dtype=np.float32)
    t = oq.tiers_threshold(s, 0.30, 0.15, 0.03)
    #            >hi   =hi     (med,hi]  =med   (med,hi] =low    (low,med] <=low
    assert t.tolist() == [0, 1, 1, 2, 1, 3, 2, 3]


def test_topk_matches_bruteforce_rank_definition():
    rng = np.random.default_rng(3)
    for n, ks in [(12, (3, 4, 2)), (40, (0, 17, 5)), (576, (173, 403, 0)), (576, (249, 56, 168))]:
        s = (rng.integers(0, 9, n) / 8.0).astype(np.float32)           # many ties
        t = oq.tiers_topk(s, *ks)
        rank = np.array([sum(1 for j in range(n) if s[j] > s[i] or (s[j] == s[i] and j < i)) for i in range(n)])
        exp = np.full(n, 3)
        exp[rank < ks[0] + ks[1] + ks[2]] = 2
        exp[rank < ks[0] + ks[1]] = 1
        exp[rank < ks[0]] = 0
        assert np.array_equal(t, exp)
        assert np.bincount(t, minlength=4).tolist() == [ks[0], ks[1], ks[2], n - sum(ks)]


def test_slots_are_stable_ranks_within_tier():
    rng = np.random.default_rng(4)
    tier = rng.integers(0, 4, 576).astype(np.uint8)
    slot, cnt = oq.slots(tier)
    assert cnt.sum() == 576
    for t in range(4):
        idx = np.nonzero(tier == t)[0]
        assert np.array_equal(slot[idx], np.arange(idx.size))
        assert cnt[t] == idx.size


def test_nan_score_is_an_error():
    s = np.zeros(576, dtype=np.float32)
    s[5] = np.nan
    with pytest.raises(ValueError):
        oq.tiers_topk(s, 1, 1, 1)
    with pytest.raises(ValueError):
        oq.tiers_threshold(s, 0.3, 0.15, 0.03)


# ---- byte accounting -----------------------------------------------------------------------------
def test_compressed_bytes_closed_form_and_paper_mix():
    assert oq.compressed_bytes_per_plane(1, 0, 0) == 256
    assert oq.compressed_bytes_per_plane(0, 1, 0) == 144       # 128 codes + 4 fp32 scales
    assert oq.compressed_bytes_per_plane(0, 0, 1) == 88        # 64 codes + 4 scales + 4 fp16 zeros
    # the tier shares the paper prints (Compression Analysis) give a ratio of the same order as its 2.20x
    g = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            g[line[0]] = float(line[1])
    kept = g["share_fp16"] + g["share_int8"] * 144 / 256 + g["share_int4"] * 88 / 256
    ratio = 100.0 / kept
    assert 0.8 * g["compression_reported"] < ratio < 1.2 * g["compression_reported"]
