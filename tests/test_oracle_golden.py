"""The image-only walk of Algorithm 1 (oracle.cache.ImageSideOracle) against the full oracle, and the
committed whole-workload records against a fresh evaluation of a few of their frames (CPU only)."""
import os

import numpy as np
import pytest

from oracle.cache import ImageSideOracle, OracleConfig, SaliCacheOracle
from paper_2602_14236_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_image_side_walk_equals_the_full_oracle():
    """Same rows, tiers and slots with and without the K/V tensors: duplicates (pointer rows), a
    moving scene, threshold tiers; then top-k tiers with a pool that overflows."""
    v = synth.video(1, 6)
    frames = [v.frame(0), v.frame(0), v.frame(1), v.frame(2), v.frame(2), v.frame(4)]
    rng = np.random.default_rng(1)
    for kw in (dict(cap_fp16=4000, cap_int8=4000, cap_int4=4000),
               dict(tier_mode=1, k_fp16=100, k_int8=200, k_int4=150, cap_fp16=250, cap_int8=1000, cap_int4=1000)):
        cfg = OracleConfig(src_h=336, src_w=336, n_layers=1, n_heads=1, max_frames=8, **kw)
        full, img = SaliCacheOracle(cfg), ImageSideOracle(cfg)
        for t, f in enumerate(frames):
            kv = rng.standard_normal((1, 2, 1, 576, 128)).astype(np.float16)
            r_full = full.step(f, kv, t)
            r_img, a = img.step(f, t)
            assert r_full.as_tuple() == r_img.as_tuple(), t
            if r_full.stored:
                assert np.array_equal(full.tier[t], a["tier"]) and np.array_equal(full.slot[t], a["slot"])
                assert np.array_equal(full.last_scores, a["scores"])
            if t > 0:
                assert full.last_gate == a["gate"] and np.array_equal(full.last_dp, a["dp"])
        assert full.cursor == img.cursor and full.overflow == img.overflow
    assert img.overflow                      # the second configuration runs out of fp16 rows at the third stored frame


@pytest.mark.parametrize("cfg_id,frames", [(2, (0, 17)), (5, (8, 9, 58, 120)), (3, (40, 1234))])
def test_committed_records_are_what_the_oracle_computes(cfg_id, frames):
    path = os.path.join(GOLDEN, f"image_side_cfg{cfg_id}.npz")
    g = np.load(path)
    wl = synth.WORKLOADS[cfg_id]
    n = g["rows"].shape[0]
    video = synth.video(cfg_id, n)
    orc = ImageSideOracle(OracleConfig(src_h=wl.height, src_w=wl.width, flow_levels=wl.flow_levels, tier_mode=wl.tier_mode,
                                       k_fp16=wl.k_fp16, k_int8=wl.k_int8, k_int4=wl.k_int4))
    for t in frames:
        a = orc.analyze_pair(video.frame(t - 1) if t > 0 else None, video.frame(t), float(g["tau_t"][t]),
                             float(g["theta_r"][t]))
        assert int(a["redundant"]) == int(g["redundant"][t]) == int(g["rows"][t, 2] == 0)
        if a["gate"] is not None:
            assert a["gate"][0] == int(g["n_static"][t])
            assert np.array_equal(a["dp"].astype(np.float32), g["dp"][t])
        if not a["redundant"]:
            assert np.array_equal(a["scores"], g["scores"][t]) and np.array_equal(a["tier"], g["tier"][t])
            assert tuple(int(v) for v in g["rows"][t, 6:10]) == tuple(int(v) for v in a["cnt"])


def test_record_bookkeeping_is_consistent():
    """Rows of every record: bases are the running sums of the stored frames' counts, pointer rows name
    the last stored frame, counts add up to 576."""
    for cfg_id in (2, 3, 4, 5):
        g = np.load(os.path.join(GOLDEN, f"image_side_cfg{cfg_id}.npz"))
        rows = g["rows"]
        base = [0, 0, 0]
        last = -1
        for t, r in enumerate(rows):
            assert r[0] == t
            if r[2] == 1:
                assert (r[1], r[3], r[4], r[5]) == (t, base[0], base[1], base[2]) and r[6:10].sum() == 576
                assert np.array_equal(np.bincount(g["tier"][t], minlength=4), r[6:10])
                base = [base[0] + r[6], base[1] + r[7], base[2] + r[8]]
                last = t
            else:
                assert r[1] == last and g["redundant"][t] == 1 and not r[3:].any()
