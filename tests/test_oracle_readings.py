"""Pins of three readings the other oracle tests leave open (CPU only).

1. The luma weights of the temporal filter's gray conversion act on colour: every other flow pin
   feeds R = G = B images, for which any weights that sum to 256 give the same gray.
2. The frame a new frame is compared with after a redundant frame: the temporal filter takes the
   optical flow between *adjacent* frames (Temporal Filtering via Optical Flow), so the reference is
   frame t-1 even when t-1 was itself redundant, while the cache entry points at the last *stored*
   frame (Algorithm 1).  A slow drift separates the two readings.
3. The oracle's non-finite flag."""
import numpy as np

from oracle import flow as of
from oracle import saliency as osal
from oracle.cache import OracleConfig, SaliCacheOracle

from _util import DRIFT_SHIFTS, drift_frame as _drift_frame


# ---- 1. gray weights ---------------------------------------------------------------------------
def test_gray_of_primaries_and_white():
    px = np.array([[[255, 0, 0], [0, 255, 0], [0, 0, 255], [255, 255, 255], [0, 0, 0]]], dtype=np.uint8)
    g = of.gray_float(px) * 255.0
    # 77 * 255 + 128 = 19763 -> 77;  150 * 255 + 128 = 38378 -> 149;  29 * 255 + 128 = 7523 -> 29
    assert np.array_equal(np.rint(g).astype(int)[0], [77, 149, 29, 255, 0])
    assert np.all(g == np.rint(g))                       # an 8-bit gray, divided by 255


def test_gray_is_the_broadcast_luma_to_one_level():
    """The integer weights are the 8-bit form of the ITU-R BT.601 luma 0.299 R + 0.587 G + 0.114 B:
    on random colours the two agree to one level (swapped or permuted weights miss by dozens)."""
    rng = np.random.default_rng(5)
    rgb = rng.integers(0, 256, (40, 50, 3), dtype=np.uint8)
    y = 0.299 * rgb[..., 0] + 0.587 * rgb[..., 1] + 0.114 * rgb[..., 2]
    g = of.gray_float(rgb) * 255.0
    assert np.abs(g - y).max() <= 1.0
    # the spatial filter's gray is the same image
    assert np.array_equal(np.rint(g).astype(np.uint8), osal.gray_y8(rgb))


def test_red_texture_has_2_7_times_the_gray_contrast_of_blue_texture():
    """What the flow sees of a texture that lives in one colour channel only: red weighs 77 / 256,
    blue 29 / 256, so the same texture has 77 / 29 = 2.66 times the gray contrast in red."""
    h = w = 72
    yy, xx = np.meshgrid(np.arange(h, dtype=np.float64), np.arange(w, dtype=np.float64), indexing="ij")
    tex = 128 + 100 * np.sin(0.5 * xx + 0.2 * yy) * np.sin(0.45 * yy - 0.1 * xx)

    def frame(channel):
        f = np.full((h, w, 3), 128.0)
        f[..., channel] = tex
        return np.clip(np.rint(f), 0, 255).astype(np.uint8)

    g_red, g_green, g_blue = (of.gray_float(frame(c)) for c in range(3))
    span = lambda g: float(g.max() - g.min())
    assert 2.5 < span(g_red) / span(g_blue) < 2.8
    assert 1.85 < span(g_green) / span(g_red) < 2.05          # 150 / 77 = 1.95


# ---- 2. reference frame after a redundant frame -------------------------------------------------
def _drift_oracle():
    o = SaliCacheOracle(OracleConfig(src_h=96, src_w=96, flow_levels=2, tau_t=0.5, theta_r=0.90, n_layers=1,
                                     n_heads=1, cap_fp16=4000, cap_int8=4000, cap_int4=4000, max_frames=8))
    rng = np.random.default_rng(3)
    rows, gates = [], []
    for t, s in enumerate(DRIFT_SHIFTS):
        kv = rng.standard_normal((1, 2, 1, 576, 128)).astype(np.float16)
        rows.append(o.step(_drift_frame(s), kv, t))
        gates.append(o.last_gate)
    return o, rows, gates


def test_slow_drift_is_measured_against_the_adjacent_frame():
    o, rows, gates = _drift_oracle()
    # 0.3 px per frame stays under tau_t = 0.5 against the adjacent frame: frames 1, 2, 3 are pointers
    # to frame 0 although frame 3 has drifted 0.9 px from it; the 1.5 px jump of frame 4 is stored
    assert [r.stored for r in rows] == [1, 0, 0, 0, 1]
    assert [r.src for r in rows] == [0, 0, 0, 0, 4]
    for g in gates[1:4]:
        assert g[0] >= 560 and g[2]                      # nearly every patch static
    assert gates[4][0] <= 16 and not gates[4][2]
    # the per-patch motion of the last redundant frame is the adjacent-frame drift, not the drift
    # accumulated since the stored frame
    d_adj = of.patch_motion(of.flow(_drift_frame(0.6), _drift_frame(0.9), 2, 3))
    assert abs(np.median(d_adj) - 0.3) < 0.05
    # the other reading would decide differently: measured against the last stored frame, frame 2
    # (0.6 px) is already over the threshold
    d_far, dp_far, gate_far = o.flow_score(_drift_frame(0.0), _drift_frame(0.6))
    assert abs(np.median(dp_far) - 0.6) < 0.05
    assert gate_far[0] <= 57 and not gate_far[2]
    # and the pointer rows hold no pool rows of their own
    assert o.cursor == [rows[0].n16 + rows[4].n16, rows[0].n8 + rows[4].n8, rows[0].n4 + rows[4].n4]


# ---- 3. non-finite flag --------------------------------------------------------------------------
def test_nonfinite_flag_only_for_kept_tokens():
    cfg = OracleConfig(src_h=96, src_w=96, tier_mode=1, k_fp16=10, k_int8=10, k_int4=10, n_layers=1, n_heads=1,
                       cap_fp16=100, cap_int8=100, cap_int4=100, max_frames=4)
    scores = np.linspace(1.0, 0.0, 576).astype(np.float32)         # tokens 0..29 kept, the rest pruned
    kv = np.random.default_rng(0).standard_normal((1, 2, 1, 576, 128)).astype(np.float16)
    o = SaliCacheOracle(cfg)
    o.kv_compress(kv, scores, 0)
    assert not o.nonfinite
    bad = kv.copy()
    bad[0, 1, 0, 400, 7] = np.float16(np.inf)                      # a pruned token: never read
    o.kv_compress(bad, scores, 1)
    assert not o.nonfinite
    for tok, val in ((3, np.inf), (15, -np.inf), (25, np.nan)):    # one kept token of each tier
        o2 = SaliCacheOracle(cfg)
        bad = kv.copy()
        bad[0, 0, 0, tok, 100] = np.float16(val)
        o2.kv_compress(bad, scores, 0)
        assert o2.nonfinite, tok
