"""Oracle: saliency map (Canny edges + LAB colour variance) and patch pooling.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Follows Spatial Filtering via Saliency-Guided Quantization (saliency map
S in [0,1]^{HxW}, Eq. 7) and Implementation Details (Canny edge detection
combined with adaptive thresholding on the local colour variance in LAB).
The paper gives no filter sizes, thresholds or combination rule; the readings
taken, all in integer arithmetic so that scores are exact on any machine:

  gray      Y8 = (77 R + 150 G + 29 B + 128) >> 8
  Canny     5x5 binomial blur (>> 8 with rounding) -> 3x3 Sobel -> squared magnitude ->
            non-maximum suppression with exact direction tests (tan 22.5 deg = sqrt2 - 1)
            and an asymmetric tie rule (> first neighbour, >= second) -> double threshold
            lo = 50, hi = 100 on the magnitude -> 8-connected hysteresis.  E in {0, 1}.
  colour    sRGB -> linear (12 bit LUT) -> white-normalised XYZ (12-bit matrix, rows sum
            to 4096) -> cube-root LUT -> 8-bit L, a, b; 5x5 window N = 25 sum v^2 - (sum v)^2
            per channel, V = N_L + N_a + N_b; C = 1 iff V * H*W > sum of V over the frame
            (above the frame mean: the adaptive threshold) and V >= 10000.
  map       S = (E + C) / 2
  pooling   Eq. 7 over the proportional patch partition; q_i = sum of (E + C) in patch i,
            score_i = floor(q_i * 2^15 / |P_i|) / 65536   (an exact fp32 value)

All stencils replicate the border, except that non-maximum suppression treats
out-of-image neighbours as magnitude 0.
"""
from __future__ import annotations

import numpy as np
from scipy import ndimage

CANNY_LO = 50
CANNY_HI = 100
V_MIN = 10000
BINOMIAL5 = np.array([1, 4, 6, 4, 1], dtype=np.int64)


# ---------------------------------------------------------------------------
# patch partition (shared by flow pooling and saliency pooling)
# ---------------------------------------------------------------------------
def patch_edges(size, grid=24):
    """Row (or column) boundaries: patch r covers [floor(r*size/grid), floor((r+1)*size/grid))."""
    return np.array([(r * size) // grid for r in range(grid + 1)], dtype=np.int64)


# ---------------------------------------------------------------------------
# gray and Canny
# ---------------------------------------------------------------------------
def gray_y8(rgb):
    rgb = np.asarray(rgb)
    if rgb.dtype != np.uint8 or rgb.ndim != 3 or rgb.shape[2] != 3:
        raise TypeError("uint8 HxWx3 expected")
    r = rgb[:, :, 0].astype(np.int64)
    g = rgb[:, :, 1].astype(np.int64)
    b = rgb[:, :, 2].astype(np.int64)
    return ((77 * r + 150 * g + 29 * b + 128) >> 8).astype(np.uint8)


def _shift(a, dy, dx):
    """a[clamp(y + dy), clamp(x + dx)] (replicate border)."""
    h, w = a.shape
    ys = np.clip(np.arange(h) + dy, 0, h - 1)
    xs = np.clip(np.arange(w) + dx, 0, w - 1)
    return a[np.ix_(ys, xs)]


def blur5(y8):
    y = y8.astype(np.int64)
    acc = np.zeros_like(y)
    for a in range(-2, 3):
        for b in range(-2, 3):
            acc += BINOMIAL5[a + 2] * BINOMIAL5[b + 2] * _shift(y, a, b)
    return ((acc + 128) >> 8).astype(np.uint8)


def sobel(bl):
    b = bl.astype(np.int64)
    gx = (_shift(b, -1, 1) + 2 * _shift(b, 0, 1) + _shift(b, 1, 1)) \
        - (_shift(b, -1, -1) + 2 * _shift(b, 0, -1) + _shift(b, 1, -1))
    gy = (_shift(b, 1, -1) + 2 * _shift(b, 1, 0) + _shift(b, 1, 1)) \
        - (_shift(b, -1, -1) + 2 * _shift(b, -1, 0) + _shift(b, -1, 1))
    return gx, gy


def _shift_zero(a, dy, dx):
    """a[y + dy, x + dx], 0 outside the image."""
    h, w = a.shape
    p = np.zeros((h + 2, w + 2), dtype=a.dtype)
    p[1:-1, 1:-1] = a
    return p[1 + dy:1 + dy + h, 1 + dx:1 + dx + w]


def nms(gx, gy):
    """Boolean mask of pixels that survive non-maximum suppression, and m2 = gx^2 + gy^2."""
    m2 = gx * gx + gy * gy
    s = np.abs(gx) + np.abs(gy)
    s2 = s * s
    is_h = s2 < 2 * gx * gx            # |gy| < (sqrt2 - 1)|gx|: gradient along x
    is_v = s2 < 2 * gy * gy
    is_d = (~is_h) & (~is_v) & (gx * gy > 0)
    first = np.where(is_h, _shift_zero(m2, 0, -1),
            np.where(is_v, _shift_zero(m2, -1, 0),
            np.where(is_d, _shift_zero(m2, -1, -1), _shift_zero(m2, -1, 1))))
    second = np.where(is_h, _shift_zero(m2, 0, 1),
             np.where(is_v, _shift_zero(m2, 1, 0),
             np.where(is_d, _shift_zero(m2, 1, 1), _shift_zero(m2, 1, -1))))
    keep = (m2 > first) & (m2 >= second)
    return keep, m2


def classify(keep, m2, lo=CANNY_LO, hi=CANNY_HI):
    """0 = none, 1 = weak, 2 = strong."""
    cls = np.zeros(m2.shape, dtype=np.uint8)
    cls[keep & (m2 >= lo * lo)] = 1
    cls[keep & (m2 >= hi * hi)] = 2
    return cls


def hysteresis(cls):
    """Strong pixels plus weak pixels 8-connected to a strong one through weak/strong pixels."""
    cand = cls > 0
    lab, n = ndimage.label(cand, structure=np.ones((3, 3), dtype=bool))
    has_strong = np.zeros(n + 1, dtype=bool)
    has_strong[np.unique(lab[cls == 2])] = True
    has_strong[0] = False
    return (has_strong[lab] & cand).astype(np.uint8)


def canny(rgb, lo=CANNY_LO, hi=CANNY_HI):
    gx, gy = sobel(blur5(gray_y8(rgb)))
    keep, m2 = nms(gx, gy)
    return hysteresis(classify(keep, m2, lo, hi))


# ---------------------------------------------------------------------------
# 8-bit LAB
# ---------------------------------------------------------------------------
def _check_not_near_half(v):
    frac = v - np.floor(v)
    if np.any(np.abs(frac - 0.5) < 1e-9):
        raise AssertionError("table entry on a rounding boundary")


def lin_table():
    c = np.arange(256, dtype=np.float64) / 255.0
    lin = np.where(c <= 0.04045, c / 12.92, ((c + 0.055) / 1.055) ** 2.4)
    v = 4095.0 * lin
    _check_not_near_half(v)
    return np.floor(v + 0.5).astype(np.int64)


def fl_table():
    u = np.arange(4096, dtype=np.float64) / 4095.0
    d = 6.0 / 29.0
    f = np.where(u > d ** 3, np.cbrt(u), u / (3 * d * d) + 4.0 / 29.0)
    v = 32768.0 * f
    _check_not_near_half(v)
    return np.floor(v + 0.5).astype(np.int64)


XYZ_ROWS = np.array([[1777, 1541, 778], [871, 2929, 296], [73, 448, 3575]], dtype=np.int64)


def lab8(rgb):
    """-> L8, a8, b8 as int64 arrays in [0, 255]."""
    lin = lin_table()
    fl = fl_table()
    r = lin[rgb[:, :, 0]]
    g = lin[rgb[:, :, 1]]
    b = lin[rgb[:, :, 2]]
    t = [(XYZ_ROWS[k, 0] * r + XYZ_ROWS[k, 1] * g + XYZ_ROWS[k, 2] * b + 2048) >> 12 for k in range(3)]
    fx, fy, fz = fl[t[0]], fl[t[1]], fl[t[2]]
    num = (116 * fy - 524288) * 255 + 1638400
    assert (num >= 0).all()
    l8 = np.clip(num // 3276800, 0, 255)
    a8 = np.clip((500 * (fx - fy) + 4194304 + 16384) >> 15, 0, 255)     # arithmetic shift = floor
    b8 = np.clip((200 * (fy - fz) + 4194304 + 16384) >> 15, 0, 255)
    return l8, a8, b8


def colour_variance(rgb):
    """V = sum over L, a, b of 25 * sum(v^2) - (sum v)^2 in the 5x5 window (replicate border)."""
    total = np.zeros(rgb.shape[:2], dtype=np.int64)
    for ch in lab8(rgb):
        s1 = np.zeros_like(ch)
        s2 = np.zeros_like(ch)
        for dy in range(-2, 3):
            for dx in range(-2, 3):
                v = _shift(ch, dy, dx)
                s1 += v
                s2 += v * v
        total += 25 * s2 - s1 * s1
    return total


def colour_mask(v, v_min=V_MIN):
    h, w = v.shape
    m = int(v.sum())
    return ((v * (h * w) > m) & (v >= v_min)).astype(np.uint8)


# ---------------------------------------------------------------------------
# map and pooling
# ---------------------------------------------------------------------------
def saliency_map2(rgb, lo=CANNY_LO, hi=CANNY_HI, v_min=V_MIN):
    """S2 = E + C in {0, 1, 2}; the saliency map of the paper is S = S2 / 2."""
    return (canny(rgb, lo, hi) + colour_mask(colour_variance(rgb), v_min)).astype(np.uint8)


def pool(s2, grid=24):
    """Eq. 7 -> (scores fp32 [grid*grid], q int64 [grid*grid], area int64 [grid*grid])."""
    h, w = s2.shape
    ye, xe = patch_edges(h, grid), patch_edges(w, grid)
    q = np.zeros(grid * grid, dtype=np.int64)
    area = np.zeros(grid * grid, dtype=np.int64)
    for r in range(grid):
        for c in range(grid):
            blk = s2[ye[r]:ye[r + 1], xe[c]:xe[c + 1]]
            q[r * grid + c] = int(blk.astype(np.int64).sum())
            area[r * grid + c] = blk.size
    s_fix = (q * 32768) // area
    scores = (s_fix.astype(np.float64) / 65536.0).astype(np.float32)    # exact: s_fix <= 2^16
    return scores, q, area


def saliency_pool(rgb, grid=24, lo=CANNY_LO, hi=CANNY_HI, v_min=V_MIN):
    """-> (scores fp32 [grid*grid], S2 uint8 [H, W])."""
    s2 = saliency_map2(rgb, lo, hi, v_min)
    scores, _, _ = pool(s2, grid)
    return scores, s2
