"""Pins of the saliency oracle (CPU only): brute force on 8x8 images with naive loops written
here from the stage definitions, the CIE L*a*b* closed form, and hand-checkable edge cases."""
import math

import numpy as np
import pytest

from oracle import saliency as osal


# ---------------------------------------------------------------------------
# a second, naive implementation: scalar loops, no shared helpers
# ---------------------------------------------------------------------------
def _clampi(v, lo, hi):
    return lo if v < lo else hi if v > hi else v


def _srgb_lin(c):
    return c / 12.92 if c <= 0.04045 else ((c + 0.055) / 1.055) ** 2.4


def _labf(u):
    d = 6.0 / 29.0
    return u ** (1.0 / 3.0) if u > d ** 3 else u / (3 * d * d) + 4.0 / 29.0


def brute_s2(rgb, lo, hi, v_min):
    h, w, _ = rgb.shape
    px = [[tuple(int(c) for c in rgb[y, x]) for x in range(w)] for y in range(h)]
    y8 = [[(77 * r + 150 * g + 29 * b + 128) >> 8 for (r, g, b) in row] for row in px]
    k = [1, 4, 6, 4, 1]
    bl = [[0] * w for _ in range(h)]
    for y in range(h):
        for x in range(w):
            acc = 0
            for a in range(-2, 3):
                for b in range(-2, 3):
                    acc += k[a + 2] * k[b + 2] * y8[_clampi(y + a, 0, h - 1)][_clampi(x + b, 0, w - 1)]
            bl[y][x] = (acc + 128) >> 8
    B = lambda yy, xx: bl[_clampi(yy, 0, h - 1)][_clampi(xx, 0, w - 1)]
    gx = [[0] * w for _ in range(h)]
    gy = [[0] * w for _ in range(h)]
    m2 = [[0] * w for _ in range(h)]
    for y in range(h):
        for x in range(w):
            gx[y][x] = (B(y - 1, x + 1) + 2 * B(y, x + 1) + B(y + 1, x + 1)) - (B(y - 1, x - 1) + 2 * B(y, x - 1) + B(y + 1, x - 1))
            gy[y][x] = (B(y + 1, x - 1) + 2 * B(y + 1, x) + B(y + 1, x + 1)) - (B(y - 1, x - 1) + 2 * B(y - 1, x) + B(y - 1, x + 1))
            m2[y][x] = gx[y][x] ** 2 + gy[y][x] ** 2
    M = lambda yy, xx: m2[yy][xx] if 0 <= yy < h and 0 <= xx < w else 0
    cls = [[0] * w for _ in range(h)]
    for y in range(h):
        for x in range(w):
            ax, ay = abs(gx[y][x]), abs(gy[y][x])
            # direction by angle: within 22.5 degrees of the x axis, of the y axis, else a diagonal
            if ay < (math.sqrt(2) - 1) * ax:
                n1, n2 = M(y, x - 1), M(y, x + 1)
            elif ax < (math.sqrt(2) - 1) * ay:
                n1, n2 = M(y - 1, x), M(y + 1, x)
            elif gx[y][x] * gy[y][x] > 0:
                n1, n2 = M(y - 1, x - 1), M(y + 1, x + 1)
            else:
                n1, n2 = M(y - 1, x + 1), M(y + 1, x - 1)
            if m2[y][x] > n1 and m2[y][x] >= n2:
                if m2[y][x] >= hi * hi:
                    cls[y][x] = 2
                elif m2[y][x] >= lo * lo:
                    cls[y][x] = 1
    edge = [[1 if cls[y][x] == 2 else 0 for x in range(w)] for y in range(h)]
    stack = [(y, x) for y in range(h) for x in range(w) if cls[y][x] == 2]
    while stack:
        y, x = stack.pop()
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                yy, xx = y + dy, x + dx
                if 0 <= yy < h and 0 <= xx < w and cls[yy][xx] == 1 and not edge[yy][xx]:
                    edge[yy][xx] = 1
                    stack.append((yy, xx))
    # 8-bit LAB from the float definition of the tables
    lin = [int(math.floor(4095 * _srgb_lin(v / 255.0) + 0.5)) for v in range(256)]
    fl = [int(math.floor(32768 * _labf(t / 4095.0) + 0.5)) for t in range(4096)]
    lab = [[None] * w for _ in range(h)]
    for y in range(h):
        for x in range(w):
            r, g, b = (lin[c] for c in px[y][x])
            tx = (1777 * r + 1541 * g + 778 * b + 2048) // 4096
            ty = (871 * r + 2929 * g + 296 * b + 2048) // 4096
            tz = (73 * r + 448 * g + 3575 * b + 2048) // 4096
            L = _clampi(((116 * fl[ty] - 524288) * 255 + 1638400) // 3276800, 0, 255)
            A = _clampi((500 * (fl[tx] - fl[ty]) + 4194304 + 16384) // 32768, 0, 255)     # floor division
            Bb = _clampi((200 * (fl[ty] - fl[tz]) + 4194304 + 16384) // 32768, 0, 255)
            lab[y][x] = (L, A, Bb)
    var = [[0] * w for _ in range(h)]
    total = 0
    for y in range(h):
        for x in range(w):
            v = 0
            for c in range(3):
                vals = [lab[_clampi(y + a, 0, h - 1)][_clampi(x + b, 0, w - 1)][c] for a in range(-2, 3) for b in range(-2, 3)]
                v += 25 * sum(t * t for t in vals) - sum(vals) ** 2
            var[y][x] = v
            total += v
    out = np.zeros((h, w), dtype=np.uint8)
    for y in range(h):
        for x in range(w):
            c = 1 if (var[y][x] * h * w > total and var[y][x] >= v_min) else 0
            out[y, x] = edge[y][x] + c
    return out


def _blocky(rng, h, w):
    img = np.zeros((h, w, 3), dtype=np.uint8)
    img[:] = rng.integers(0, 256, 3)
    for _ in range(3):
        y0, x0 = rng.integers(0, h - 1), rng.integers(0, w - 1)
        y1, x1 = rng.integers(y0 + 1, h + 1), rng.integers(x0 + 1, w + 1)
        img[y0:y1, x0:x1] = rng.integers(0, 256, 3)
    noise = rng.integers(-6, 7, img.shape)
    return np.clip(img.astype(np.int64) + noise, 0, 255).astype(np.uint8)


@pytest.mark.parametrize("seed", range(12))
def test_bruteforce_8x8(seed):
    rng = np.random.default_rng(100 + seed)
    rgb = _blocky(rng, 8, 8) if seed % 3 else rng.integers(0, 256, (8, 8, 3), dtype=np.uint8)
    lo, hi = ((50, 100), (20, 60), (5, 300))[seed % 3]
    got = osal.saliency_map2(rgb, lo, hi, 10000)
    assert np.array_equal(got, brute_s2(rgb, lo, hi, 10000))


@pytest.mark.parametrize("seed", range(3))
def test_bruteforce_nonsquare(seed):
    rng = np.random.default_rng(200 + seed)
    rgb = _blocky(rng, 11, 17)
    got = osal.saliency_map2(rgb, 30, 80, 2000)
    exp = brute_s2(rgb, 30, 80, 2000)
    assert np.array_equal(got, exp)
    assert exp.any()        # the case is not vacuous


# ---------------------------------------------------------------------------
# closed forms and special cases
# ---------------------------------------------------------------------------
def test_constant_image_has_zero_saliency():
    rgb = np.full((48, 48, 3), 93, dtype=np.uint8)
    scores, s2 = osal.saliency_pool(rgb)
    assert not s2.any() and not scores.any()


def test_gray_pixels_have_neutral_chroma_and_lab_extremes():
    v = np.arange(256, dtype=np.uint8)
    rgb = np.stack([v, v, v], axis=-1)[None, :, :]
    l8, a8, b8 = osal.lab8(rgb)
    assert np.all(a8 == 128) and np.all(b8 == 128)
    assert l8[0, 0] == 0 and l8[0, 255] == 255
    assert np.all(np.diff(l8[0]) >= 0)


def test_lab8_within_one_level_of_cie_formula():
    rng = np.random.default_rng(5)
    rgb = rng.integers(0, 256, (64, 64, 3), dtype=np.uint8)
    l8, a8, b8 = osal.lab8(rgb)
    m = np.array([[0.4124564, 0.3575761, 0.1804375], [0.2126729, 0.7151522, 0.0721750], [0.0193339, 0.1191920, 0.9503041]])
    white = np.array([0.95047, 1.0, 1.08883])
    c = rgb.astype(np.float64) / 255.0
    lin = np.where(c <= 0.04045, c / 12.92, ((c + 0.055) / 1.055) ** 2.4)
    xyz = lin @ m.T / white
    d = 6.0 / 29.0
    f = np.where(xyz > d ** 3, np.cbrt(xyz), xyz / (3 * d * d) + 4.0 / 29.0)
    L = (116 * f[..., 1] - 16) * 255 / 100
    A = 500 * (f[..., 0] - f[..., 1]) + 128
    B = 200 * (f[..., 1] - f[..., 2]) + 128
    assert np.max(np.abs(l8 - L)) <= 1.0
    assert np.max(np.abs(a8 - np.clip(A, 0, 255))) <= 1.0
    assert np.max(np.abs(b8 - np.clip(B, 0, 255))) <= 1.0


def test_tables_shape_and_ends():
    lin, fl = osal.lin_table(), osal.fl_table()
    assert lin[0] == 0 and lin[255] == 4095 and np.all(np.diff(lin) >= 0)
    assert fl[4095] == 32768 and fl[0] == round(32768 * 4 / 29) and np.all(np.diff(fl) >= 0)
    assert XYZ_rows_sum()


def XYZ_rows_sum():
    return np.all(osal.XYZ_ROWS.sum(axis=1) == 4096)


def test_vertical_step_gives_one_edge_column():
    rgb = np.zeros((40, 40, 3), dtype=np.uint8)
    rgb[:, :20] = 60
    rgb[:, 20:] = 160                      # step of 100 >> 25
    e = osal.canny(rgb)
    cols = np.nonzero(e.any(axis=0))[0]
    assert cols.size == 1                   # a single-pixel line
    # blurred profile is symmetric about the step, so columns 19 and 20 tie; the tie rule
    # (> left neighbour, >= right neighbour) keeps the left one
    assert cols[0] == 19
    assert e[:, 19].all()


def test_weak_only_contour_is_dropped_and_chain_with_one_strong_pixel_is_kept():
    cls = np.zeros((9, 12), dtype=np.uint8)
    cls[2, 1:10] = 1                        # weak chain, no strong pixel
    cls[6, 1:10] = 1                        # weak chain ...
    cls[7, 10] = 2                          # ... touching one strong pixel diagonally
    e = osal.hysteresis(cls)
    assert not e[2].any()
    assert e[6, 1:10].all() and e[7, 10] == 1
    assert e.sum() == 10


def test_step_below_weak_threshold_has_no_edges():
    rgb = np.zeros((32, 32, 3), dtype=np.uint8)
    rgb[:, :16] = 100
    rgb[:, 16:] = 110                       # |g| = 4 * 10 = 40 < lo = 50
    assert not osal.canny(rgb).any()


def test_uniform_variance_gives_empty_colour_mask():
    v = np.full((24, 24), 12345, dtype=np.int64)
    assert not osal.colour_mask(v).any()    # strict '>' against the frame mean
    v[3, 3] += 1
    m = osal.colour_mask(v)
    assert m.sum() == 1 and m[3, 3] == 1
    v2 = np.full((24, 24), 50, dtype=np.int64)
    v2[0, 0] = 9999
    assert not osal.colour_mask(v2).any()   # above the mean but under the floor V_min


def test_variance_of_two_level_window_closed_form():
    # L-only pattern: left half gray 50, right half gray 200; at a pixel whose window holds
    # k columns of one and 5-k of the other: N = 25*sum v^2 - (sum v)^2 = 25*k*(5-k)*(dL)^2
    rgb = np.zeros((20, 20, 3), dtype=np.uint8)
    rgb[:, :10] = 50
    rgb[:, 10:] = 200
    l8, a8, b8 = osal.lab8(rgb)
    dl = int(l8[0, 19] - l8[0, 0])
    v = osal.colour_variance(rgb)
    assert v[10, 2] == 0
    assert v[10, 8] == 25 * (5 * 1) * (5 * 4) * dl * dl // 25     # 5 px of one column differ: n1 = 5, n0 = 20
    assert v[10, 9] == 10 * 15 * dl * dl


def test_pooling_partition_and_scores():
    for h, w in [(336, 336), (360, 640), (1080, 1920), (50, 77)]:
        ye, xe = osal.patch_edges(h), osal.patch_edges(w)
        assert ye[0] == 0 and ye[-1] == h and xe[-1] == w
        assert (np.diff(ye) > 0).all() and (np.diff(xe) > 0).all()
        assert np.diff(ye).sum() * np.diff(xe).sum() == h * w
    assert set(np.diff(osal.patch_edges(336))) == {14}             # the paper's 14 x 14 patches
    s2 = np.zeros((336, 336), dtype=np.uint8)
    s2[0:14, 14:28] = 2                                             # patch 1 fully salient
    s2[14:28, 0:7] = 1                                              # patch 24: half the pixels at S = 1/2
    scores, q, area = osal.pool(s2)
    assert scores[1] == 1.0 and scores[24] == 0.25 and scores[0] == 0.0
    assert np.all(q <= 2 * area) and area.sum() == 336 * 336
    assert scores.dtype == np.float32
