"""Brute-force pin of the whole flow oracle on a tiny textured image pair (CPU only).

A second implementation of the method's steps (Implementation Details: Farneback's algorithm with a
0.5-scale pyramid; Temporal Filtering via Optical Flow), written pixel by pixel with scalar loops
and different numerical routes from `oracle/flow.py`: the pyramid as an explicit 5x5 sum, the
polynomial expansion of every pixel as its own weighted least-squares problem solved with `lstsq`
on the 49x6 design matrix (the oracle solves normal equations for all pixels at once), the
aggregation as a direct two-dimensional 11x11 window sum of 2x2 matrix products (the oracle blurs
five scalar fields separably), the update as `np.linalg.solve` of the 2x2 system (the oracle uses
Cramer's rule), bilinear sampling and level transfer as scalar code.  Both are float64, so they
must agree to rounding on any input; a dropped term, a swapped axis, a wrong clamp or sign in the
oracle shows up here."""
import math

import numpy as np

from oracle import flow as oflow


def _clamp(v, lo, hi):
    return lo if v < lo else (hi if v > hi else v)


def _texture(h, w, seed, shift=(0.0, 0.0)):
    """Smooth random texture (sum of a few sinusoids) evaluated analytically, optionally shifted."""
    rng = np.random.default_rng(seed)
    waves = [(rng.uniform(0.15, 0.6), rng.uniform(0.15, 0.6), rng.uniform(0, 2 * math.pi), rng.uniform(0.1, 0.25))
             for _ in range(5)]
    img = np.zeros((h, w))
    for y in range(h):
        for x in range(w):
            yy, xx = y - shift[1], x - shift[0]
            img[y, x] = 0.5 + sum(a * math.sin(fx * xx + fy * yy + ph) for fx, fy, ph, a in waves)
    return img


def _down(f):
    h, w = f.shape
    k = [1 / 16, 4 / 16, 6 / 16, 4 / 16, 1 / 16]
    out = np.zeros(((h + 1) // 2, (w + 1) // 2))
    for y in range(out.shape[0]):
        for x in range(out.shape[1]):
            acc = 0.0
            for a in range(-2, 3):
                for b in range(-2, 3):
                    acc += k[a + 2] * k[b + 2] * f[_clamp(2 * y + a, 0, h - 1), _clamp(2 * x + b, 0, w - 1)]
            out[y, x] = acc
    return out


def _expand_pixel(f, y, x):
    """Weighted least squares of one pixel: returns (A 2x2, b 2)."""
    h, w = f.shape
    g = [math.exp(-(k * k) / (2.0 * 1.5 * 1.5)) for k in range(-3, 4)]
    gs = sum(g)
    rows, rhs = [], []
    for dy in range(-3, 4):
        for dx in range(-3, 4):
            wgt = math.sqrt(g[dy + 3] / gs * g[dx + 3] / gs)
            rows.append([wgt, wgt * dx, wgt * dy, wgt * dx * dx, wgt * dy * dy, wgt * dx * dy])
            rhs.append(wgt * f[_clamp(y + dy, 0, h - 1), _clamp(x + dx, 0, w - 1)])
    r = np.linalg.lstsq(np.array(rows), np.array(rhs), rcond=None)[0]
    a = np.array([[r[3], r[5] / 2.0], [r[5] / 2.0, r[4]]])       # [[A_xx, A_xy], [A_xy, A_yy]]
    return a, np.array([r[1], r[2]])


def _expand(f):
    h, w = f.shape
    a = [[None] * w for _ in range(h)]
    b = [[None] * w for _ in range(h)]
    for y in range(h):
        for x in range(w):
            a[y][x], b[y][x] = _expand_pixel(f, y, x)
    return a, b


def _bilinear(grid, h, w, sy, sx):
    """grid[y][x] -> numpy value; coordinates clamped to the image."""
    sy, sx = _clamp(sy, 0.0, h - 1.0), _clamp(sx, 0.0, w - 1.0)
    y0, x0 = int(math.floor(sy)), int(math.floor(sx))
    y1, x1 = min(y0 + 1, h - 1), min(x0 + 1, w - 1)
    fy, fx = sy - y0, sx - x0
    top = grid[y0][x0] * (1 - fx) + grid[y0][x1] * fx
    bot = grid[y1][x0] * (1 - fx) + grid[y1][x1] * fx
    return top * (1 - fy) + bot * fy


def _iterate(a1, b1, a2, b2, prior, h, w):
    """One displacement update; prior[y][x] = np.array([u, v])."""
    g = [math.exp(-(k * k) / (2.0 * 2.5 * 2.5)) for k in range(-5, 6)]
    gs = sum(g)
    # per-pixel normal-equation terms at the warped position
    ata = [[None] * w for _ in range(h)]
    atb = [[None] * w for _ in range(h)]
    for y in range(h):
        for x in range(w):
            d = prior[y][x]
            a2s = _bilinear(a2, h, w, y + d[1], x + d[0])
            b2s = _bilinear(b2, h, w, y + d[1], x + d[0])
            a = 0.5 * (a1[y][x] + a2s)
            db = -0.5 * (b2s - b1[y][x]) + a @ d
            ata[y][x] = a.T @ a
            atb[y][x] = a.T @ db
    out = [[None] * w for _ in range(h)]
    for y in range(h):
        for x in range(w):
            gm = np.zeros((2, 2))
            hv = np.zeros(2)
            for dy in range(-5, 6):
                for dx in range(-5, 6):
                    wgt = g[dy + 5] / gs * g[dx + 5] / gs
                    yy, xx = _clamp(y + dy, 0, h - 1), _clamp(x + dx, 0, w - 1)
                    gm += wgt * ata[yy][xx]
                    hv += wgt * atb[yy][xx]
            lam = 1e-4 + 1e-2 * 0.5 * (gm[0, 0] + gm[1, 1])
            out[y][x] = np.linalg.solve(gm + lam * np.eye(2), hv + lam * prior[y][x])
    return out


def _flow_by_definition(f1, f2, levels, iters):
    p1, p2 = [f1], [f2]
    for _ in range(levels - 1):
        p1.append(_down(p1[-1]))
        p2.append(_down(p2[-1]))
    d = None
    for lvl in range(levels - 1, -1, -1):
        h, w = p1[lvl].shape
        a1, b1 = _expand(p1[lvl])
        a2, b2 = _expand(p2[lvl])
        if d is None:
            prior = [[np.zeros(2) for _ in range(w)] for _ in range(h)]
        else:
            ch, cw = len(d), len(d[0])
            prior = [[2.0 * _bilinear(d, ch, cw, y / 2.0, x / 2.0) for x in range(w)] for y in range(h)]
        for _ in range(iters):
            prior = _iterate(a1, b1, a2, b2, prior, h, w)
        d = prior
    return np.array([[d[y][x] for x in range(len(d[0]))] for y in range(len(d))])


def test_whole_flow_equals_pixel_by_pixel_definition_on_a_tiny_texture():
    h, w = 19, 26                                    # odd height: ragged pyramid level (10 x 13)
    f1 = _texture(h, w, seed=4)
    f2 = _texture(h, w, seed=4, shift=(1.3, -0.7))   # sub-pixel motion, so the bilinear warp matters
    ref = _flow_by_definition(f1, f2, levels=2, iters=2)
    got = oflow.flow_from_gray(f1, f2, levels=2, iters=2)
    assert got.shape == ref.shape == (h, w, 2)
    assert np.abs(got - ref).max() < 1e-9, np.abs(got - ref).max()
    # the pair really moves, and both components are exercised with their own sign
    centre = got[6:13, 8:18].reshape(-1, 2).mean(axis=0)
    assert centre[0] > 0.3 and centre[1] < -0.05


def test_pyramid_and_expansion_equal_their_scalar_definitions():
    f = _texture(11, 14, seed=9)
    assert np.abs(oflow.downsample(f) - _down(f)).max() < 1e-14
    a, b, _ = oflow.poly_expansion(f)
    for (y, x) in ((0, 0), (5, 7), (10, 13), (3, 0), (0, 9)):       # corners, edges (replicated border), interior
        am, bv = _expand_pixel(f, y, x)
        assert np.allclose([a[y, x, 0], a[y, x, 1], a[y, x, 2]], [am[0, 0], am[0, 1], am[1, 1]], rtol=0, atol=1e-12)
        assert np.allclose(b[y, x], bv, rtol=0, atol=1e-12)
