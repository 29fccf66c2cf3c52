"""Oracle: dense polynomial-expansion optical flow, per-patch motion, redundancy gate.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Follows Temporal Filtering via Optical Flow (Eq. 5, Eq. 6, the redundancy rule
R_frame > theta_R) and Implementation Details (Farneback's algorithm, pyramid
scale 0.5, 3 levels).  Float64 throughout.  The paper fixes nothing beyond the
pyramid; the readings taken:

  gray       Y8 = (77 R + 150 G + 29 B + 128) >> 8, f = Y8 / 255
  pyramid    level l+1 = 5x5 binomial [1 4 6 4 1]/16 filter of level l sampled at even
             positions, size ceil(h/2) x ceil(w/2)
  expansion  f(x + delta) ~ c + b.delta + delta^T A delta by weighted least squares over
             the 7x7 neighbourhood, Gaussian weight sigma = 1.5 (normalised)
  estimate   at each level, K = 3 times:  x~ = x + d~(x); A2, b2 of the new frame sampled
             bilinearly at x~ (coordinates clamped); A = (A1 + A2)/2;
             db = -(b2 - b1)/2 + A d~;  G = w * (A^T A), h = w * (A^T db) with a
             normalised 11x11 Gaussian window sigma = 2.5;
             lambda = 1e-4 + 1e-2 (G11 + G22)/2;  d = (G + lambda I)^-1 (h + lambda d~)
             (lambda = 0 is Farneback's d = G^-1 h; the prior-centred ridge term keeps
             flat regions at their prior and bounds the conditioning)
  transfer   d~_l(y, x) = 2 * bilinear(d_{l+1}; y/2, x/2)
  Eq. 5      Delta P_i = sqrt(mean over patch i of (u^2 + v^2)), the RMS flow magnitude in
             source pixels (the sentence before Eq. 5 and Algorithm 1 both say optical flow)
  Eq. 6      n_static = #{Delta P_i < tau_t} (strict), R = n_static / N_p in fp32,
             redundant iff R > theta_R (strict)

Flow (u, v) at (x, y): the content at (x, y) of the earlier frame appears at
(x + u, y + v) in the later frame.  All stencils replicate the border.
"""
from __future__ import annotations

import numpy as np

POLY_N = 3
POLY_SIGMA = 1.5
WIN_R = 5
WIN_SIGMA = 2.5
ITERS = 3
LAMBDA_ABS = 1e-4
LAMBDA_REL = 1e-2


def gray_float(rgb):
    rgb = np.asarray(rgb)
    r = rgb[:, :, 0].astype(np.int64)
    g = rgb[:, :, 1].astype(np.int64)
    b = rgb[:, :, 2].astype(np.int64)
    y8 = (77 * r + 150 * g + 29 * b + 128) >> 8
    return y8.astype(np.float64) / 255.0


def _take(a, ys, xs):
    """a[clamp(ys), clamp(xs)] on the outer product of two index vectors."""
    h, w = a.shape[:2]
    return a[np.ix_(np.clip(ys, 0, h - 1), np.clip(xs, 0, w - 1))]


def downsample(f):
    h, w = f.shape
    h2, w2 = (h + 1) // 2, (w + 1) // 2
    k = np.array([1.0, 4.0, 6.0, 4.0, 1.0]) / 16.0
    out = np.zeros((h2, w2))
    for a in range(-2, 3):
        for b in range(-2, 3):
            out += k[a + 2] * k[b + 2] * _take(f, 2 * np.arange(h2) + a, 2 * np.arange(w2) + b)
    return out


def pyramid(f, levels):
    pyr = [np.asarray(f, dtype=np.float64)]
    for _ in range(levels - 1):
        pyr.append(downsample(pyr[-1]))
    return pyr


def poly_expansion(f, n=POLY_N, sigma=POLY_SIGMA):
    """Weighted least-squares quadratic fit at every pixel.

    Returns A [h, w, 3] = (A_xx, A_xy, A_yy), b [h, w, 2] = (b_x, b_y), c [h, w].
    The six unknowns (c, b_x, b_y, r_xx, r_yy, r_xy) of
        f(x + dx, y + dy) ~ c + b_x dx + b_y dy + r_xx dx^2 + r_yy dy^2 + r_xy dx dy
    solve the normal equations (B^T W B) r = B^T W f; A_xy = r_xy / 2.
    """
    h, w = f.shape
    ks = np.arange(-n, n + 1)
    g = np.exp(-(ks.astype(np.float64) ** 2) / (2.0 * sigma * sigma))
    g /= g.sum()
    basis = []
    weights = []
    samples = []
    for dy in ks:
        for dx in ks:
            basis.append([1.0, dx, dy, dx * dx, dy * dy, dx * dy])
            weights.append(g[dy + n] * g[dx + n])
            samples.append(_take(f, np.arange(h) + dy, np.arange(w) + dx).reshape(-1))
    bmat = np.array(basis, dtype=np.float64)                # [49, 6]
    wvec = np.array(weights, dtype=np.float64)              # [49]
    fmat = np.stack(samples, axis=0)                        # [49, h*w]
    normal = bmat.T @ (wvec[:, None] * bmat)                # [6, 6]
    rhs = bmat.T @ (wvec[:, None] * fmat)                   # [6, h*w]
    r = np.linalg.solve(normal, rhs)
    c = r[0].reshape(h, w)
    b = np.stack([r[1], r[2]], axis=-1).reshape(h, w, 2)
    a = np.stack([r[3], r[5] / 2.0, r[4]], axis=-1).reshape(h, w, 3)
    return a, b, c


def bilinear(field, ys, xs):
    """Sample field [h, w, ...] at real coordinates (ys, xs) (same shape), clamped to the image."""
    h, w = field.shape[:2]
    ys = np.clip(ys, 0.0, h - 1.0)
    xs = np.clip(xs, 0.0, w - 1.0)
    y0 = np.floor(ys).astype(np.int64)
    x0 = np.floor(xs).astype(np.int64)
    y1 = np.minimum(y0 + 1, h - 1)
    x1 = np.minimum(x0 + 1, w - 1)
    fy = ys - y0
    fx = xs - x0
    extra = (1,) * (field.ndim - 2)
    fy = fy.reshape(fy.shape + extra)
    fx = fx.reshape(fx.shape + extra)
    top = field[y0, x0] * (1 - fx) + field[y0, x1] * fx
    bot = field[y1, x0] * (1 - fx) + field[y1, x1] * fx
    return top * (1 - fy) + bot * fy


def window_blur(field, radius=WIN_R, sigma=WIN_SIGMA):
    """Normalised separable Gaussian window w(dy) w(dx), |dy|, |dx| <= radius, applied to every
    channel of field [h, w, C]: the row pass followed by the column pass."""
    h, w = field.shape[:2]
    ks = np.arange(-radius, radius + 1)
    g = np.exp(-(ks.astype(np.float64) ** 2) / (2.0 * sigma * sigma))
    g /= g.sum()
    rows = np.zeros_like(field)
    for dx in ks:
        rows += g[dx + radius] * _take(field, np.arange(h), np.arange(w) + dx)
    out = np.zeros_like(field)
    for dy in ks:
        out += g[dy + radius] * _take(rows, np.arange(h) + dy, np.arange(w))
    return out


def flow_iteration(a1, b1, a2, b2, prior, lam_abs=LAMBDA_ABS, lam_rel=LAMBDA_REL):
    """One displacement update at one level.  prior, result: [h, w, 2] = (u, v)."""
    h, w = prior.shape[:2]
    yy, xx = np.meshgrid(np.arange(h, dtype=np.float64), np.arange(w, dtype=np.float64), indexing="ij")
    ys = yy + prior[:, :, 1]
    xs = xx + prior[:, :, 0]
    a2s = bilinear(a2, ys, xs)
    b2s = bilinear(b2, ys, xs)
    axx = 0.5 * (a1[:, :, 0] + a2s[:, :, 0])
    axy = 0.5 * (a1[:, :, 1] + a2s[:, :, 1])
    ayy = 0.5 * (a1[:, :, 2] + a2s[:, :, 2])
    dbx = -0.5 * (b2s[:, :, 0] - b1[:, :, 0]) + axx * prior[:, :, 0] + axy * prior[:, :, 1]
    dby = -0.5 * (b2s[:, :, 1] - b1[:, :, 1]) + axy * prior[:, :, 0] + ayy * prior[:, :, 1]
    # G' = A^T A, h' = A^T db with A = [[axx, axy], [axy, ayy]]
    field = np.stack([axx * axx + axy * axy,
                      axy * (axx + ayy),
                      axy * axy + ayy * ayy,
                      axx * dbx + axy * dby,
                      axy * dbx + ayy * dby], axis=-1)
    agg = window_blur(field)
    g11, g12, g22, h1, h2 = (agg[:, :, k] for k in range(5))
    lam = lam_abs + lam_rel * 0.5 * (g11 + g22)
    m11 = g11 + lam
    m22 = g22 + lam
    r1 = h1 + lam * prior[:, :, 0]
    r2 = h2 + lam * prior[:, :, 1]
    # 2x2 solve by Cramer's rule (lambda = 0 on a flat region is 0/0, as in the plain method)
    det = m11 * m22 - g12 * g12
    with np.errstate(divide="ignore", invalid="ignore"):
        u = (m22 * r1 - g12 * r2) / det
        v = (m11 * r2 - g12 * r1) / det
    return np.stack([u, v], axis=-1)


def upsample_flow(d, h, w):
    """d~_l(y, x) = 2 * bilinear(d_{l+1}; y/2, x/2)."""
    yy, xx = np.meshgrid(np.arange(h, dtype=np.float64), np.arange(w, dtype=np.float64), indexing="ij")
    return 2.0 * bilinear(d, yy / 2.0, xx / 2.0)


def flow_from_gray(f_prev, f_cur, levels=3, iters=ITERS, lam_abs=LAMBDA_ABS, lam_rel=LAMBDA_REL):
    """Coarse-to-fine flow between two float gray images -> [h, w, 2] = (u, v)."""
    p1 = pyramid(f_prev, levels)
    p2 = pyramid(f_cur, levels)
    d = None
    for lvl in range(levels - 1, -1, -1):
        h, w = p1[lvl].shape
        a1, b1, _ = poly_expansion(p1[lvl])
        a2, b2, _ = poly_expansion(p2[lvl])
        d = np.zeros((h, w, 2)) if d is None else upsample_flow(d, h, w)
        for _ in range(iters):
            d = flow_iteration(a1, b1, a2, b2, d, lam_abs, lam_rel)
    return d


def flow(prev_rgb, cur_rgb, levels=3, iters=ITERS):
    return flow_from_gray(gray_float(prev_rgb), gray_float(cur_rgb), levels, iters)


def patch_motion(d, grid=24):
    """Eq. 5: RMS flow magnitude per patch, float64 [grid*grid], token i = grid*r + c."""
    h, w = d.shape[:2]
    ye = [(r * h) // grid for r in range(grid + 1)]
    xe = [(c * w) // grid for c in range(grid + 1)]
    mag2 = d[:, :, 0] ** 2 + d[:, :, 1] ** 2
    out = np.zeros(grid * grid)
    for r in range(grid):
        for c in range(grid):
            out[r * grid + c] = np.sqrt(mag2[ye[r]:ye[r + 1], xe[c]:xe[c + 1]].mean())
    return out


def gate(dp, tau_t, theta_r):
    """Eq. 6 and the redundancy rule.  Decisions are taken in fp32, the precision the kernel
    holds Delta P_i in.  -> (n_static, R fp32, redundant bool, margin) where margin is the
    distance of the nearest Delta P_i to tau_t (how fragile n_static is)."""
    dp32 = np.asarray(dp, dtype=np.float32)
    tau = np.float32(tau_t)
    n_static = int(np.count_nonzero(dp32 < tau))
    r = np.float32(n_static) / np.float32(dp32.size)
    redundant = bool(r > np.float32(theta_r))
    margin = float(np.min(np.abs(np.asarray(dp, dtype=np.float64) - float(tau))))
    return n_static, r, redundant, margin
