"""Pins of the flow / gate oracle (CPU only): invariants, closed forms on quadratic images, an
independently written weighted-least-squares solve for the single-iteration case, and the
rational boundary of the redundancy gate."""
import numpy as np
import pytest

from oracle import flow as of


def _texture(h, w, seed, shift=(0.0, 0.0)):
    """Smooth band-limited texture, evaluated analytically at (x - sx, y - sy)."""
    rng = np.random.default_rng(seed)
    yy, xx = np.meshgrid(np.arange(h, dtype=np.float64), np.arange(w, dtype=np.float64), indexing="ij")
    xx = xx - shift[0]
    yy = yy - shift[1]
    img = np.zeros((h, w))
    for _ in range(10):
        fx, fy = rng.uniform(-0.8, 0.8, 2)
        img += rng.uniform(0.3, 1.0) * np.sin(fx * xx + fy * yy + rng.uniform(0, 6.28))
    return img


def _to_rgb_u8(img):
    g = np.clip(np.rint(128 + 35 * img), 0, 255).astype(np.uint8)
    return np.stack([g, g, g], axis=-1)


# ---- invariants --------------------------------------------------------------------------------
def test_identical_frames_give_exactly_zero_flow_and_full_redundancy():
    rgb = _to_rgb_u8(_texture(72, 96, 1))
    d = of.flow(rgb, rgb.copy(), levels=3)
    assert np.all(d == 0.0)
    dp = of.patch_motion(d)
    n, r, red, _ = of.gate(dp, 0.5, 0.9)
    assert n == 576 and r == np.float32(1.0) and red
    n0, r0, red0, _ = of.gate(dp, 0.0, 0.9)          # strict '<': nothing is below a zero threshold
    assert n0 == 0 and r0 == 0.0 and not red0


def test_pyramid_of_constant_is_constant_and_sizes_are_ceil_halved():
    pyr = of.pyramid(np.full((45, 71), 0.375), 4)
    assert [p.shape for p in pyr] == [(45, 71), (23, 36), (12, 18), (6, 9)]
    for p in pyr:
        assert np.all(p == 0.375)


def test_downsample_matches_direct_definition():
    rng = np.random.default_rng(2)
    f = rng.uniform(0, 1, (9, 12))
    out = of.downsample(f)
    k = [1 / 16, 4 / 16, 6 / 16, 4 / 16, 1 / 16]
    for i in range(out.shape[0]):
        for j in range(out.shape[1]):
            acc = 0.0
            for a in range(-2, 3):
                for b in range(-2, 3):
                    acc += k[a + 2] * k[b + 2] * f[min(max(2 * i + a, 0), 8), min(max(2 * j + b, 0), 11)]
            assert abs(out[i, j] - acc) < 1e-14


# ---- expansion: closed form on a quadratic -----------------------------------------------------
A0 = np.array([[0.08, -0.03], [-0.03, 0.11]])       # G = A^T A must dominate the ridge term
B0 = np.array([0.2, -0.15])
C0 = 0.4


def _quadratic(h, w, shift=(0.0, 0.0)):
    yy, xx = np.meshgrid(np.arange(h, dtype=np.float64), np.arange(w, dtype=np.float64), indexing="ij")
    x = xx - shift[0]
    y = yy - shift[1]
    return A0[0, 0] * x * x + 2 * A0[0, 1] * x * y + A0[1, 1] * y * y + B0[0] * x + B0[1] * y + C0


def test_expansion_of_quadratic_image_is_exact_in_the_interior():
    f = _quadratic(40, 50)
    a, b, c = of.poly_expansion(f)
    n = of.POLY_N
    yy, xx = np.meshgrid(np.arange(40.0), np.arange(50.0), indexing="ij")
    inner = (slice(n, 40 - n), slice(n, 50 - n))
    assert np.allclose(a[inner][..., 0], A0[0, 0], atol=1e-12)
    assert np.allclose(a[inner][..., 1], A0[0, 1], atol=1e-12)
    assert np.allclose(a[inner][..., 2], A0[1, 1], atol=1e-12)
    bx = B0[0] + 2 * (A0[0, 0] * xx + A0[0, 1] * yy)       # gradient of the quadratic
    by = B0[1] + 2 * (A0[0, 1] * xx + A0[1, 1] * yy)
    assert np.allclose(b[inner][..., 0], bx[inner], atol=1e-11)
    assert np.allclose(b[inner][..., 1], by[inner], atol=1e-11)
    assert np.allclose(c[inner], f[inner], atol=1e-11)


@pytest.mark.parametrize("levels,size,d", [(1, 64, (1.3, -0.7)), (2, 160, (2.6, 1.9)), (1, 64, (-0.4, 0.25))])
def test_translated_quadratic_recovers_real_displacement(levels, size, d):
    f1 = _quadratic(size, size)
    f2 = _quadratic(size, size, shift=d)              # f2(x) = f1(x - d)
    flow = of.flow_from_gray(f1, f2, levels=levels)
    margin = sum(2 ** l * (of.POLY_N + of.ITERS * of.WIN_R) for l in range(levels)) + 4
    core = flow[margin:size - margin, margin:size - margin]
    assert core.size > 0
    assert np.max(np.abs(core[..., 0] - d[0])) < 1e-4
    assert np.max(np.abs(core[..., 1] - d[1])) < 1e-4


# ---- integer translation of a textured uint8 image (quality, stated tolerance) -------------------
@pytest.mark.parametrize("levels,shift,tol", [(1, (1, 0), 0.10), (2, (2, -1), 0.05), (2, (-3, 2), 0.05)])
def test_integer_translation_of_texture(levels, shift, tol):
    h = w = 64
    big = _texture(h + 16, w + 16, 11)
    f1 = _to_rgb_u8(big[8:8 + h, 8:8 + w])
    f2 = _to_rgb_u8(big[8 - shift[1]:8 - shift[1] + h, 8 - shift[0]:8 - shift[0] + w])   # content moves by +shift
    d = of.flow(f1, f2, levels=levels)
    core = d[16:-16, 16:-16]
    epe = np.sqrt((core[..., 0] - shift[0]) ** 2 + (core[..., 1] - shift[1]) ** 2)
    assert np.median(epe) < tol


# ---- single iteration, lambda = 0: independent weighted least squares ---------------------------
def _wls_expansion_pixel(f, y, x, n, sigma):
    h, w = f.shape
    rows, rhs = [], []
    for dy in range(-n, n + 1):
        for dx in range(-n, n + 1):
            wt = np.exp(-(dx * dx + dy * dy) / (2 * sigma * sigma))
            sw = np.sqrt(wt)
            rows.append(sw * np.array([1.0, dx, dy, dx * dx, dy * dy, dx * dy]))
            rhs.append(sw * f[min(max(y + dy, 0), h - 1), min(max(x + dx, 0), w - 1)])
    r, *_ = np.linalg.lstsq(np.array(rows), np.array(rhs), rcond=None)
    amat = np.array([[r[3], r[5] / 2], [r[5] / 2, r[4]]])
    return amat, np.array([r[1], r[2]])


def test_single_iteration_equals_textbook_weighted_least_squares():
    h = w = 16
    f1 = 0.5 + 0.2 * _texture(h, w, 21)
    f2 = 0.5 + 0.2 * _texture(h, w, 21, shift=(0.6, -0.4))
    got = of.flow_from_gray(f1, f2, levels=1, iters=1, lam_abs=0.0, lam_rel=0.0)
    exp1 = [[_wls_expansion_pixel(f1, y, x, 3, 1.5) for x in range(w)] for y in range(h)]
    exp2 = [[_wls_expansion_pixel(f2, y, x, 3, 1.5) for x in range(w)] for y in range(h)]
    for y in range(0, h, 3):
        for x in range(0, w, 3):
            rows, rhs = [], []
            for dy in range(-5, 6):
                for dx in range(-5, 6):
                    yy, xx = min(max(y + dy, 0), h - 1), min(max(x + dx, 0), w - 1)
                    wt = np.exp(-(dx * dx + dy * dy) / (2 * 2.5 * 2.5))
                    amat = 0.5 * (exp1[yy][xx][0] + exp2[yy][xx][0])
                    db = -0.5 * (exp2[yy][xx][1] - exp1[yy][xx][1])
                    rows.append(np.sqrt(wt) * amat)          # minimise sum w |A d - db|^2
                    rhs.append(np.sqrt(wt) * db)
            dd, *_ = np.linalg.lstsq(np.concatenate(rows), np.concatenate(rhs), rcond=None)
            assert np.allclose(got[y, x], dd, rtol=1e-7, atol=1e-9)


def test_ridge_term_is_prior_centred():
    # flat image pair: G = h = 0, so every iteration must return its prior unchanged
    z = np.zeros((20, 20, 3))
    zb = np.zeros((20, 20, 2))
    prior = np.random.default_rng(0).uniform(-1, 1, (20, 20, 2))
    out = of.flow_iteration(z, zb, z, zb, prior)
    assert np.allclose(out, prior, atol=1e-15)


def test_bilinear_and_upsample():
    f = np.arange(12, dtype=np.float64).reshape(3, 4)
    ys = np.array([[0.5, 1.25, 7.0]])
    xs = np.array([[0.5, 2.75, -3.0]])
    got = of.bilinear(f, ys, xs)
    assert np.allclose(got, [[2.5, 7.75, 8.0]])          # linear ramp: value = 4y + x, clamped at the border
    d = np.zeros((2, 3, 2))
    d[..., 0] = [[0, 1, 2], [0, 1, 2]]
    up = of.upsample_flow(d, 4, 6)
    assert np.allclose(up[0, :, 0], [0, 1, 2, 3, 4, 4])  # 2 * d(x / 2), clamped at the last sample


# ---- Eq. 5 / Eq. 6 ------------------------------------------------------------------------------
def test_patch_motion_of_constant_flow():
    d = np.zeros((336, 336, 2))
    d[..., 0] = 3.0
    d[..., 1] = -4.0
    dp = of.patch_motion(d)
    assert dp.shape == (576,) and np.allclose(dp, 5.0)
    d[:14, 14:28] = 0.0                                   # token index = 24 * row + col
    assert of.patch_motion(d)[1] == 0.0


def test_patch_motion_is_rms_not_mean():
    d = np.zeros((48, 48, 2))
    d[0, 0, 0] = 2.0                                      # one pixel of a 2x2 patch
    dp = of.patch_motion(d)
    assert np.isclose(dp[0], np.sqrt(4.0 / 4.0))


def test_gate_rational_boundary():
    dp = np.full(576, 1.0)
    dp[:432] = 0.1
    n, r, red, _ = of.gate(dp, 0.5, 0.75)
    assert n == 432 and r == np.float32(0.75) and not red   # R must EXCEED theta_R
    dp[432] = 0.1
    n, r, red, _ = of.gate(dp, 0.5, 0.75)
    assert n == 433 and red
    dp = np.full(576, 0.5)
    assert of.gate(dp, 0.5, 0.9)[0] == 0                  # Delta P equal to tau_t is not static
