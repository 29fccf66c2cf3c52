"""GPU parity: saliency map and pooled scores against the oracle, through the C ABI.
The whole stage is integer arithmetic, so maps and scores must be bit-exact."""
import numpy as np
import pytest
import torch

from oracle import saliency as osal
from paper_2602_14236_amd import synth

from _util import lib_config, params

pytestmark = pytest.mark.gpu


def _run(ctx, rgb):
    h, w, _ = rgb.shape
    d_rgb = torch.from_numpy(rgb).cuda()
    salmap = torch.full((h, w), 77, dtype=torch.uint8, device="cuda")
    scores = torch.full((576,), -1.0, dtype=torch.float32, device="cuda")
    ctx.saliency_pool(d_rgb, salmap, scores)
    torch.cuda.synchronize()
    return scores.cpu().numpy(), salmap.cpu().numpy()


def _check(ctx, rgb, lo=50, hi=100):
    got_scores, got_map = _run(ctx, rgb)
    exp_scores, exp_map = osal.saliency_pool(rgb, 24, lo, hi)
    bad = np.argwhere(got_map != exp_map)
    assert bad.size == 0, f"{len(bad)} map pixels differ, first {bad[:5].tolist()}"
    assert np.array_equal(got_scores.view(np.uint32), exp_scores.view(np.uint32))
    return exp_map


def test_config1_frames_bit_exact():
    from paper_2602_14236_amd import binding
    ctx = binding.SaliContext(lib_config(params()))
    v = synth.video(1)
    for t in (0, 1, 5):
        print("cfg1 frame", t, flush=True)
        m = _check(ctx, v.frame(t))
        assert (m == 1).any() and (m == 2).any()
    ctx.close()


@pytest.mark.parametrize("h,w", [(24, 24), (50, 77), (97, 33), (360, 640), (129, 257)])
def test_ragged_sizes_bit_exact(h, w):
    from paper_2602_14236_amd import binding
    ctx = binding.SaliContext(lib_config(params(h, w, flow_levels=1)))
    rng = np.random.default_rng(h * 1000 + w)
    # blocky image with noise: plenty of strong and weak edges, tiles with ragged tails
    img = np.zeros((h, w, 3), dtype=np.int64)
    img[:] = rng.integers(0, 256, 3)
    for _ in range(12):
        y0, x0 = rng.integers(0, h - 1), rng.integers(0, w - 1)
        y1, x1 = rng.integers(y0 + 1, h + 1), rng.integers(x0 + 1, w + 1)
        img[y0:y1, x0:x1] = rng.integers(0, 256, 3)
    yy, xx = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    img[..., 0] += (20 * np.sin(xx / 5.0)).astype(np.int64)            # soft gradients -> weak edges
    img += rng.integers(-4, 5, img.shape)
    rgb = np.clip(img, 0, 255).astype(np.uint8)
    print("ragged", h, w, flush=True)
    _check(ctx, rgb)
    ctx.close()


def test_thresholds_from_config_and_degenerate_images():
    from paper_2602_14236_amd import binding
    ctx = binding.SaliContext(lib_config(params(96, 96, flow_levels=1, canny_lo=10, canny_hi=30)))
    rng = np.random.default_rng(3)
    noise = rng.integers(0, 256, (96, 96, 3), dtype=np.uint8)        # pure noise: long tangled weak chains
    _check(ctx, noise, 10, 30)
    const = np.full((96, 96, 3), 131, dtype=np.uint8)
    s, m = _run(ctx, const)
    assert not m.any() and not s.any()
    step = np.zeros((96, 96, 3), dtype=np.uint8)
    step[:, 48:] = 255
    _check(ctx, step, 10, 30)
    ctx.close()


def test_long_weak_spiral_reaches_its_one_strong_pixel():
    """Hysteresis needs global connectivity: a one-pixel spiral that is weak everywhere except at its
    inner end must be kept whole."""
    from paper_2602_14236_amd import binding
    h = w = 120
    ctx = binding.SaliContext(lib_config(params(h, w, flow_levels=1, canny_lo=20, canny_hi=200)))
    img = np.full((h, w), 100, dtype=np.uint8)
    y, x, dy, dx, run = 60, 60, 0, 1, 6
    pts = []
    for leg in range(16):
        for _ in range(run):
            pts.append((y, x))
            y, x = y + dy, x + dx
        dy, dx = dx, -dy
        run += 6 if leg % 2 else 0
    for (py, px) in pts:
        if 2 <= py < h - 2 and 2 <= px < w - 2:
            img[py - 1:py + 2, px - 1:px + 2] = 112            # faint ridge: weak response
    img[58:63, 58:63] = 255                                   # bright blob at the inner end: strong
    rgb = np.stack([img, img, img], axis=-1)
    m = _check(ctx, rgb, 20, 200)
    assert (m >= 1).sum() > 200
    ctx.close()
