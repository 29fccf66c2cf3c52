"""Shared helpers of the GPU parity tests: one parameter dict -> library config and oracle config."""
import numpy as np

from oracle.cache import OracleConfig

FLOW_RTOL = 1e-3
FLOW_ATOL = 1e-4


DRIFT_SHIFTS = (0.0, 0.3, 0.6, 0.9, 2.4)       # px; a slow pan of 0.3 px per frame, then a jump


def drift_frame(shift, h=96, w=96):
    """Band-limited texture evaluated analytically at x - shift (no interpolation), as uint8 RGB."""
    rng = np.random.default_rng(11)
    yy, xx = np.meshgrid(np.arange(h, dtype=np.float64), np.arange(w, dtype=np.float64), indexing="ij")
    img = np.zeros((h, w))
    for _ in range(10):
        fx, fy = rng.uniform(-0.8, 0.8, 2)
        img += rng.uniform(0.3, 1.0) * np.sin(fx * (xx - shift) + fy * yy + rng.uniform(0, 6.28))
    g = np.clip(np.rint(128 + 35 * img), 0, 255).astype(np.uint8)
    return np.stack([g, g, g], axis=-1)


def _render_range(args):
    cfg_id, n, lo, hi = args
    from paper_2602_14236_amd import synth
    v = synth.video(cfg_id, n)
    return lo, [v.frame(t) for t in range(lo, hi)]


class FramePrefetcher:
    """Renders the frames of a workload in worker processes (spawned: they import numpy only and never
    touch the GPU), a chunk ahead of the consumer; frame(t) must be asked for in ascending order."""

    def __init__(self, cfg_id, n, chunk=8, workers=8):
        import multiprocessing as mp
        from concurrent.futures import ProcessPoolExecutor
        self.pool = ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn"))
        self.chunks = [(cfg_id, n, lo, min(n, lo + chunk)) for lo in range(0, n, chunk)]
        self.depth = 2 * workers
        self.futs = {}
        self.next_submit = 0
        self.cur = None
        self._fill()

    def _fill(self):
        while self.next_submit < len(self.chunks) and len(self.futs) < self.depth:
            c = self.chunks[self.next_submit]
            self.futs[c[2]] = self.pool.submit(_render_range, c)
            self.next_submit += 1

    def frame(self, t):
        if self.cur is None or not (self.cur[0] <= t < self.cur[0] + len(self.cur[1])):
            lo = max(k for k in self.futs if k <= t)
            self.cur = self.futs.pop(lo).result()
            self._fill()
        return self.cur[1][t - self.cur[0]]

    def close(self):
        self.pool.shutdown(wait=False, cancel_futures=True)


def params(src_h=336, src_w=336, **kw):
    p = dict(src_h=src_h, src_w=src_w, flow_levels=3, flow_iters=3, tau_t=0.5, theta_r=0.90, canny_lo=50,
             canny_hi=100, tier_mode=0, tau_high=0.30, tau_med=0.15, tau_low=0.03, k_fp16=0, k_int8=0, k_int4=0,
             n_layers=1, n_heads=2, cap_fp16=1200, cap_int8=1200, cap_int4=1200, max_frames=8, budget_tokens=0, tiles_per_frame=1, adapt_rate_q8=0)
    p.update(kw)
    return p


def lib_config(p):
    from paper_2602_14236_amd import binding
    return binding.make_config(p["src_h"], p["src_w"], **{k: v for k, v in p.items() if k not in ("src_h", "src_w")})


def oracle_config(p):
    return OracleConfig(grid=24, head_dim=128, **p)


def workload_params(wl, frames=None, n_layers=None, n_heads=None, **kw):
    """Parameters of a benchmark workload (paper_2602_14236_amd.synth.Workload), optionally cut down."""
    frames = wl.frames if frames is None else frames
    nl = wl.n_layers if n_layers is None else n_layers
    nh = wl.n_heads if n_heads is None else n_heads
    if wl.tier_mode == 1:
        caps = dict(cap_fp16=wl.k_fp16 * frames, cap_int8=wl.k_int8 * frames, cap_int4=wl.k_int4 * frames)
    else:
        caps = dict(cap_fp16=576 * frames, cap_int8=576 * frames, cap_int4=576 * frames)
    p = params(wl.height, wl.width, flow_levels=wl.flow_levels, tier_mode=wl.tier_mode, k_fp16=wl.k_fp16,
               k_int8=wl.k_int8, k_int4=wl.k_int4, n_layers=nl, n_heads=nh, max_frames=frames, **caps)
    p.update(kw)
    return p


def close(a, b, rtol=FLOW_RTOL, atol=FLOW_ATOL):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.abs(a - b) <= atol + rtol * np.abs(b)


def pool_arrays(ctx):
    """Pool contents as numpy arrays shaped like the oracle's [n_l, 2, n_h, cap, row]."""
    c = ctx.cfg
    v = ctx.pool_views()
    shp = (c.n_layers, 2, c.n_heads)
    out = {}
    for k, t in v.items():
        a = t.cpu().numpy()
        out[k] = a.reshape(shp + a.shape[1:])
    return out


def assert_same(got, exp, name):
    """Bit-exact comparison that reports a short summary instead of dumping the arrays."""
    got = np.asarray(got)
    exp = np.asarray(exp)
    assert got.shape == exp.shape, f"{name}: shape {got.shape} != {exp.shape}"
    if got.dtype.kind == "f":
        got = got.view({2: np.uint16, 4: np.uint32, 8: np.uint64}[got.dtype.itemsize])
        exp = exp.view(got.dtype)
    bad = np.argwhere(got != exp)
    if bad.size:
        first = [tuple(int(v) for v in b) for b in bad[:4]]
        vals = [(got[b], exp[b]) for b in first]
        raise AssertionError(f"{name}: {len(bad)} of {got.size} differ; first at {first}: (got, expected) = {vals}")


def fp16_operand_bounds(orc, q, lo, hi, sm, q_per_kv):
    """Elementwise error bounds of attention whose operands are rounded to fp16 (the matrix-core path;
    derivation in tests/test_gpu_attention.py::test_attend_grouped_queries):
    (bound on out [n_q, 128], bound on lse [n_q]) from the oracle's dequantised rows."""
    from oracle.attention import cached_tokens
    u = 2.0 ** -11
    k, v = cached_tokens(orc, 0, lo, hi)                       # float64 [n_heads, n_tok, 128]
    qf = np.asarray(q, dtype=np.float64)
    bound = np.zeros((qf.shape[0], 128))
    lse_bound = np.zeros(qf.shape[0])
    for j in range(qf.shape[0]):
        h = j // q_per_kv
        s = sm * (k[h] @ qf[j])
        s_abs = sm * (np.abs(k[h]) @ np.abs(qf[j]))
        p = np.exp(s - s.max())
        p /= p.sum()
        bound[j] = 2.0 * u * (2.0 + 2.0 * s_abs.max()) * (p @ np.abs(v[h])) + 1e-6
        lse_bound[j] = 2.0 * u * (1.0 + s_abs.max()) + 1e-6
    return bound, lse_bound
