"""Seeded synthetic inputs: video frames and per-frame K/V tensors.

This module only *draws inputs*.  It holds none of the method's arithmetic
(no flow, saliency, tiering or quantisation) and imports neither the HIP
binding nor the CPU oracle; both sides are fed from here so that they see
byte-identical data.

The paper evaluates on an unnamed private set of video clips and on K/V
tensors of a trained LLaVA-1.6 model (Experimental Setup); neither can be
shipped, so five seeded generators with the paper's shapes (576 visual tokens
per frame on a 24x24 grid, 336x336 canonical frames, LLaVA-shaped K/V) stand
in for them.

Scene recipe (all configs): per channel a low-frequency sinusoid background,
six textured ellipses that translate with constant velocity and wrap at the
frame border, fresh Gaussian sensor noise (sigma = 2 grey levels) on every
frame, rounded and clamped to uint8, interleaved HWC.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 20260214
GRID = 24
TOKENS = GRID * GRID


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and presets of one of the five benchmark configurations."""
    index: int
    name: str
    frames: int
    height: int
    width: int
    flow_levels: int
    n_layers: int
    n_heads: int
    head_dim: int
    tier_mode: int                      # 0 = thresholds (Eq. 8), 1 = top-k counts
    k_fp16: int
    k_int8: int
    k_int4: int
    heavy_tail: bool = False            # Student-t(3) values + outlier channels
    subpixel: bool = False              # real-valued velocities up to 12 px/frame

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def elems_per_token(self) -> int:
        return self.n_layers * 2 * self.n_heads * self.head_dim


WORKLOADS: Dict[int, Workload] = {
    1: Workload(1, "cfg1-8f-336-1layer", 8, 336, 336, 3, 1, 32, 128, 0, 0, 0, 0),
    2: Workload(2, "cfg2-64f-336-7B-int8", 64, 336, 336, 3, 32, 32, 128, 1, 173, 403, 0),
    3: Workload(3, "cfg3-1800f-640x360-4layer", 1800, 360, 640, 3, 4, 32, 128, 1, 249, 56, 168),
    4: Workload(4, "cfg4-256f-1080p-13B-int4", 256, 1080, 1920, 5, 40, 40, 128, 1, 173, 0, 403,
                subpixel=True),
    5: Workload(5, "cfg5-128f-336-adversarial", 128, 336, 336, 3, 32, 32, 128, 0, 0, 0, 0,
                heavy_tail=True),
}


# --------------------------------------------------------------------------
# scenes
# --------------------------------------------------------------------------
@dataclasses.dataclass
class _Ellipse:
    cx: float
    cy: float
    ax: float
    ay: float
    angle: float
    colour: np.ndarray      # (3,)
    l1: float
    l2: float
    vx: float
    vy: float


@dataclasses.dataclass
class _Scene:
    h: int
    w: int
    lam_x: np.ndarray
    lam_y: np.ndarray
    phi_x: np.ndarray
    phi_y: np.ndarray
    ellipses: List[_Ellipse]


def _draw_scene(rng: np.random.Generator, h: int, w: int, subpixel: bool, tex_scale: float) -> _Scene:
    lam_x = rng.uniform(0.5, 1.5, 3) * w
    lam_y = rng.uniform(0.5, 1.5, 3) * w
    phi_x = rng.uniform(0.0, 2 * math.pi, 3)
    phi_y = rng.uniform(0.0, 2 * math.pi, 3)
    ells = []
    for _ in range(6):
        ax, ay = rng.uniform(w / 16.0, w / 6.0, 2)
        cx = rng.uniform(0, w)
        cy = rng.uniform(0, h)
        ang = rng.uniform(0, math.pi)
        col = rng.uniform(40.0, 215.0, 3)
        l1, l2 = rng.uniform(6.0, 12.0, 2) * tex_scale
        if subpixel:
            mag = rng.uniform(2.0, 12.0)
            th = rng.uniform(0, 2 * math.pi)
            vx, vy = mag * math.cos(th), mag * math.sin(th)
        else:
            while True:
                vx, vy = (int(v) for v in rng.integers(-4, 5, 2))
                if vx != 0 or vy != 0:
                    break
        ells.append(_Ellipse(cx, cy, ax, ay, ang, col, l1, l2, float(vx), float(vy)))
    return _Scene(h, w, lam_x, lam_y, phi_x, phi_y, ells)


def _render(scene: _Scene, offsets: np.ndarray, noise_rng: Optional[np.random.Generator]) -> np.ndarray:
    """Paint the scene with ellipse k displaced by offsets[k] = (dx, dy)."""
    h, w = scene.h, scene.w
    yy, xx = np.meshgrid(np.arange(h, dtype=np.float64), np.arange(w, dtype=np.float64), indexing="ij")
    img = np.empty((h, w, 3), dtype=np.float64)
    for c in range(3):
        img[:, :, c] = 128.0 + 40.0 * np.sin(2 * math.pi * xx / scene.lam_x[c] + scene.phi_x[c]) \
                                   * np.sin(2 * math.pi * yy / scene.lam_y[c] + scene.phi_y[c])
    for k, e in enumerate(scene.ellipses):            # fixed paint order
        cx = e.cx + offsets[k, 0]
        cy = e.cy + offsets[k, 1]
        dx = np.mod(xx - cx + w / 2.0, w) - w / 2.0     # wrap at the border
        dy = np.mod(yy - cy + h / 2.0, h) - h / 2.0
        ca, sa = math.cos(e.angle), math.sin(e.angle)
        p = ca * dx + sa * dy
        q = -sa * dx + ca * dy
        inside = (p / e.ax) ** 2 + (q / e.ay) ** 2 <= 1.0
        tex = 30.0 * np.sin(2 * math.pi * p / e.l1) * np.sin(2 * math.pi * q / e.l2)
        for c in range(3):
            ch = img[:, :, c]
            ch[inside] = e.colour[c] + tex[inside]
    if noise_rng is not None:
        img += noise_rng.normal(0.0, 2.0, img.shape)
    return np.clip(np.rint(img), 0, 255).astype(np.uint8)


class Video:
    """Lazily rendered frame sequence of one workload; `frame(t)` is 0-based."""

    def __init__(self, workload: Workload, n_frames: Optional[int] = None):
        self.workload = workload
        self.n_frames = workload.frames if n_frames is None else int(n_frames)
        self._plan = _plan_frames(workload, self.n_frames)
        self._cache: Dict[int, np.ndarray] = {}

    def __len__(self) -> int:
        return self.n_frames

    def frame(self, t: int) -> np.ndarray:
        if not 0 <= t < self.n_frames:
            raise IndexError(t)
        kind, arg = self._plan[t]
        if kind == "copy":
            return self.frame(arg)
        if t in self._cache:
            return self._cache[t]
        wl = self.workload
        if kind == "noise":
            rng = np.random.default_rng([wl.seed, 7, t])
            out = rng.integers(0, 256, (wl.height, wl.width, 3), dtype=np.uint8)
        elif kind == "scene":
            scene, offsets, noisy = arg
            nrng = np.random.default_rng([wl.seed, 1, t]) if noisy else None
            out = _render(scene, offsets, nrng)
        elif kind == "split":
            # left part frozen (byte copy of frame `src`), right part moved: see _plan_frames
            src, scene, offsets, x_split = arg
            out = self.frame(src).copy()
            moved = _render(scene, offsets, None)
            out[:, x_split:, :] = moved[:, x_split:, :]
        else:  # pragma: no cover
            raise AssertionError(kind)
        if len(self._cache) > 8:
            self._cache.pop(next(iter(self._cache)))
        self._cache[t] = out
        return out

    def kind(self, t: int) -> str:
        return self._plan[t][0]


def _plan_frames(wl: Workload, n: int):
    """Per frame: ("scene", (scene, offsets, noisy)) | ("copy", src) | ("noise", None) | ("split", ...)."""
    rng = np.random.default_rng([wl.seed, 0])
    tex_scale = wl.height / 336.0 if wl.subpixel else 1.0
    plan = []
    if wl.index in (1, 2, 4):
        scene = _draw_scene(rng, wl.height, wl.width, wl.subpixel, tex_scale)
        vel = np.array([[e.vx, e.vy] for e in scene.ellipses])
        for t in range(n):
            plan.append(("scene", (scene, vel * t, True)))
        if wl.index == 1 and n > 3:
            plan[3] = ("copy", 2)          # 1-based frame 4 is a byte copy of frame 3
        return plan
    if wl.index == 3:
        scene = _draw_scene(rng, wl.height, wl.width, False, 1.0)
        vel = np.array([[e.vx, e.vy] for e in scene.ellipses])
        # alternate moving and near-static runs; static share about 40 %
        moving_flags = []
        static = False
        while len(moving_flags) < n:
            run = int(rng.integers(5, 61)) if static else int(rng.integers(8, 91))
            moving_flags += [not static] * run
            static = not static
        off = np.zeros_like(vel)
        for t in range(n):
            if t > 0 and moving_flags[t]:
                off = off + vel
            plan.append(("scene", (scene, off.copy(), True)))
        return plan
    if wl.index == 5:
        scene = None
        off = None
        vel = None
        noise_at = {21, 22, 70, 101}
        dup_runs = [(5, 8), (40, 47), (90, 92)]            # inclusive ranges copying the frame before them
        split_at = 58                                      # the rational-boundary frame
        tau0_at = 120                                      # a duplicate used by the tau_t = 0 sub-run
        for t in range(n):
            if t % 16 == 0:                                # scene cut
                scene = _draw_scene(rng, wl.height, wl.width, False, 1.0)
                vel = np.array([[e.vx, e.vy] for e in scene.ellipses])
                off = np.zeros_like(vel)
                plan.append(("scene", (scene, off.copy(), True)))
                continue
            off = off + vel
            if t in noise_at:
                plan.append(("noise", None))
            elif any(a <= t <= b for a, b in dup_runs) or t == tau0_at:
                src = t - 1
                while plan[src][0] == "copy":
                    src = plan[src][1]
                plan.append(("copy", src))
            elif t == split_at:
                src = t - 1
                while plan[src][0] == "copy":
                    src = plan[src][1]
                plan.append(("split", (src, _split_scene(wl), _SPLIT_SHIFT, _SPLIT_X)))
            elif t == split_at - 1:
                plan.append(("scene", (_split_scene(wl), np.zeros((1, 2)), False)))
            else:
                plan.append(("scene", (scene, off.copy(), True)))
        return plan
    raise ValueError(wl.index)


# The rational-boundary pair of config 5: frame 57 is a noise-free texture; frame 58 keeps
# columns [0, _SPLIT_X) byte-identical and shows the same texture displaced in the rest.
_SPLIT_X = 252                     # 18 of 24 patch columns (18 * 24 = 432 patches) stay frozen
_SPLIT_SHIFT = np.array([[3.0, 2.0]])


class _TextureScene(_Scene):
    pass


def _split_scene(wl: Workload) -> _Scene:
    """A full-frame textured 'ellipse' (semi-axes far larger than the frame) and no background motion."""
    rng = np.random.default_rng([wl.seed, 5])
    sc = _draw_scene(rng, wl.height, wl.width, False, 1.0)
    big = _Ellipse(wl.width / 2.0, wl.height / 2.0, 1e6, 1e6, 0.3, np.array([120.0, 130.0, 110.0]),
                   9.0, 11.0, 0.0, 0.0)
    sc.ellipses = [big]
    return sc


def gate_schedule(config: int) -> Dict[int, Tuple[float, float]]:
    """Frames at which a workload changes the temporal thresholds: {frame: (tau_t, theta_R)}; the
    values hold from that frame on until the next entry.  Config 5 evaluates its rational-boundary
    frame (exactly 432 of 576 static patches) with theta_R = 0.75 and one duplicate frame with
    tau_t = 0 (strict '<': no patch is below a zero threshold); everything else runs at the
    defaults (0.5 px, 0.90)."""
    if config == 5:
        return {58: (0.5, 0.75), 59: (0.5, 0.90), 120: (0.0, 0.90), 121: (0.5, 0.90)}
    return {}


def video(config: int, n_frames: Optional[int] = None) -> Video:
    return Video(WORKLOADS[config], n_frames)


# --------------------------------------------------------------------------
# K/V tensors
# --------------------------------------------------------------------------
def kv_channel_scale(wl: Workload, n_layers: Optional[int] = None, n_heads: Optional[int] = None):
    """Per-channel lognormal(0, 0.5) scale, fixed per workload: torch fp32 [n_l, 2, n_h, 1, D] (CPU).
    n_layers / n_heads cut the tensor down to its leading layers / heads."""
    import torch
    nl = wl.n_layers if n_layers is None else n_layers
    nh = wl.n_heads if n_heads is None else n_heads
    g = torch.Generator(device="cpu")
    g.manual_seed(wl.seed * 1000 + 17)
    c = torch.exp(0.5 * torch.randn((nl, 2, wl.n_heads, 1, wl.head_dim), generator=g, dtype=torch.float32))
    if wl.heavy_tail:
        # four fixed outlier dims per head, scaled x20
        gi = torch.Generator(device="cpu")
        gi.manual_seed(wl.seed * 1000 + 23)
        for h in range(wl.n_heads):
            dims = torch.randperm(wl.head_dim, generator=gi)[:4]
            c[:, :, h, 0, dims] *= 20.0
    return c[:, :, :nh].contiguous()


def kv_frame(wl: Workload, t: int, device="cpu", n_layers: Optional[int] = None, n_heads: Optional[int] = None,
             scale=None):
    """K/V of frame t: fp16 [n_l, 2, n_h, 576, D], drawn on `device` from a (seed, t) generator.

    The draw depends on the device's RNG, so a caller that needs the same bytes on host and
    GPU draws once and copies.
    """
    import torch
    nl = wl.n_layers if n_layers is None else n_layers
    nh = wl.n_heads if n_heads is None else n_heads
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(wl.seed * 100003 + t)
    shape = (nl, 2, nh, TOKENS, wl.head_dim)
    if scale is None:
        scale = kv_channel_scale(wl, nl, nh)
    scale = scale.to(dev)
    out = torch.empty(shape, dtype=torch.float16, device=dev)
    for l in range(nl):                                   # layer at a time keeps the fp32 temporaries small
        z = torch.randn(shape[1:], generator=g, dtype=torch.float32, device=dev)
        if wl.heavy_tail:
            chi = torch.randn((3,) + shape[1:], generator=g, dtype=torch.float32, device=dev).square_().sum(0)
            z = z / torch.sqrt(chi / 3.0)
        out[l] = (z * scale[l]).clamp_(-65504.0, 65504.0).to(torch.float16)
    return out
