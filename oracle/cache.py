"""Oracle: the per-frame pipeline of Algorithm 1 with a compacted mixed-precision cache.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Algorithm 1: for every frame, (t > 1) compute R_frame by optical flow against
the previous frame; if R_frame > theta_R the cache entry of t is a pointer to
the previous entry and nothing else happens; otherwise compute the saliency
map, pool it per patch, assign Q(s_i) and store (K_i, V_i) at that precision.
Just-In-Time Dequantization: entries are expanded again when read.

Memory budget (Experimental Setup: the methods are compared under a strict budget of 784
patches; the paper gives no eviction rule for its own method).  Reading taken, `budget_tokens`
> 0: the cache may hold at most that many patches (tokens kept at any precision; pruned tokens
and pointer entries hold nothing).  Before a frame is stored, the oldest stored frames are
evicted whole, oldest first (the order of the sliding-window baseline, at the granularity of a
cache entry because pointer entries share a stored frame's rows), until the new frame's kept
tokens fit the budget and its rows fit the pools.  An evicted frame and every pointer entry that
referred to it hold no data afterwards (src = -1).  The pools are then rings: a frame's rows of a
pool are one run [base, base + n); the run goes at the pool's cursor if it ends inside the pool,
else at row 0, and a place is free if it touches no row of a frame still held; the cursor
follows the newest run.  Frame ids must increase from call to call in this mode.

Dynamic-resolution encoding (Background, Adapter Projection: the vision encoder of the model the
paper uses cuts a high-resolution frame into several images of 576 patches each).  Reading taken,
`tiles_per_frame` = T > 1: a video frame is T images ("tiles"), its N_p = 576 T patches are the
patches of all of them; cache entry e = t T + j holds tile j of frame t.  The flow is taken per
tile against the same tile of the adjacent frame; Eq. 6 counts the static patches of all tiles
and the reuse rule takes ONE decision for the frame; a redundant frame's entries point at the last
stored entry of their own tile; otherwise every tile gets its saliency scores and its tiers
(Eq. 8 per patch; top-k counts per tile) and is stored as an entry of its own.

Adaptive thresholds (Discussion: the thresholds need tuning per video domain; Conclusion: adaptive
thresholds are future work; the paper gives no rule).  Reading taken, `tier_mode` = 2: Eq. 8 is
applied to every frame with the thresholds in force, and after a frame has been stored each
threshold moves a fraction alpha = adapt_rate_q8 / 256 of the way to the score quantile that would
have given the target share of its tier in that frame (targets k_fp16, k_int8, k_int4 tokens:
q_high = the score of rank k_fp16 in (score descending, index ascending) order, i.e. the largest
score outside the top k_fp16; q_med, q_low at ranks k_fp16 + k_int8 and k_fp16 + k_int8 + k_int4;
0 if that rank does not exist).  Thresholds and quantiles live on the score lattice (integers in
units of 2^-16, floor): tau <- tau + floor((q - tau) * adapt_rate_q8 / 256), so both sides of a
parity test do integer arithmetic.  The state starts from the configured tau_high / tau_med /
tau_low and is carried from stored frame to stored frame (pointer frames leave it alone).

Storage reading (the paper describes none): three pools indexed
[layer][K|V][head][slot][...], slots handed out in token order per tier; a
frame-table row (frame_id, src, stored, base16, base8, base4, n16, n8, n4, np)
per frame; a pointer frame carries the `src` of the last stored frame.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np

from . import flow as oflow
from . import quant as oq
from . import saliency as osal


@dataclasses.dataclass
class OracleConfig:
    src_h: int
    src_w: int
    grid: int = 24
    flow_levels: int = 3
    flow_iters: int = 3
    tau_t: float = 0.5
    theta_r: float = 0.90
    canny_lo: int = 50
    canny_hi: int = 100
    tier_mode: int = 0
    tau_high: float = 0.30
    tau_med: float = 0.15
    tau_low: float = 0.03
    k_fp16: int = 0
    k_int8: int = 0
    k_int4: int = 0
    n_layers: int = 1
    n_heads: int = 32
    head_dim: int = 128
    cap_fp16: int = 0
    cap_int8: int = 0
    cap_int4: int = 0
    max_frames: int = 0
    budget_tokens: int = 0          # 0 = no budget (append only)
    tiles_per_frame: int = 1        # images (of grid x grid patches each) that make up one video frame
    adapt_rate_q8: int = 0          # tier_mode 2: step of the threshold update in 1/256


@dataclasses.dataclass
class FrameRow:
    frame_id: int
    src: int
    stored: int
    base16: int = 0
    base8: int = 0
    base4: int = 0
    n16: int = 0
    n8: int = 0
    n4: int = 0
    npr: int = 0

    def as_tuple(self):
        return (self.frame_id, self.src, self.stored, self.base16, self.base8, self.base4,
                self.n16, self.n8, self.n4, self.npr)


class _FrameTable:
    """Frame-table rows, pool cursors and (with a budget) the set of frames still held.  Shared by the
    full oracle and the image-only walk so that both hand out the same rows."""

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        self.cursor = [0, 0, 0]
        self.last_src = -1
        self.rows: Dict[int, FrameRow] = {}
        self.held = []                  # stored frames still in the cache, oldest first (budget mode)
        self.overflow = False
        self.last_src_tile = {}         # tile index -> last stored entry of that tile (tiles_per_frame > 1)
        self.adapt_tau = [to_lattice(cfg.tau_high), to_lattice(cfg.tau_med), to_lattice(cfg.tau_low)]
        assert cfg.tiles_per_frame == 1 or cfg.budget_tokens == 0, "a budget evicts entries, not tiled frames"

    def _place(self, pool, n, cap):
        """Base of a run of n rows in `pool`, or None if no candidate place is free."""
        if n == 0:
            return self.cursor[pool]
        candidates = ([self.cursor[pool]] if self.cursor[pool] + n <= cap else []) + ([0] if n <= cap else [])
        for b in candidates:
            free = True
            for f in self.held:
                r = self.rows[f]
                fb, fn = (r.base16, r.base8, r.base4)[pool], (r.n16, r.n8, r.n4)[pool]
                if fn > 0 and b < fb + fn and fb < b + n:
                    free = False
            if free:
                return b
        return None

    def _evict_oldest(self):
        g = self.held.pop(0)
        self.rows[g] = FrameRow(g, -1, 0)
        for f, r in self.rows.items():
            if r.stored == 0 and r.src == g:
                self.rows[f] = FrameRow(f, -1, 0)

    def pointer(self, frame_id) -> FrameRow:
        T = self.cfg.tiles_per_frame
        row = FrameRow(frame_id, self.last_src if T == 1 else self.last_src_tile.get(frame_id % T, -1), 0)
        self.rows[frame_id] = row
        return row

    def store(self, frame_id, cnt) -> FrameRow:
        """Row of a frame with cnt = (n16, n8, n4, n_pruned) tokens per tier; stored = 0 if it cannot be held."""
        c = self.cfg
        caps = (c.cap_fp16, c.cap_int8, c.cap_int4)
        n = [int(cnt[0]), int(cnt[1]), int(cnt[2])]
        if c.budget_tokens > 0:
            assert frame_id > max(self.rows, default=-1), "frame ids must increase in budget mode"
            while True:
                bases = [self._place(p, n[p], caps[p]) for p in range(3)]
                held_tokens = sum(self.rows[f].n16 + self.rows[f].n8 + self.rows[f].n4 for f in self.held)
                if held_tokens + sum(n) <= c.budget_tokens and None not in bases:
                    break
                if not self.held:
                    bases = None
                    break
                self._evict_oldest()
        else:
            bases = list(self.cursor) if all(self.cursor[p] + n[p] <= caps[p] for p in range(3)) else None
        if bases is None:
            self.overflow = True
            row = FrameRow(frame_id, -1, 0)
            self.rows[frame_id] = row
            return row
        row = FrameRow(frame_id, frame_id, 1, bases[0], bases[1], bases[2], n[0], n[1], n[2], int(cnt[3]))
        for p in range(3):
            if n[p] > 0:
                self.cursor[p] = bases[p] + n[p]
        self.last_src = frame_id
        self.last_src_tile[frame_id % c.tiles_per_frame] = frame_id
        self.rows[frame_id] = row
        if c.budget_tokens > 0:
            self.held.append(frame_id)
        return row


def to_lattice(x):
    """floor(clamp(x, 0, 1) * 2^16): a score or threshold in units of 2^-16."""
    return int(np.floor(min(max(float(np.float32(x)), 0.0), 1.0) * 65536.0))


def assign_tiers(c: OracleConfig, scores, adapt_tau=None):
    """Eq. 8 (mode 0), the top-k counts (mode 1), or Eq. 8 with the adaptive thresholds in force
    (mode 2; adapt_tau = the three thresholds in units of 2^-16)."""
    if c.tier_mode == 0:
        return oq.tiers_threshold(scores, c.tau_high, c.tau_med, c.tau_low)
    if c.tier_mode == 2:
        return oq.tiers_threshold(scores, *(np.float32(t) / np.float32(65536.0) for t in adapt_tau))
    return oq.tiers_topk(scores, c.k_fp16, c.k_int8, c.k_int4)


def adapted_thresholds(c: OracleConfig, adapt_tau, scores):
    """The thresholds after a stored frame with these scores (tier_mode 2)."""
    s = np.asarray(scores, dtype=np.float32)
    order = sorted(range(s.size), key=lambda i: (-float(s[i]), i))
    ranks = (c.k_fp16, c.k_fp16 + c.k_int8, c.k_fp16 + c.k_int8 + c.k_int4)
    out = []
    for tau, r in zip(adapt_tau, ranks):
        q = to_lattice(s[order[r]]) if r < s.size else 0
        out.append(tau + ((q - tau) * c.adapt_rate_q8) // 256)          # floor division
    return out


class SaliCacheOracle:
    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        nl, nh, d = cfg.n_layers, cfg.n_heads, cfg.head_dim
        g = d // oq.GROUP
        self.pool16 = np.zeros((nl, 2, nh, cfg.cap_fp16, d), dtype=np.float16)
        self.codes8 = np.zeros((nl, 2, nh, cfg.cap_int8, d), dtype=np.int8)
        self.scale8 = np.zeros((nl, 2, nh, cfg.cap_int8, g), dtype=np.float32)
        self.codes4 = np.zeros((nl, 2, nh, cfg.cap_int4, d // 2), dtype=np.uint8)
        self.scale4 = np.zeros((nl, 2, nh, cfg.cap_int4, g), dtype=np.float32)
        self.zero4 = np.zeros((nl, 2, nh, cfg.cap_int4, g), dtype=np.float16)
        self.table = _FrameTable(cfg)
        self.tier: Dict[int, np.ndarray] = {}
        self.slot: Dict[int, np.ndarray] = {}
        self.prev_gray: Optional[np.ndarray] = None
        self.prev_tile_grays = None
        self.nonfinite = False
        self.last_gate = None
        self.last_dp = None
        self.last_scores = None

    # rows, cursors and the overflow flag live in the frame table
    rows = property(lambda self: self.table.rows)
    cursor = property(lambda self: self.table.cursor)
    last_src = property(lambda self: self.table.last_src)
    overflow = property(lambda self: self.table.overflow)

    # ---- the stand-alone calls ------------------------------------------------
    def flow_score(self, prev_rgb, cur_rgb):
        c = self.cfg
        d = oflow.flow(prev_rgb, cur_rgb, c.flow_levels, c.flow_iters)
        dp = oflow.patch_motion(d, c.grid)
        return d, dp, oflow.gate(dp, c.tau_t, c.theta_r)

    def saliency_pool(self, rgb):
        c = self.cfg
        return osal.saliency_pool(rgb, c.grid, c.canny_lo, c.canny_hi)

    def assign_tiers(self, scores):
        return assign_tiers(self.cfg, scores, self.table.adapt_tau)

    def kv_compress(self, kv_fp16, scores, frame_id):
        """kv_fp16: [n_l, 2, n_h, N, D].  Stores the frame; returns its table row."""
        tier = self.assign_tiers(scores)
        slot, cnt = oq.slots(tier)
        c = self.cfg
        if oq.has_nonfinite(kv_fp16[:, :, :, tier != oq.T_PRUNE, :]):
            self.nonfinite = True
        row = self.table.store(frame_id, cnt)
        if not row.stored:
            return row
        if c.tier_mode == 2:
            self.table.adapt_tau = adapted_thresholds(c, self.table.adapt_tau, scores)
        b16, b8, b4 = row.base16, row.base8, row.base4
        i16 = np.nonzero(tier == oq.T_FP16)[0]
        i8 = np.nonzero(tier == oq.T_INT8)[0]
        i4 = np.nonzero(tier == oq.T_INT4)[0]
        if i16.size:
            self.pool16[:, :, :, b16 + slot[i16], :] = kv_fp16[:, :, :, i16, :]
        if i8.size:
            q, s = oq.quant_int8(kv_fp16[:, :, :, i8, :])
            self.codes8[:, :, :, b8 + slot[i8], :] = q
            self.scale8[:, :, :, b8 + slot[i8], :] = s
        if i4.size:
            q, s, z = oq.quant_int4(kv_fp16[:, :, :, i4, :])
            self.codes4[:, :, :, b4 + slot[i4], :] = oq.pack_nibbles(q)
            self.scale4[:, :, :, b4 + slot[i4], :] = s
            self.zero4[:, :, :, b4 + slot[i4], :] = z
        self.tier[frame_id] = tier
        self.slot[frame_id] = slot
        return row

    def kv_decompress(self, frame_id):
        """-> (kv fp16 [n_l, 2, n_h, N, D], valid uint8 [N]); a pointer frame reads its source."""
        row = self.rows[frame_id]
        if row.src < 0:
            raise KeyError("frame holds no data")
        src = self.rows[row.src]
        tier, slot = self.tier[row.src], self.slot[row.src]
        c = self.cfg
        n = tier.size
        out = np.zeros((c.n_layers, 2, c.n_heads, n, c.head_dim), dtype=np.float16)
        i16 = np.nonzero(tier == oq.T_FP16)[0]
        i8 = np.nonzero(tier == oq.T_INT8)[0]
        i4 = np.nonzero(tier == oq.T_INT4)[0]
        if i16.size:
            out[:, :, :, i16, :] = self.pool16[:, :, :, src.base16 + slot[i16], :]
        if i8.size:
            out[:, :, :, i8, :] = oq.dequant_int8(self.codes8[:, :, :, src.base8 + slot[i8], :],
                                                  self.scale8[:, :, :, src.base8 + slot[i8], :])
        if i4.size:
            out[:, :, :, i4, :] = oq.dequant_int4(
                oq.unpack_nibbles(self.codes4[:, :, :, src.base4 + slot[i4], :]),
                self.scale4[:, :, :, src.base4 + slot[i4], :],
                self.zero4[:, :, :, src.base4 + slot[i4], :])
        valid = (tier != oq.T_PRUNE).astype(np.uint8)
        return out, valid

    # ---- Algorithm 1, one loop body -------------------------------------------
    def step(self, rgb, kv_fp16, frame_id):
        c = self.cfg
        gray = oflow.gray_float(rgb)
        redundant = False
        self.last_gate = None
        self.last_dp = None
        if self.prev_gray is not None:
            d = oflow.flow_from_gray(self.prev_gray, gray, c.flow_levels, c.flow_iters)
            dp = oflow.patch_motion(d, c.grid)
            self.last_dp = dp
            self.last_gate = oflow.gate(dp, c.tau_t, c.theta_r)
            redundant = self.last_gate[2]
        self.prev_gray = gray
        if redundant:
            return self.table.pointer(frame_id)
        scores, _ = self.saliency_pool(rgb)
        self.last_scores = scores
        return self.kv_compress(kv_fp16, scores, frame_id)


def step_tiles(orc: SaliCacheOracle, rgbs, kvs, frame_t):
    """Algorithm 1 for a video frame of T = tiles_per_frame images: one gate over the patches of all
    tiles, then per tile either a pointer entry or saliency -> tiers -> storage.  Entry ids t T + j.
    -> (rows of the T entries, gate or None)."""
    c = orc.cfg
    T = c.tiles_per_frame
    assert len(rgbs) == T and len(kvs) == T
    grays = [oflow.gray_float(r) for r in rgbs]
    redundant, gate = False, None
    orc.last_dp = None
    if orc.prev_tile_grays is not None:
        dps = [oflow.patch_motion(oflow.flow_from_gray(pg, g, c.flow_levels, c.flow_iters), c.grid)
               for pg, g in zip(orc.prev_tile_grays, grays)]
        orc.last_dp = dps
        gate = oflow.gate(np.concatenate(dps), c.tau_t, c.theta_r)          # Eq. 6 over all T * 576 patches
        redundant = gate[2]
    orc.prev_tile_grays = grays
    orc.last_gate = gate
    rows = []
    for j in range(T):
        e = frame_t * T + j
        if redundant:
            rows.append(orc.table.pointer(e))
        else:
            scores, _ = orc.saliency_pool(rgbs[j])
            rows.append(orc.kv_compress(kvs[j], scores, e))
    return rows, gate


class ImageSideOracle:
    """Algorithm 1 without the K/V tensors: everything the image decides.

    Per frame: the temporal filter against the adjacent frame (Eq. 5, Eq. 6, R_frame > theta_R), and
    for a non-redundant frame the saliency scores (Eq. 7), tiers (Eq. 8) and compaction indices;
    then the frame-table row, whose pool bases advance by the tier counts exactly as in
    SaliCacheOracle.kv_compress (same overflow rule).  The pools themselves are not kept, so whole
    workloads at their stated K/V shapes can be walked; `analyze_pair` needs no history and may be
    evaluated for many frames independently, `commit` is the sequential part.
    """

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        self.table = _FrameTable(cfg)
        self.prev_rgb = None

    rows = property(lambda self: self.table.rows)
    cursor = property(lambda self: self.table.cursor)
    last_src = property(lambda self: self.table.last_src)
    overflow = property(lambda self: self.table.overflow)

    def analyze_pair(self, prev_rgb, rgb, tau_t=None, theta_r=None):
        """prev_rgb None = first frame (never redundant).  -> dict(redundant, dp, gate, scores, tier, slot, cnt)."""
        c = self.cfg
        tau_t = c.tau_t if tau_t is None else tau_t
        theta_r = c.theta_r if theta_r is None else theta_r
        out = dict(redundant=False, dp=None, gate=None, scores=None, tier=None, slot=None, cnt=None)
        if prev_rgb is not None:
            d = oflow.flow_from_gray(oflow.gray_float(prev_rgb), oflow.gray_float(rgb), c.flow_levels, c.flow_iters)
            out["dp"] = oflow.patch_motion(d, c.grid)
            out["gate"] = oflow.gate(out["dp"], tau_t, theta_r)
            out["redundant"] = bool(out["gate"][2])
        if out["redundant"]:
            return out                      # Algorithm 1: pointer, then `continue`
        out["scores"], _ = osal.saliency_pool(rgb, c.grid, c.canny_lo, c.canny_hi)
        out["tier"] = assign_tiers(c, out["scores"], self.table.adapt_tau)
        out["slot"], out["cnt"] = oq.slots(out["tier"])
        return out

    def commit(self, frame_id, a) -> FrameRow:
        if a["redundant"]:
            return self.table.pointer(frame_id)
        row = self.table.store(frame_id, a["cnt"])
        if row.stored and self.cfg.tier_mode == 2:
            # (an image-only walk with adaptive thresholds must go frame by frame: analyze_pair of frame t
            # needs the thresholds that frame t - 1 left)
            self.table.adapt_tau = adapted_thresholds(self.cfg, self.table.adapt_tau, a["scores"])
        return row

    def step(self, rgb, frame_id, tau_t=None, theta_r=None):
        a = self.analyze_pair(self.prev_rgb, rgb, tau_t, theta_r)
        self.prev_rgb = rgb
        return self.commit(frame_id, a), a
