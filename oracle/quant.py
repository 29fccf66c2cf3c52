"""Oracle: tier assignment, compaction indices, mixed-precision quantisation.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Follows Spatial Filtering via Saliency-Guided Quantization (Eq. 8), Algorithm 1
("store (K_i, V_i) with precision Q(s_i)") and Implementation Details
(symmetric min-max INT8, asymmetric INT4).  The paper leaves granularity,
rounding and storage format open; the readings taken are:

  * one decision per patch/token, shared by K and V, all layers and heads;
  * quantisation group = 32 consecutive head-dim values of one token in one
    (layer, K|V, head); fp32 scale per group, fp16 zero-point (= group minimum,
    itself an fp16 input value) for INT4;
  * every floating-point step is ONE IEEE fp32 operation, in this order:
      INT8  m = max|x|; scale = m / 127; inv = 127 / m; q = clamp(rne(x * inv), -127, 127)
            dequant  x^ = float(q) * scale
      INT4  mn = min x; mx = max x; range = mx - mn; scale = range / 15; inv = 15 / range;
            q = clamp(rne((x - mn) * inv), 0, 15)
            dequant  x^ = fma(float(q), scale, mn)   (single rounding)
    m == 0 (resp. range == 0) gives scale 0 and all codes 0;
  * dequantised values are rounded to fp16 (nearest-even); FP16-tier rows are
    stored verbatim; pruned rows read back as zeros with valid = 0.

Tier codes: 0 = FP16, 1 = INT8, 2 = INT4, 3 = PRUNE.
"""
from __future__ import annotations

import numpy as np

T_FP16, T_INT8, T_INT4, T_PRUNE = 0, 1, 2, 3
GROUP = 32


# ---------------------------------------------------------------------------
# tiers and compaction indices
# ---------------------------------------------------------------------------
def tiers_threshold(scores, tau_high, tau_med, tau_low):
    """Eq. 8 with the inequalities as printed, evaluated in fp32."""
    s = np.asarray(scores, dtype=np.float32)
    if np.isnan(s).any():
        raise ValueError("NaN score")
    th, tm, tl = np.float32(tau_high), np.float32(tau_med), np.float32(tau_low)
    tier = np.full(s.shape, T_PRUNE, dtype=np.uint8)
    tier[s > tl] = T_INT4          # tau_low < s <= tau_med
    tier[s > tm] = T_INT8          # tau_med < s <= tau_high
    tier[s > th] = T_FP16          # s > tau_high
    return tier


def tiers_topk(scores, k_fp16, k_int8, k_int4):
    """Fraction mode (benchmark configs, not in the paper): rank tokens by
    (score descending, token index ascending); the first k_fp16 are FP16, the
    next k_int8 INT8, the next k_int4 INT4, the rest pruned."""
    s = np.asarray(scores, dtype=np.float32)
    if np.isnan(s).any():
        raise ValueError("NaN score")
    n = s.size
    if min(k_fp16, k_int8, k_int4) < 0 or k_fp16 + k_int8 + k_int4 > n:
        raise ValueError("bad k")
    order = sorted(range(n), key=lambda i: (-float(s[i]), i))
    tier = np.full(n, T_PRUNE, dtype=np.uint8)
    for rank, i in enumerate(order):
        if rank < k_fp16:
            tier[i] = T_FP16
        elif rank < k_fp16 + k_int8:
            tier[i] = T_INT8
        elif rank < k_fp16 + k_int8 + k_int4:
            tier[i] = T_INT4
    return tier


def slots(tier):
    """slot_i = number of tokens j < i in the same tier; counts per tier (n16, n8, n4, np)."""
    tier = np.asarray(tier)
    slot = np.zeros(tier.size, dtype=np.int32)
    counts = np.zeros(4, dtype=np.int32)
    for i, t in enumerate(tier):
        slot[i] = counts[t]
        counts[t] += 1
    return slot, counts


# ---------------------------------------------------------------------------
# group quantisers (last axis of x is split into groups of 32)
# ---------------------------------------------------------------------------
def _groups(x_fp16):
    x = np.asarray(x_fp16)
    if x.dtype != np.float16:
        raise TypeError("fp16 input expected")
    if x.shape[-1] % GROUP:
        raise ValueError("last axis must be a multiple of 32")
    xg = x.reshape(x.shape[:-1] + (x.shape[-1] // GROUP, GROUP)).astype(np.float32)   # exact widening
    return xg


def quant_int8(x_fp16):
    """-> codes int8 [..., D], scale fp32 [..., D/32]."""
    xg = _groups(x_fp16)
    m = np.max(np.abs(xg), axis=-1)                                  # fp32, exact
    nz = m > 0
    with np.errstate(divide="ignore", invalid="ignore"):
        scale = np.where(nz, m / np.float32(127.0), np.float32(0.0)).astype(np.float32)
        inv = np.where(nz, np.float32(127.0) / m, np.float32(0.0)).astype(np.float32)
    prod = (xg * inv[..., None]).astype(np.float32)                  # one fp32 multiply
    q = np.clip(np.rint(prod), -127, 127).astype(np.int8)            # round half to even
    return q.reshape(x_fp16.shape), scale


def dequant_int8(codes, scale):
    """-> fp16 [..., D]."""
    qg = codes.reshape(codes.shape[:-1] + (codes.shape[-1] // GROUP, GROUP)).astype(np.float32)
    xh = (qg * scale[..., None].astype(np.float32)).astype(np.float32)   # one fp32 multiply
    return xh.astype(np.float16).reshape(codes.shape)


def quant_int4(x_fp16):
    """-> codes uint8 in [0, 15] [..., D] (unpacked), scale fp32 [..., D/32], zero fp16 [..., D/32]."""
    xg = _groups(x_fp16)
    mn = np.min(xg, axis=-1)
    mx = np.max(xg, axis=-1)
    rng = (mx - mn).astype(np.float32)                               # one fp32 subtract
    nz = rng > 0
    with np.errstate(divide="ignore", invalid="ignore"):
        scale = np.where(nz, rng / np.float32(15.0), np.float32(0.0)).astype(np.float32)
        inv = np.where(nz, np.float32(15.0) / rng, np.float32(0.0)).astype(np.float32)
    diff = (xg - mn[..., None]).astype(np.float32)                   # one fp32 subtract
    prod = (diff * inv[..., None]).astype(np.float32)                # one fp32 multiply
    q = np.clip(np.rint(prod), 0, 15).astype(np.uint8)
    zero = mn.astype(np.float16)                                     # lossless: mn is an fp16 input value
    return q.reshape(x_fp16.shape), scale, zero


def dequant_int4(codes, scale, zero):
    """-> fp16 [..., D].  x^ = fma(q, scale, zero): the product q*scale (<= 28 significant bits)
    and the sum with an fp16 zero-point are exact in float64, so one float64 -> fp32 rounding
    is the correctly rounded fused multiply-add."""
    qg = codes.reshape(codes.shape[:-1] + (codes.shape[-1] // GROUP, GROUP)).astype(np.float64)
    exact = qg * scale[..., None].astype(np.float64) + zero[..., None].astype(np.float64)
    xh = exact.astype(np.float32)
    return xh.astype(np.float16).reshape(codes.shape)


def pack_nibbles(codes):
    """Element 2j in the low nibble, 2j+1 in the high nibble of byte j."""
    c = np.asarray(codes, dtype=np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(packed):
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = p & 0x0F
    out[..., 1::2] = p >> 4
    return out


def has_nonfinite(x_fp16):
    return not np.isfinite(np.asarray(x_fp16, dtype=np.float32)).all()


def compressed_bytes_per_plane(n16, n8, n4, head_dim=128):
    """Stored bytes of one frame in one (layer, K|V, head): fp16 rows, int8 codes + fp32 scales,
    int4 codes + fp32 scales + fp16 zeros."""
    g = head_dim // GROUP
    return n16 * head_dim * 2 + n8 * (head_dim + 4 * g) + n4 * (head_dim // 2 + 4 * g + 2 * g)
