"""Oracle: single-query attention over the mixed-precision cache.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Just-In-Time Dequantization says that quantised cache entries are dequantised
while attention is computed, and Implementation Details that the
dequantisation is fused with the attention computation.  The paper gives no
formula beyond that, so the oracle is the plain definition written out:

  for one layer and every head h, with one query vector q_h,
    s_j   = softmax_scale * <q_h, K^_j>           over the cached tokens j
    p     = softmax(s)
    out_h = sum_j p_j V^_j,      lse_h = log sum_j exp(s_j)

where K^, V^ are the dequantised cache entries and everything is float64.

Readings (the paper is silent on all of them):
  * "fused" (Implementation Details) is read as: the dequantised values never
    exist as an fp16 tensor.  K^ = code * scale (INT8), code * scale + zero
    (INT4), taken as exact real numbers of the stored codes, fp32 scales and
    fp16 zero-points; FP16-tier rows are used as stored.  This differs from
    attention over the output of dequantise-on-read (which rounds every value
    to fp16) by at most 2^-11 relative per element; a pin bounds the gap;
  * the cached sequence is the LOGICAL one: frames frame_lo .. frame_hi - 1 in
    order, each contributing the kept tokens of its cache entry.  A redundant
    frame's entry is a pointer (Algorithm 1), so the tokens of its source
    frame appear once more: reuse saves memory, it does not drop the frame
    from the sequence;
  * pruned tokens are not in the cache and take no part in the softmax;
  * grouped-query attention (the 8-KV-head variants of the model family the paper uses): query
    head j reads K/V head j // q_per_kv, nothing else changes;
  * frames that hold no data (never stored, or dropped on overflow)
    contribute nothing; with no token at all out = 0 and lse = -inf.

Pins (tests/test_oracle_attention.py): a library scaled-dot-product attention
on an all-FP16 cache, the uniform-logits closed form (mean of V^, lse = log n),
a dominant key, brute-force Python loops from the raw codes with a pointer
frame and pruned tokens, the log-sum-exp merge of two frame ranges, and the
bounded gap to attention over the dequantise-on-read output.
"""
from __future__ import annotations

import numpy as np

from . import quant as oq


def _dequantised_rows(cache, layer, which, row):
    """The kept tokens of stored frame `row` in pool order, K (which = 0) or V (1):
    float64 [n_heads, n16 + n8 + n4, head_dim], no rounding."""
    g = oq.GROUP
    p16 = cache.pool16[layer, which][:, row.base16:row.base16 + row.n16, :].astype(np.float64)
    c8 = cache.codes8[layer, which][:, row.base8:row.base8 + row.n8, :].astype(np.float64)
    s8 = np.repeat(cache.scale8[layer, which][:, row.base8:row.base8 + row.n8, :].astype(np.float64), g, axis=-1)
    c4 = oq.unpack_nibbles(cache.codes4[layer, which][:, row.base4:row.base4 + row.n4, :]).astype(np.float64)
    s4 = np.repeat(cache.scale4[layer, which][:, row.base4:row.base4 + row.n4, :].astype(np.float64), g, axis=-1)
    z4 = np.repeat(cache.zero4[layer, which][:, row.base4:row.base4 + row.n4, :].astype(np.float64), g, axis=-1)
    return np.concatenate([p16, c8 * s8, c4 * s4 + z4], axis=1)


def cached_tokens(cache, layer, frame_lo, frame_hi):
    """K^, V^ of the logical token sequence of frames [frame_lo, frame_hi):
    two float64 arrays [n_heads, n_tokens, head_dim] (n_tokens may be 0)."""
    ks, vs = [], []
    for f in range(frame_lo, frame_hi):
        row = cache.rows.get(f)
        if row is None or row.src < 0:
            continue
        src = cache.rows[row.src]
        ks.append(_dequantised_rows(cache, layer, 0, src))
        vs.append(_dequantised_rows(cache, layer, 1, src))
    c = cache.cfg
    if not ks:
        empty = np.zeros((c.n_heads, 0, c.head_dim), dtype=np.float64)
        return empty, empty.copy()
    return np.concatenate(ks, axis=1), np.concatenate(vs, axis=1)


def attend_decode(cache, layer, q, frame_lo, frame_hi, softmax_scale, q_per_kv=1):
    """q: [n_heads * q_per_kv, head_dim] (fp16 values); with grouped-query attention query head j
    reads K/V head j // q_per_kv.  -> (out float64 [n_q, head_dim], lse float64 [n_q])."""
    k, v = cached_tokens(cache, layer, frame_lo, frame_hi)
    qf = np.asarray(q).astype(np.float64)
    n_heads, n_tok, d = k.shape
    n_q = n_heads * q_per_kv
    assert qf.shape == (n_q, d)
    out = np.zeros((n_q, d), dtype=np.float64)
    lse = np.full(n_q, -np.inf, dtype=np.float64)
    if n_tok == 0:
        return out, lse
    for j in range(n_q):
        h = j // q_per_kv
        s = float(softmax_scale) * (k[h] @ qf[j])
        m = s.max()
        e = np.exp(s - m)
        z = e.sum()
        out[j] = (e / z) @ v[h]
        lse[j] = m + np.log(z)
    return out, lse
