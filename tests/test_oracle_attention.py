"""Pins of the attention oracle (Just-In-Time Dequantization: attention over the mixed-precision
cache).  CPU only.  Each test fixes the oracle to something it does not compute itself: a library
attention routine, closed forms, brute-force loops, the log-sum-exp merge identity."""
import math

import numpy as np
import pytest
import torch

from oracle import quant as oq
from oracle.attention import attend_decode, cached_tokens
from oracle.cache import FrameRow, OracleConfig, SaliCacheOracle


def _kv(seed, nl=1, nh=2, n=576, d=128, amp=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((nl, 2, nh, n, d)) * amp).astype(np.float16)


def _q(seed, nh=2, d=128, amp=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((nh, d)) * amp).astype(np.float16)


def _cache(frames=4, **kw):
    base = dict(src_h=96, src_w=96, n_layers=1, n_heads=2, cap_fp16=576 * frames, cap_int8=576 * frames,
                cap_int4=576 * frames, max_frames=frames)
    base.update(kw)
    return SaliCacheOracle(OracleConfig(**base))


def _mixed_scores(seed):
    # thresholds 0.30 / 0.15 / 0.03: all four tiers occur
    rng = np.random.default_rng(seed)
    return (rng.integers(0, 40, 576) / 64.0).astype(np.float32)


def _token_value(cache, src, tok, which, head=0, layer=0):
    """Dequantised K (which = 0) or V (1) of one token of stored frame `src`, from the raw pool
    entries: 128 Python floats, no rounding (None if the token is pruned)."""
    tier, slot = int(cache.tier[src][tok]), int(cache.slot[src][tok])
    row = cache.rows[src]
    if tier == oq.T_PRUNE:
        return None
    if tier == oq.T_FP16:
        return [float(x) for x in cache.pool16[layer, which, head, row.base16 + slot]]
    if tier == oq.T_INT8:
        codes = cache.codes8[layer, which, head, row.base8 + slot]
        scale = cache.scale8[layer, which, head, row.base8 + slot]
        return [int(codes[d]) * float(scale[d // 32]) for d in range(128)]
    packed = cache.codes4[layer, which, head, row.base4 + slot]
    scale = cache.scale4[layer, which, head, row.base4 + slot]
    zero = cache.zero4[layer, which, head, row.base4 + slot]
    out = []
    for d in range(128):
        code = (int(packed[d // 2]) >> (4 * (d % 2))) & 0xF        # element 2k in the low nibble of byte k
        out.append(code * float(scale[d // 32]) + float(zero[d // 32]))
    return out


def _pointer(cache, frame_id):
    """Algorithm 1, redundant frame: the entry is a pointer to the last stored frame."""
    cache.rows[frame_id] = FrameRow(frame_id, cache.last_src, 0)


def test_all_fp16_cache_equals_library_attention():
    c = _cache(frames=2)
    kv0, kv1 = _kv(1), _kv(2)
    ones = np.ones(576, dtype=np.float32)            # every score above tau_high: FP16 tier, stored verbatim
    c.kv_compress(kv0, ones, 0)
    c.kv_compress(kv1, ones, 1)
    q = _q(3)
    scale = 1.0 / math.sqrt(128.0)
    out, lse = attend_decode(c, 0, q, 0, 2, scale)
    k = torch.from_numpy(np.concatenate([kv0[0, 0], kv1[0, 0]], axis=1).astype(np.float64))[None]   # [1, H, N, D]
    v = torch.from_numpy(np.concatenate([kv0[0, 1], kv1[0, 1]], axis=1).astype(np.float64))[None]
    qq = torch.from_numpy(q.astype(np.float64))[None, :, None, :]                                  # [1, H, 1, D]
    ref = torch.nn.functional.scaled_dot_product_attention(qq, k, v, scale=scale)[0, :, 0, :].numpy()
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)
    ref_lse = torch.logsumexp(scale * (k[0] @ qq[0, :, 0, :, None])[..., 0], dim=-1).numpy()
    assert np.allclose(lse, ref_lse, rtol=1e-12)


def test_zero_query_gives_mean_of_cached_values_and_log_count():
    c = _cache(frames=2)
    scores = _mixed_scores(0)
    c.kv_compress(_kv(4), scores, 0)
    c.kv_compress(_kv(5), scores, 1)
    out, lse = attend_decode(c, 0, np.zeros((2, 128), dtype=np.float16), 0, 2, 0.125)
    tier = oq.tiers_threshold(scores, 0.30, 0.15, 0.03)
    n_kept = int((tier != oq.T_PRUNE).sum())
    assert 0 < n_kept < 576
    for head in (0, 1):
        total = np.zeros(128)
        for f in (0, 1):
            for tok in range(576):
                v = _token_value(c, f, tok, 1, head=head)
                if v is not None:
                    total += np.array(v)
        assert np.allclose(out[head], total / (2 * n_kept), rtol=1e-12, atol=1e-14)
    assert np.allclose(lse, math.log(2 * n_kept), rtol=1e-13)


def test_dominant_key_returns_its_value():
    c = _cache(frames=1)
    kv = _kv(6, amp=0.25)
    q = _q(7)
    kv[0, 0, :, 100, :] = q * np.float16(4.0)        # key 100 is 4 q: logit 4 |q|^2 * scale, far above the rest
    c.kv_compress(kv, np.ones(576, dtype=np.float32), 0)
    out, _ = attend_decode(c, 0, q, 0, 1, 1.0)
    assert np.allclose(out, kv[0, 1, :, 100, :].astype(np.float64), atol=1e-9)


def test_brute_force_loops_with_pointer_frame_and_pruned_tokens():
    c = _cache(frames=4, n_heads=1)
    s0, s2 = _mixed_scores(1), _mixed_scores(2)
    c.kv_compress(_kv(8, nh=1), s0, 0)
    _pointer(c, 1)                                   # frame 1 re-uses frame 0
    c.kv_compress(_kv(9, nh=1), s2, 2)
    q = _q(10, nh=1)
    scale = 0.2
    out, lse = attend_decode(c, 0, q, 0, 3, scale)
    # the definition with explicit loops over the logical sequence 0, 1 (= 0 again), 2
    logits, values = [], []
    for f in (0, 1, 2):
        src = c.rows[f].src
        for tok in range(576):
            kvec = _token_value(c, src, tok, 0)
            if kvec is None:
                continue
            logits.append(scale * sum(float(a) * b for a, b in zip(q[0], kvec)))
            values.append(_token_value(c, src, tok, 1))
    m = max(logits)
    w = [math.exp(x - m) for x in logits]
    z = sum(w)
    ref = [sum(wi * vi[d] for wi, vi in zip(w, values)) / z for d in range(128)]
    assert np.allclose(out[0], ref, rtol=1e-10, atol=1e-12)
    assert abs(lse[0] - (m + math.log(z))) < 1e-10
    # the pointer frame counts: dropping it changes the answer
    out_without, _ = attend_decode(c, 0, q, 0, 1, scale)
    k_all, _ = cached_tokens(c, 0, 0, 3)
    n0 = int((c.tier[0] != oq.T_PRUNE).sum())
    n2 = int((c.tier[2] != oq.T_PRUNE).sum())
    assert k_all.shape[1] == 2 * n0 + n2
    assert not np.allclose(out, out_without)


def test_range_starting_inside_a_pointer_run_reads_the_source_outside_the_range():
    c = _cache(frames=4, n_heads=1)
    c.kv_compress(_kv(11, nh=1), _mixed_scores(3), 0)
    _pointer(c, 1)
    _pointer(c, 2)
    q = _q(12, nh=1)
    a, lse_a = attend_decode(c, 0, q, 1, 3, 0.3)     # two copies of frame 0's tokens
    b, lse_b = attend_decode(c, 0, q, 0, 1, 0.3)     # one copy
    assert np.allclose(a, b, rtol=1e-12, atol=1e-14)          # the softmax ignores a uniform multiplicity
    assert np.allclose(lse_a, lse_b + math.log(2.0), rtol=1e-13)


def test_log_sum_exp_merge_of_two_ranges_equals_the_whole():
    c = _cache(frames=4)
    for f in range(4):
        c.kv_compress(_kv(20 + f), _mixed_scores(10 + f), f)
    q = _q(30)
    whole, lse = attend_decode(c, 0, q, 0, 4, 0.15)
    a, la = attend_decode(c, 0, q, 0, 1, 0.15)
    b, lb = attend_decode(c, 0, q, 1, 4, 0.15)
    m = np.maximum(la, lb)
    wa, wb = np.exp(la - m), np.exp(lb - m)
    merged = (a * wa[:, None] + b * wb[:, None]) / (wa + wb)[:, None]
    assert np.allclose(whole, merged, rtol=1e-12, atol=1e-14)
    assert np.allclose(lse, m + np.log(wa + wb), rtol=1e-13)


def test_scale_on_the_logits_equals_scale_on_the_query():
    c = _cache(frames=1)
    c.kv_compress(_kv(40), _mixed_scores(4), 0)
    q = _q(41)
    a, la = attend_decode(c, 0, q, 0, 1, 0.25)
    b, lb = attend_decode(c, 0, (q * np.float16(2.0)).astype(np.float16), 0, 1, 0.125)   # doubling is exact in fp16
    assert np.allclose(a, b, rtol=1e-13, atol=0) and np.allclose(la, lb, rtol=1e-13)


def test_layers_and_heads_are_independent():
    c = _cache(frames=1, n_layers=2, n_heads=3)
    kv = _kv(50, nl=2, nh=3)
    c.kv_compress(kv, _mixed_scores(5), 0)
    q = _q(51, nh=3)
    out1, _ = attend_decode(c, 1, q, 0, 1, 0.1)
    # the same data as a one-layer, one-head cache
    c1 = _cache(frames=1, n_layers=1, n_heads=1)
    c1.kv_compress(kv[1:2, :, 2:3], _mixed_scores(5), 0)
    ref, _ = attend_decode(c1, 0, q[2:3], 0, 1, 0.1)
    assert np.array_equal(out1[2], ref[0])


def test_empty_cache_range():
    c = _cache(frames=3)
    c.kv_compress(_kv(60), np.zeros(576, dtype=np.float32), 0)     # every token pruned
    c.rows[1] = FrameRow(1, -1, 0)                                 # dropped frame
    out, lse = attend_decode(c, 0, _q(61), 0, 3, 1.0)
    assert not out.any() and np.all(np.isneginf(lse))


def test_gap_to_attention_over_dequantise_on_read_output_is_bounded():
    """The fused reading uses unrounded dequantised values; dequantise-on-read rounds each to fp16
    (relative 2^-11).  The two attentions must agree to about that, and they must not be equal
    (otherwise the reading would not matter)."""
    c = _cache(frames=2)
    for f in range(2):
        c.kv_compress(_kv(70 + f), _mixed_scores(20 + f), f)
    q = _q(71)
    scale = 1.0 / math.sqrt(128.0)
    out, _ = attend_decode(c, 0, q, 0, 2, scale)
    ks, vs = [], []
    for f in range(2):
        dense, valid = c.kv_decompress(f)
        ks.append(dense[0, 0][:, valid == 1, :].astype(np.float64))
        vs.append(dense[0, 1][:, valid == 1, :].astype(np.float64))
    k, v = np.concatenate(ks, axis=1), np.concatenate(vs, axis=1)
    ref = np.zeros_like(out)
    for h in range(2):
        s_ = scale * (k[h] @ q[h].astype(np.float64))
        e = np.exp(s_ - s_.max())
        ref[h] = (e / e.sum()) @ v[h]
    gap = np.abs(out - ref).max()
    assert 0.0 < gap < 2e-3 * np.abs(v).max()


def test_grouped_queries_equal_plain_attention_on_a_cache_with_repeated_heads():
    """q_per_kv query heads share one K/V head: the same numbers must come out of the plain path
    on a cache whose K/V heads were repeated q_per_kv times before storing."""
    g = 4
    kv = _kv(80, nh=2)
    scores = _mixed_scores(30)
    c = _cache(frames=1, n_heads=2)
    c.kv_compress(kv, scores, 0)
    q = _q(81, nh=2 * g)
    out, lse = attend_decode(c, 0, q, 0, 1, 0.11, q_per_kv=g)
    wide = _cache(frames=1, n_heads=2 * g)
    wide.kv_compress(np.repeat(kv, g, axis=2), scores, 0)          # head j of the wide cache = head j // g
    ref, ref_lse = attend_decode(wide, 0, q, 0, 1, 0.11)
    assert out.shape == (2 * g, 128)
    assert np.array_equal(out, ref) and np.array_equal(lse, ref_lse)
    # and the heads of a group really see different queries
    assert not np.allclose(out[0], out[1])


def test_fp16_operand_error_bound_holds_for_an_emulated_matrix_core_path():
    """The tolerance used for the matrix-core attention kernel (operands K^, V^ and the softmax
    weights rounded to fp16, accumulation in higher precision) is derived to first order; here the
    same roundings are applied in NumPy and the result must stay inside the bound, with room to
    spare, on a cache with all tiers, a pointer frame and a sharp softmax."""
    from _util import fp16_operand_bounds
    cache = _cache(frames=4)
    for f in range(3):
        cache.kv_compress(_kv(50 + f, amp=0.8), _mixed_scores(60 + f), f)
    _pointer(cache, 3)
    for scale, seed in ((1.0 / math.sqrt(128.0), 1), (0.6, 2)):       # the second one: a few tokens dominate
        q = np.concatenate([_q(seed, nh=2), _q(seed + 10, nh=2)]).reshape(2, 2, 128).transpose(1, 0, 2).reshape(4, 128)
        exact, exact_lse = attend_decode(cache, 0, q, 0, 4, scale, q_per_kv=2)
        k, v = cached_tokens(cache, 0, 0, 4)
        k16 = k.astype(np.float16).astype(np.float64)
        v16 = v.astype(np.float16).astype(np.float64)
        out = np.zeros_like(exact)
        lse = np.zeros_like(exact_lse)
        for j in range(4):
            h = j // 2
            s = scale * (k16[h] @ q[j].astype(np.float64))
            m = s.max()
            p = np.exp(s - m)
            p16 = p.astype(np.float16).astype(np.float64)
            out[j] = (p16 @ v16[h]) / p.sum()
            lse[j] = m + math.log(p.sum())
        bound, lse_bound = fp16_operand_bounds(cache, q, 0, 4, scale, 2)
        err = np.abs(out - exact)
        assert err.max() > 0.0 and np.all(err <= bound), (err.max(), float((bound / np.maximum(err, 1e-300)).min()))
        assert np.all(np.abs(lse - exact_lse) <= lse_bound)
        assert float((bound / np.maximum(err, 1e-300)).min()) > 4.0      # the worst case is not what typically happens

