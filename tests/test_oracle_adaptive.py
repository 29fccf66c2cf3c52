"""Pins of the oracle's adaptive-threshold mode (tier_mode 2; CPU only).  The paper names adaptive
thresholds as future work and gives no rule; the rule pinned here is the library's reading: Eq. 8 with
the thresholds in force, which after every stored frame move a fraction alpha of the way to the score
quantiles that would have met the target tier shares."""
import numpy as np

from oracle import quant as oq
from oracle.cache import OracleConfig, SaliCacheOracle, adapted_thresholds, assign_tiers, to_lattice


def _cfg(**kw):
    base = dict(src_h=96, src_w=96, n_layers=1, n_heads=1, cap_fp16=20000, cap_int8=20000, cap_int4=20000, max_frames=64,
                tier_mode=2, k_fp16=100, k_int8=150, k_int4=200, adapt_rate_q8=128)
    base.update(kw)
    return OracleConfig(**base)


def _kv(seed):
    return np.random.default_rng(seed).standard_normal((1, 2, 1, 576, 128)).astype(np.float16)


def _lattice_scores(rng, hi=65536):
    return (rng.integers(0, hi + 1, 576) / 65536.0).astype(np.float32)


def test_rate_zero_is_eq8_with_the_configured_thresholds():
    rng = np.random.default_rng(1)
    a = SaliCacheOracle(_cfg(adapt_rate_q8=0))
    b = SaliCacheOracle(_cfg(tier_mode=0))
    for f in range(4):
        s = _lattice_scores(rng)
        ra, rb = a.kv_compress(_kv(f), s, f), b.kv_compress(_kv(f), s, f)
        assert ra.as_tuple() == rb.as_tuple() and np.array_equal(a.tier[f], b.tier[f])
    assert a.table.adapt_tau == [to_lattice(0.30), to_lattice(0.15), to_lattice(0.03)] == [19660, 9830, 1966]


def test_rate_one_meets_the_targets_on_a_repeated_frame():
    """alpha = 1: the thresholds become the frame's quantiles, so the same scores (all distinct) presented
    again fall into the tiers with exactly the target counts."""
    rng = np.random.default_rng(2)
    s = (rng.permutation(576) * 100 / 65536.0).astype(np.float32)          # distinct lattice values
    o = SaliCacheOracle(_cfg(adapt_rate_q8=256))
    r0 = o.kv_compress(_kv(0), s, 0)
    assert (r0.n16, r0.n8, r0.n4) != (100, 150, 200)                       # the configured thresholds do not meet them
    r1 = o.kv_compress(_kv(1), s, 1)
    assert (r1.n16, r1.n8, r1.n4, r1.npr) == (100, 150, 200, 126)
    assert np.array_equal(o.tier[1], oq.tiers_topk(s, 100, 150, 200))       # = the top-k assignment


def test_geometric_approach_to_a_fixed_quantile():
    """Constant scores: the distance of a threshold to its quantile shrinks by (1 - alpha) per stored frame
    (up to the floor of the lattice arithmetic), monotonically, from above and from below."""
    rng = np.random.default_rng(3)
    s = (rng.permutation(576) * 100 / 65536.0).astype(np.float32)
    cfg = _cfg(adapt_rate_q8=64, tau_high=0.9, tau_med=0.5, tau_low=0.0)
    order = sorted(range(576), key=lambda i: (-float(s[i]), i))
    q = [to_lattice(s[order[r]]) for r in (100, 250, 450)]
    tau = [to_lattice(0.9), to_lattice(0.5), 0]
    t = list(tau)
    for step in range(1, 30):
        t = adapted_thresholds(cfg, t, s)
        for k in range(3):
            exact = q[k] + (tau[k] - q[k]) * 0.75 ** step
            assert abs(t[k] - exact) <= step + 1                            # one lattice unit of floor per step
            assert min(tau[k], q[k]) <= t[k] <= max(tau[k], q[k])
    assert t[0] >= t[1] >= t[2]
    assert abs(t[1] - q[1]) < 40


def test_update_rule_by_hand_and_missing_rank():
    cfg = _cfg(k_fp16=2, k_int8=1, k_int4=573, adapt_rate_q8=128)
    s = np.zeros(576, dtype=np.float32)
    s[[5, 9, 11]] = [0.75, 0.5, 0.25]
    # ranks: 5, 9, 11, then the zeros by index.  q_high = score of rank 2 = 0.25 -> 16384; q_med = rank 3 = 0;
    # q_low = rank 576 does not exist -> 0
    out = adapted_thresholds(cfg, [19660, 9830, 1966], s)
    assert out == [19660 + (16384 - 19660) * 128 // 256, 9830 + (0 - 9830) * 128 // 256, 1966 + (0 - 1966) * 128 // 256]
    assert out == [18022, 4915, 983]
    # tiers come from the thresholds in force, strict '>' as printed in Eq. 8
    tier = assign_tiers(cfg, np.array([18023, 18022, 4916, 4915, 984, 983, 0], dtype=np.float32) / 65536.0, out)
    assert list(tier) == [0, 1, 1, 2, 2, 3, 3]


def test_pointer_frames_leave_the_thresholds_alone():
    from _util import drift_frame
    o = SaliCacheOracle(OracleConfig(src_h=96, src_w=96, flow_levels=2, n_layers=1, n_heads=1, cap_fp16=9000, cap_int8=9000,
                                     cap_int4=9000, max_frames=8, tier_mode=2, k_fp16=100, k_int8=150, k_int4=200,
                                     adapt_rate_q8=128))
    o.step(drift_frame(0.0), _kv(0), 0)
    t1 = list(o.table.adapt_tau)
    assert t1 != [19660, 9830, 1966]
    row = o.step(drift_frame(0.0), _kv(1), 1)
    assert row.stored == 0 and o.table.adapt_tau == t1
    o.step(drift_frame(3.0), _kv(2), 2)
    assert o.table.adapt_tau != t1
