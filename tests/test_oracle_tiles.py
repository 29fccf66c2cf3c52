"""Pins of the oracle's reading of dynamic-resolution frames (several images of 576 patches per video
frame): one reuse decision over the patches of all tiles, entries per tile (CPU only)."""
import numpy as np

from oracle.cache import OracleConfig, SaliCacheOracle, step_tiles

from _util import drift_frame


def _kv(seed):
    return np.random.default_rng(seed).standard_normal((1, 2, 1, 576, 128)).astype(np.float16)


def _cfg(T, **kw):
    return OracleConfig(src_h=96, src_w=96, flow_levels=2, n_layers=1, n_heads=1, cap_fp16=6000, cap_int8=6000,
                        cap_int4=6000, max_frames=32, tiles_per_frame=T, **kw)


def test_one_tile_is_the_plain_step():
    frames = [drift_frame(0.0), drift_frame(0.0), drift_frame(2.0), drift_frame(2.2)]
    a, b = SaliCacheOracle(_cfg(1)), SaliCacheOracle(_cfg(1))
    for t, f in enumerate(frames):
        kv = _kv(t)
        ra = a.step(f, kv, t)
        (rb,), gate = step_tiles(b, [f], [kv], t)
        assert ra.as_tuple() == rb.as_tuple() and a.last_gate == gate
    assert [a.rows[t].stored for t in range(4)] == [1, 0, 1, 0]


def test_one_decision_for_all_tiles_of_a_frame():
    """Two tiles.  Frame 1: tile 0 unchanged, tile 1 moved by 2 px: 576 of 1152 patches static, R = 0.5, the
    frame is stored whole (tile by tile, tile 0 alone would have been redundant).  Frame 2: both unchanged:
    redundant, each entry points at the last stored entry of its own tile.  Frame 3: both drift 0.3 px:
    still redundant against the adjacent frame."""
    o = SaliCacheOracle(_cfg(2))
    seq = [(0.0, 5.0), (0.0, 7.0), (0.0, 7.0), (0.3, 7.3), (3.0, 7.3)]
    gates = []
    for t, (s0, s1) in enumerate(seq):
        rows, gate = step_tiles(o, [drift_frame(s0), drift_frame(s1)], [_kv(10 * t), _kv(10 * t + 1)], t)
        gates.append(gate)
    st = [o.rows[e].stored for e in range(10)]
    src = [o.rows[e].src for e in range(10)]
    assert st == [1, 1, 1, 1, 0, 0, 0, 0, 1, 1]
    assert src == [0, 1, 2, 3, 2, 3, 2, 3, 8, 9]
    assert gates[0] is None
    n1, r1, red1, _ = gates[1]
    assert 576 <= n1 <= 600 and abs(float(r1) - n1 / 1152.0) < 1e-7 and not red1
    assert gates[2][0] == 1152 and gates[2][2]
    assert gates[3][0] >= 1100 and gates[3][2]
    n4 = gates[4][0]
    assert 560 <= n4 <= 620 and not gates[4][2]           # tile 1 static, tile 0 jumped
    # entries are stored in tile order, pools advance by each entry's counts
    r = [o.rows[e] for e in (0, 1, 2, 3, 8, 9)]
    for a, b in zip(r[:-1], r[1:]):
        assert (b.base16, b.base8, b.base4) == (a.base16 + a.n16, a.base8 + a.n8, a.base4 + a.n4)
    # a pointer entry reads back its own tile's data
    out5, _ = o.kv_decompress(5)
    out3, _ = o.kv_decompress(3)
    assert np.array_equal(out5.view(np.uint16), out3.view(np.uint16))
