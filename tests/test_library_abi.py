"""CPU-only checks of the boundary: the library loads, exports every symbol the header declares,
and its host-only entry points validate their arguments."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "sali.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sali_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2602_14236_amd import binding
    lib = binding.load_library()
    names = _declared_symbols()
    assert {"sali_flow_score", "sali_saliency_pool", "sali_kv_compress", "sali_kv_decompress", "sali_step"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(binding.EXPORTS) == set(names)


def test_host_only_calls():
    from paper_2602_14236_amd import binding
    cfg = binding.make_config(336, 336, n_layers=32, n_heads=32, tier_mode=1, k_fp16=173, k_int8=403,
                              cap_fp16=173 * 64, cap_int8=403 * 64, max_frames=64)
    scratch, pools, tables = binding.workspace_bytes(cfg)
    lay = binding.pool_offsets(cfg)
    planes = 32 * 2 * 32
    assert lay.off_fp16 == 0
    assert lay.off_codes8 >= planes * 173 * 64 * 256
    assert lay.off_scale8 - lay.off_codes8 >= planes * 403 * 64 * 128
    assert pools == lay.total_bytes >= planes * 64 * (173 * 256 + 403 * 144)
    assert scratch > 336 * 336 * 4 * 24 and tables > 64 * 576 * 5
    for bad in (dict(src_h=10), dict(flow_levels=0), dict(canny_lo=0), dict(tier_mode=3), dict(adapt_rate_q8=257), dict(tiles_per_frame=9), dict(n_heads=0),
                dict(max_frames=0), dict(tau_low=0.5), dict(flow_levels=6, src_h=24, src_w=24),
                dict(cap_fp16=1 << 24), dict(cap_int4=(1 << 24) + 5)):       # a pool plane stays under 4 GiB
        kw = dict(src_h=336, src_w=336)
        kw.update(bad)
        h, w = kw.pop("src_h"), kw.pop("src_w")
        with pytest.raises(binding.SaliError) as e:
            binding.workspace_bytes(binding.make_config(h, w, **kw))
        assert e.value.code == -4
    assert binding.error_string(0) == "ok" and "align" in binding.error_string(-3)


def test_struct_sizes_match_header():
    import ctypes
    from paper_2602_14236_amd import binding
    assert ctypes.sizeof(binding.sali_frame_row) == 48
    assert ctypes.sizeof(binding.sali_gate) == 16
    assert ctypes.sizeof(binding.sali_config) == 120
    assert ctypes.sizeof(binding.sali_pool_layout) == 56
