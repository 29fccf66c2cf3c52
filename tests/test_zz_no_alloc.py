"""sali_attend_decode_static (partial results in the library's own static device array, nothing
allocated) against sali_attend_decode on the same cache, through the C ABI.  Both run the same
kernels on the same values in the same order, so the results must be bit-identical; two calls in a
row, the second over a smaller range, show that nothing left in the array by one call reaches the
next."""
import math

import numpy as np
import pytest
import torch

from _util import lib_config, params

pytestmark = pytest.mark.gpu


def _cache(n_frames, n_heads, seed):
    from paper_2602_14236_amd import binding
    p = params(96, 96, tier_mode=1, k_fp16=173, k_int8=259, k_int4=100, n_layers=2, n_heads=n_heads,
               cap_fp16=173 * n_frames, cap_int8=259 * n_frames, cap_int4=100 * n_frames, max_frames=n_frames)
    ctx = binding.SaliContext(lib_config(p))
    g = torch.Generator(device="cpu").manual_seed(seed)
    for t in range(n_frames):
        kv = (torch.randn((2, 2, n_heads, 576, 128), generator=g) * 0.7).to(torch.float16)
        ctx.kv_compress(kv.cuda(), torch.rand(576, generator=g).cuda(), t)
    torch.cuda.synchronize()
    return ctx


def _both(ctx, layer, q, lo, hi, sm):
    n_heads = q.shape[0]
    res = []
    for fn in (ctx.attend_decode, ctx.attend_decode_static):
        out = torch.full((n_heads, 128), 7.0, dtype=torch.float32, device="cuda")
        lse = torch.full((n_heads,), 7.0, dtype=torch.float32, device="cuda")
        fn(layer, q, lo, hi, sm, out, lse)
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), lse.cpu().numpy()))
    return res


def test_static_scratch_attention_equals_workspace_attention():
    from paper_2602_14236_amd import binding
    n, nh = 40, 3
    ctx = _cache(n, nh, 11)
    sm = 1.0 / math.sqrt(128.0)
    q = torch.randn((nh, 128), generator=torch.Generator().manual_seed(3)).to(torch.float16).cuda()
    # the larger call first, then smaller ones (fewer partials per head than the call before), an
    # empty range, and the large one again
    for layer, lo, hi in ((0, 0, n), (1, 7, 12), (0, 5, 6), (1, 9, 9), (1, 0, n)):
        print(f"layer {layer} frames [{lo}, {hi})", flush=True)
        (o_ws, l_ws), (o_st, l_st) = _both(ctx, layer, q, lo, hi, sm)
        assert np.array_equal(o_ws.view(np.uint32), o_st.view(np.uint32)), (layer, lo, hi)
        assert np.array_equal(l_ws.view(np.uint32), l_st.view(np.uint32)), (layer, lo, hi)
        if lo == hi:
            assert not o_st.any() and np.all(np.isneginf(l_st))
        else:
            assert np.isfinite(o_st).all() and np.abs(o_st).max() > 0
    assert ctx.get_status() == 0
    ctx.close()
    # a second context on the same GPU shares the array: a smaller cache after the larger one
    ctx2 = _cache(6, 2, 12)
    q2 = torch.randn((2, 128), generator=torch.Generator().manual_seed(4)).to(torch.float16).cuda()
    (o_ws, l_ws), (o_st, l_st) = _both(ctx2, 1, q2, 0, 6, sm)
    assert np.array_equal(o_ws.view(np.uint32), o_st.view(np.uint32))
    assert np.array_equal(l_ws.view(np.uint32), l_st.view(np.uint32))
    ctx2.close()


def test_static_scratch_attention_rejects_what_does_not_fit():
    from paper_2602_14236_amd import binding
    p = params(96, 96, n_layers=1, n_heads=65, cap_fp16=8, cap_int8=8, cap_int4=8, max_frames=1)
    ctx = binding.SaliContext(lib_config(p))
    q = torch.zeros((65, 128), dtype=torch.float16, device="cuda")
    out = torch.zeros((65, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.SaliError) as e:
        ctx.attend_decode_static(0, q, 0, 1, 1.0, out)
    assert e.value.code == -2
    ctx.close()
