"""Thin ctypes binding of libsali (include/sali.h): argument marshalling only.

PyTorch supplies device memory (`tensor.data_ptr()`) and streams
(`torch.cuda.current_stream().cuda_stream`); every step of the method runs in
the library's HIP kernels.  There is no CPU fallback: a missing library or a
non-zero return code raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch   # imported before the library is loaded so that both share one HIP runtime

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsali.so")
_lib = None

TOKENS = 576
MAX_BATCH = 16          # SALI_MAX_BATCH
TIER_FP16, TIER_INT8, TIER_INT4, TIER_PRUNE = 0, 1, 2, 3
FAULT_OVERFLOW, FAULT_NONFINITE, FAULT_NAN_SCORE, FAULT_NO_DATA = 1, 2, 4, 8


class SaliError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {error_string(code)} ({code})")
        self.code = code


class sali_config(C.Structure):
    _fields_ = [
        ("src_h", C.c_int32), ("src_w", C.c_int32), ("grid", C.c_int32),
        ("flow_levels", C.c_int32), ("flow_iters", C.c_int32),
        ("tau_t", C.c_float), ("theta_r", C.c_float),
        ("canny_lo", C.c_int32), ("canny_hi", C.c_int32),
        ("tier_mode", C.c_int32),
        ("tau_high", C.c_float), ("tau_med", C.c_float), ("tau_low", C.c_float),
        ("k_fp16", C.c_int32), ("k_int8", C.c_int32), ("k_int4", C.c_int32),
        ("n_layers", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32), ("group", C.c_int32),
        ("cap_fp16", C.c_int64), ("cap_int8", C.c_int64), ("cap_int4", C.c_int64),
        ("max_frames", C.c_int32), ("budget_tokens", C.c_int32), ("tiles_per_frame", C.c_int32), ("adapt_rate_q8", C.c_int32),
    ]


class sali_gate(C.Structure):
    _fields_ = [("n_static", C.c_int32), ("r_frame", C.c_float), ("redundant", C.c_int32), ("reserved", C.c_int32)]


class sali_frame_row(C.Structure):
    _fields_ = [("frame_id", C.c_int32), ("src", C.c_int32), ("stored", C.c_int32),
                ("base16", C.c_int32), ("base8", C.c_int32), ("base4", C.c_int32),
                ("n16", C.c_int32), ("n8", C.c_int32), ("n4", C.c_int32), ("n_pruned", C.c_int32),
                ("reserved", C.c_int32 * 2)]

    def as_tuple(self):
        return (self.frame_id, self.src, self.stored, self.base16, self.base8, self.base4,
                self.n16, self.n8, self.n4, self.n_pruned)


class sali_pool_layout(C.Structure):
    _fields_ = [("off_fp16", C.c_uint64), ("off_codes8", C.c_uint64), ("off_scale8", C.c_uint64),
                ("off_codes4", C.c_uint64), ("off_scale4", C.c_uint64), ("off_zero4", C.c_uint64),
                ("total_bytes", C.c_uint64)]


EXPORTS = {
    "sali_workspace_bytes": (C.c_int, [C.POINTER(sali_config), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t),
                                       C.POINTER(C.c_size_t)]),
    "sali_pool_offsets": (C.c_int, [C.POINTER(sali_config), C.POINTER(sali_pool_layout)]),
    "sali_create": (C.c_int, [C.POINTER(sali_config), C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]),
    "sali_destroy": (None, [C.c_void_p]),
    "sali_reset": (C.c_int, [C.c_void_p, C.c_void_p]),
    "sali_set_gate_thresholds": (C.c_int, [C.c_void_p, C.c_float, C.c_float]),
    "sali_set_tier_params": (C.c_int, [C.c_void_p, C.c_int32, C.c_float, C.c_float, C.c_float, C.c_int32, C.c_int32,
                                       C.c_int32]),
    "sali_flow_score": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_void_p]),
    "sali_saliency_pool": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sali_kv_compress": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "sali_kv_decompress": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sali_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "sali_analyze": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "sali_analyze_batch": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_int32, C.c_int32, C.c_void_p]),
    "sali_store": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "sali_store_batch": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_int32, C.c_int32, C.c_void_p]),
    "sali_kv_decompress_batch": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_void_p), C.c_void_p,
                                           C.c_void_p]),
    "sali_step_batch": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int32, C.c_int32,
                                  C.c_void_p]),
    "sali_attend_decode": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p,
                                     C.c_void_p, C.c_void_p]),
    "sali_attend_decode_gqa": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                         C.c_void_p, C.c_void_p, C.c_void_p]),
    "sali_attend_decode_static": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_float,
                                            C.c_void_p, C.c_void_p, C.c_void_p]),
    "sali_step_pipelined": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_void_p]),
    "sali_read_frame_table": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]),
    "sali_read_frame_tiers": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sali_read_last_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sali_read_analysis": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sali_set_profile_events": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]),
    "sali_get_status": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32), C.c_void_p]),
    "sali_error_string": (C.c_char_p, [C.c_int]),
}


def load_library():
    """Load libsali.so (built by `python -m paper_2602_14236_amd.build`); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2602_14236_amd.build` first "
                              "(there is no CPU fallback)")
        lib = C.CDLL(_LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def library_path() -> str:
    return _LIB_PATH


def error_string(code: int) -> str:
    return load_library().sali_error_string(code).decode()


def _check(code: int, what: str):
    if code != 0:
        raise SaliError(code, what)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr_array(tensors):
    """Host array of device pointers (the batched entry points read it before they return)."""
    return (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def make_config(src_h, src_w, *, flow_levels=3, flow_iters=3, tau_t=0.5, theta_r=0.90, canny_lo=50, canny_hi=100,
                tier_mode=0, tau_high=0.30, tau_med=0.15, tau_low=0.03, k_fp16=0, k_int8=0, k_int4=0,
                n_layers=1, n_heads=32, cap_fp16=0, cap_int8=0, cap_int4=0, max_frames=1,
                budget_tokens=0, tiles_per_frame=1, adapt_rate_q8=0) -> sali_config:
    return sali_config(src_h, src_w, 24, flow_levels, flow_iters, tau_t, theta_r, canny_lo, canny_hi, tier_mode,
                       tau_high, tau_med, tau_low, k_fp16, k_int8, k_int4, n_layers, n_heads, 128, 32,
                       cap_fp16, cap_int8, cap_int4, max_frames, budget_tokens, tiles_per_frame, adapt_rate_q8)


def workspace_bytes(cfg: sali_config):
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(load_library().sali_workspace_bytes(C.byref(cfg), C.byref(a), C.byref(b), C.byref(c)),
           "sali_workspace_bytes")
    return a.value, b.value, c.value


def pool_offsets(cfg: sali_config) -> sali_pool_layout:
    out = sali_pool_layout()
    _check(load_library().sali_pool_offsets(C.byref(cfg), C.byref(out)), "sali_pool_offsets")
    return out


class SaliContext:
    """Owns the three torch device buffers a context works in and forwards the C calls."""

    def __init__(self, cfg: sali_config, device="cuda:0"):
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        if self.device.type != "cuda":
            raise ValueError("libsali runs on the GPU only")
        sb, pb, tb = workspace_bytes(cfg)
        with torch.cuda.device(self.device):
            self.scratch = torch.empty(sb, dtype=torch.uint8, device=self.device)
            self.pools = torch.empty(pb, dtype=torch.uint8, device=self.device)
            self.tables = torch.zeros(tb, dtype=torch.uint8, device=self.device)
            torch.cuda.synchronize(self.device)
            h = C.c_void_p()
            _check(self.lib.sali_create(C.byref(cfg), _ptr(self.scratch), _ptr(self.pools), _ptr(self.tables),
                                        C.byref(h)), "sali_create")
        self.handle = h
        self.layout = pool_offsets(cfg)
        self.n_planes = cfg.n_layers * 2 * cfg.n_heads

    def close(self):
        if getattr(self, "handle", None):
            torch.cuda.synchronize(self.device)
            self.lib.sali_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the C calls -------------------------------------------------------------------------
    def reset(self):
        _check(self.lib.sali_reset(self.handle, _stream()), "sali_reset")

    def set_gate_thresholds(self, tau_t: float, theta_r: float):
        _check(self.lib.sali_set_gate_thresholds(self.handle, tau_t, theta_r), "sali_set_gate_thresholds")

    def set_tier_params(self, tier_mode, tau_high=0.30, tau_med=0.15, tau_low=0.03, k_fp16=0, k_int8=0, k_int4=0):
        _check(self.lib.sali_set_tier_params(self.handle, tier_mode, tau_high, tau_med, tau_low, k_fp16, k_int8,
                                             k_int4), "sali_set_tier_params")

    def flow_score(self, prev_rgb, cur_rgb, flow_uv, patch_motion, gate_out):
        _check(self.lib.sali_flow_score(self.handle, _ptr(prev_rgb), _ptr(cur_rgb), _ptr(flow_uv),
                                        _ptr(patch_motion), _ptr(gate_out), _stream()), "sali_flow_score")

    def saliency_pool(self, rgb, salmap, scores):
        _check(self.lib.sali_saliency_pool(self.handle, _ptr(rgb), _ptr(salmap), _ptr(scores), _stream()),
               "sali_saliency_pool")

    def kv_compress(self, kv, scores, frame_id: int):
        _check(self.lib.sali_kv_compress(self.handle, _ptr(kv), _ptr(scores), frame_id, _stream()),
               "sali_kv_compress")

    def kv_decompress(self, frame_id: int, out, valid=None):
        _check(self.lib.sali_kv_decompress(self.handle, frame_id, _ptr(out), _ptr(valid), _stream()),
               "sali_kv_decompress")

    def step(self, rgb, kv, frame_id: int):
        _check(self.lib.sali_step(self.handle, _ptr(rgb), _ptr(kv), frame_id, _stream()), "sali_step")

    def analyze(self, rgb, frame_id: int, stream: Optional[torch.cuda.Stream] = None):
        s = _stream() if stream is None else stream.cuda_stream
        _check(self.lib.sali_analyze(self.handle, _ptr(rgb), frame_id, s), "sali_analyze")

    def analyze_batch(self, rgb_frames, first_frame_id: int, stream: Optional[torch.cuda.Stream] = None):
        s = _stream() if stream is None else stream.cuda_stream
        _check(self.lib.sali_analyze_batch(self.handle, _ptr_array(rgb_frames), first_frame_id, len(rgb_frames), s),
               "sali_analyze_batch")

    def attend_decode(self, layer: int, q, frame_lo: int, frame_hi: int, softmax_scale: float, out, lse=None,
                      stream: Optional[torch.cuda.Stream] = None):
        s = _stream() if stream is None else stream.cuda_stream
        _check(self.lib.sali_attend_decode(self.handle, layer, _ptr(q), frame_lo, frame_hi, softmax_scale, _ptr(out),
                                           _ptr(lse), s), "sali_attend_decode")

    def attend_decode_static(self, layer: int, q, frame_lo: int, frame_hi: int, softmax_scale: float, out, lse=None,
                             stream: Optional[torch.cuda.Stream] = None):
        s = _stream() if stream is None else stream.cuda_stream
        _check(self.lib.sali_attend_decode_static(self.handle, layer, _ptr(q), frame_lo, frame_hi, softmax_scale,
                                                  _ptr(out), _ptr(lse), s), "sali_attend_decode_static")

    def attend_decode_gqa(self, layer: int, q, q_per_kv: int, frame_lo: int, frame_hi: int, softmax_scale: float, out,
                          lse=None, stream: Optional[torch.cuda.Stream] = None):
        s = _stream() if stream is None else stream.cuda_stream
        _check(self.lib.sali_attend_decode_gqa(self.handle, layer, _ptr(q), q_per_kv, frame_lo, frame_hi, softmax_scale,
                                               _ptr(out), _ptr(lse), s), "sali_attend_decode_gqa")

    def store_batch(self, kv_frames, first_frame_id: int, stream: Optional[torch.cuda.Stream] = None):
        s = _stream() if stream is None else stream.cuda_stream
        _check(self.lib.sali_store_batch(self.handle, _ptr_array(kv_frames), first_frame_id, len(kv_frames), s),
               "sali_store_batch")

    def kv_decompress_batch(self, first_frame_id: int, out_frames, valid=None,
                            stream: Optional[torch.cuda.Stream] = None):
        s = _stream() if stream is None else stream.cuda_stream
        _check(self.lib.sali_kv_decompress_batch(self.handle, first_frame_id, len(out_frames), _ptr_array(out_frames),
                                                 _ptr(valid), s), "sali_kv_decompress_batch")

    def step_batch(self, rgb_frames, kv_frames, first_frame_id: int, stream: Optional[torch.cuda.Stream] = None):
        s = _stream() if stream is None else stream.cuda_stream
        assert len(rgb_frames) == len(kv_frames)
        _check(self.lib.sali_step_batch(self.handle, _ptr_array(rgb_frames), _ptr_array(kv_frames), first_frame_id,
                                        len(rgb_frames), s), "sali_step_batch")

    def store(self, kv, frame_id: int, stream: Optional[torch.cuda.Stream] = None):
        s = _stream() if stream is None else stream.cuda_stream
        _check(self.lib.sali_store(self.handle, _ptr(kv), frame_id, s), "sali_store")

    def step_pipelined(self, rgb_next, next_frame_id: int, kv, frame_id: int, image_stream: torch.cuda.Stream,
                       kv_stream: torch.cuda.Stream):
        _check(self.lib.sali_step_pipelined(self.handle, _ptr(rgb_next), next_frame_id, _ptr(kv), frame_id,
                                            image_stream.cuda_stream, kv_stream.cuda_stream), "sali_step_pipelined")

    def read_frame_table(self, first=0, count=None):
        count = self.cfg.max_frames - first if count is None else count
        rows = (sali_frame_row * count)()
        _check(self.lib.sali_read_frame_table(self.handle, rows, first, count, _stream()), "sali_read_frame_table")
        return list(rows)

    def read_frame_tiers(self, frame_id: int):
        tier = np.empty(TOKENS, dtype=np.uint8)
        slot = np.empty(TOKENS, dtype=np.uint16)
        _check(self.lib.sali_read_frame_tiers(self.handle, frame_id, tier.ctypes.data_as(C.c_void_p),
                                              slot.ctypes.data_as(C.c_void_p), _stream()), "sali_read_frame_tiers")
        return tier, slot

    def read_last_step(self):
        dp = np.empty(TOKENS, dtype=np.float32)
        sc = np.empty(TOKENS, dtype=np.float32)
        g = sali_gate()
        _check(self.lib.sali_read_last_step(self.handle, dp.ctypes.data_as(C.c_void_p), C.byref(g),
                                            sc.ctypes.data_as(C.c_void_p), _stream()), "sali_read_last_step")
        return dp, g, sc

    def read_analysis(self, frame_id: int):
        """(Delta P [576], gate, scores [576]) of one of the most recently analysed frames."""
        dp = np.empty(TOKENS, dtype=np.float32)
        sc = np.empty(TOKENS, dtype=np.float32)
        g = sali_gate()
        _check(self.lib.sali_read_analysis(self.handle, frame_id, dp.ctypes.data_as(C.c_void_p), C.byref(g),
                                           sc.ctypes.data_as(C.c_void_p), _stream()), "sali_read_analysis")
        return dp, g, sc

    def set_profile_events(self, which: int, start: Optional[torch.cuda.Event], stop: Optional[torch.cuda.Event]):
        """Arm a pair of torch events (created with enable_timing=True and already recorded once, so that
        their HIP handles exist) around the next pack (0) / unpack (1) kernel."""
        a = None if start is None else C.c_void_p(start.cuda_event)
        b = None if stop is None else C.c_void_p(stop.cuda_event)
        _check(self.lib.sali_set_profile_events(self.handle, which, a, b), "sali_set_profile_events")

    def get_status(self) -> int:
        f = C.c_uint32()
        _check(self.lib.sali_get_status(self.handle, C.byref(f), _stream()), "sali_get_status")
        return f.value

    # ---- views of the pool buffer (for inspection; the layout is part of the ABI) ----------------
    def pool_views_flat(self):
        """The six pool arrays as they lie in memory: [cap * n_planes, row], frame-major (a stored frame
        with base b and n rows owns rows [b * P, (b + n) * P), plane p of it rows [b * P + p * n, ...))."""
        c, L, P = self.cfg, self.layout, self.n_planes
        g = c.head_dim // c.group
        buf = self.pools

        def view(off, count, dtype, shape):
            nbytes = count * torch.empty((), dtype=dtype).element_size()
            return buf[off:off + nbytes].view(dtype).view(shape)

        return {
            "fp16": view(L.off_fp16, P * c.cap_fp16 * c.head_dim, torch.float16, (P * c.cap_fp16, c.head_dim)),
            "codes8": view(L.off_codes8, P * c.cap_int8 * c.head_dim, torch.int8, (P * c.cap_int8, c.head_dim)),
            "scale8": view(L.off_scale8, P * c.cap_int8 * g, torch.float32, (P * c.cap_int8, g)),
            "codes4": view(L.off_codes4, P * c.cap_int4 * c.head_dim // 2, torch.uint8,
                           (P * c.cap_int4, c.head_dim // 2)),
            "scale4": view(L.off_scale4, P * c.cap_int4 * g, torch.float32, (P * c.cap_int4, g)),
            "zero4": view(L.off_zero4, P * c.cap_int4 * g, torch.float16, (P * c.cap_int4, g)),
        }

    def pool_views(self, planes=None):
        """Copies of the pools regrouped per plane, [n_planes (or len(planes)), rows used, row], the
        rows of a plane in the order of the frame table (what a plain [plane][cap][row] cache would
        hold): for inspection and tests.  Synchronises the device."""
        torch.cuda.synchronize(self.device)
        P = self.n_planes
        flat = self.pool_views_flat()
        rows = [r for r in self.read_frame_table(0, self.cfg.max_frames) if r.stored]
        which = {"fp16": ("base16", "n16"), "codes8": ("base8", "n8"), "scale8": ("base8", "n8"),
                 "codes4": ("base4", "n4"), "scale4": ("base4", "n4"), "zero4": ("base4", "n4")}
        sel = slice(None) if planes is None else torch.as_tensor(list(planes), device=self.device)
        n_sel = P if planes is None else len(planes)
        out = {}
        for k, a in flat.items():
            fb, fn = which[k]
            used = max([getattr(r, fb) + getattr(r, fn) for r in rows], default=0)
            t = torch.zeros((n_sel, used, a.shape[1]), dtype=a.dtype, device=a.device)
            for r in rows:
                b, n = getattr(r, fb), getattr(r, fn)
                if n > 0:
                    t[:, b:b + n] = a[b * P:(b + n) * P].view(P, n, a.shape[1])[sel]
            out[k] = t
        return out
