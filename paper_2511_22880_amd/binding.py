"""ctypes binding of include/lora.h: same names, argument marshalling only.

Device buffers come from the caller (torch tensors, or raw integer addresses); every step of the
path runs in the library's kernels.  A non-OK status raises ``LoraError`` carrying the status name
and the library's detail line.  Loading fails loudly when the shared library has not been built.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# LORA_GFX950_LIB selects another build of the same library (the measurement build with device clocks)
LIB_PATH = os.environ.get("LORA_GFX950_LIB") or os.path.join(_PKG, "liblora_gfx950.so")

LORA_MAX_RANK = 256
LORA_BF16 = 1
STATUS = ("LORA_OK", "LORA_ERR_INVALID_ARG", "LORA_ERR_SHAPE", "LORA_ERR_OOM", "LORA_ERR_NOT_RESIDENT",
          "LORA_ERR_STALE_SEGMENTS", "LORA_ERR_WORKSPACE", "LORA_ERR_DEVICE")

# every symbol include/lora.h declares
EXPORTS = (
    "lora_pool_bytes", "lora_pool_create", "lora_pool_create_live", "lora_pool_load", "lora_pool_evict",
    "lora_pool_reserve", "lora_pool_mark_resident", "lora_pool_space", "lora_pool_compact", "lora_pool_adapter_info",
    "lora_pool_destroy", "lora_pool_load_staging_bytes", "lora_pool_load_staged", "lora_segments_plan",
    "lora_segments_plan_opts", "lora_segments_set_options", "lora_segments_table_bytes", "lora_segments_upload_to",
    "lora_segments_build_opts", "lora_segments_plan_multi_opts", "lora_segments_build_multi_opts", "lora_segments_plan_ranges", "lora_segments_upload",
    "lora_segments_build", "lora_segments_build_ranges", "lora_segments_rebuild", "lora_segments_info",
    "lora_segments_export", "lora_segments_export_units", "lora_segments_export_launch_units", "lora_segments_destroy", "lora_workspace_bytes",
    "lora_shrink", "lora_expand", "lora_apply_workspace_bytes", "lora_apply", "lora_apply_static", "lora_linear_pack_weight", "lora_linear",
    "lora_profile_next_apply",
    "lora_segments_plan_multi", "lora_segments_build_multi", "lora_apply_multi",
    "lora_set_fused_apply", "lora_set_decode_single_launch", "lora_set_whole_k_limit", "lora_segments_check", "lora_set_side_stream", "lora_set_merged_launches", "lora_set_fused_wait_limit",
    "lora_status_string",
    "lora_last_error",
    "lora_place_extrapolate", "lora_place_assign",
)


class LoraError(RuntimeError):
    def __init__(self, status: int, detail: str):
        self.status = status
        self.status_name = STATUS[status] if 0 <= status < len(STATUS) else f"status {status}"
        self.detail = detail
        super().__init__(f"{self.status_name}: {detail}")


class _Desc(ctypes.Structure):
    _fields_ = [("in_features", ctypes.c_int32), ("out_features", ctypes.c_int32), ("n_adapters", ctypes.c_int32),
                ("ranks", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("dtype", ctypes.c_int32)]


class _AdapterInfo(ctypes.Structure):
    _fields_ = [("a_offset", ctypes.c_uint64), ("b_offset", ctypes.c_uint64), ("rank", ctypes.c_int32),
                ("rank_padded", ctypes.c_int32), ("scale", ctypes.c_float), ("resident", ctypes.c_int32)]


class _SegInfo(ctypes.Structure):
    _fields_ = [("n_tokens", ctypes.c_int32), ("n_active", ctypes.c_int32), ("n_segments", ctypes.c_int32),
                ("n_shrink_units", ctypes.c_int32), ("n_expand_units", ctypes.c_int32),
                ("n_k_slices", ctypes.c_int32), ("v_floats", ctypes.c_int64), ("weight_bytes", ctypes.c_int64),
                ("single_launch", ctypes.c_int32), ("launch_work_groups", ctypes.c_int32)]


class _PlanOptions(ctypes.Structure):
    _fields_ = [("whole_k_limit", ctypes.c_int32), ("merged_launches", ctypes.c_int32), ("side_stream", ctypes.c_int32),
                ("fused_apply", ctypes.c_int32), ("decode_single_launch", ctypes.c_int32),
                ("fused_wait_limit", ctypes.c_uint32), ("whole_k_max_in", ctypes.c_int32),
                ("heavy_min_tokens", ctypes.c_int32), ("heavy_min_batch", ctypes.c_int32),
                ("heavy_k_cut_max_units", ctypes.c_int32), ("big_runs_max_units", ctypes.c_int32)]


def plan_options(whole_k_limit: int = -1, merged_launches: int = -1, side_stream: int = -1, fused_apply: int = -1,
                 decode_single_launch: int = -1, fused_wait_limit: int = 0, whole_k_max_in: int = -1,
                 heavy_min_tokens: int = -1, heavy_min_batch: int = -1, heavy_k_cut_max_units: int = -1,
                 big_runs_max_units: int = -1) -> _PlanOptions:
    """lora_plan_options_t; -1 (0 for the wait limit) = the process-wide default or the built-in threshold."""
    return _PlanOptions(int(whole_k_limit), int(merged_launches), int(side_stream), int(fused_apply),
                        int(decode_single_launch), int(fused_wait_limit), int(whole_k_max_in), int(heavy_min_tokens),
                        int(heavy_min_batch), int(heavy_k_cut_max_units), int(big_runs_max_units))


def _opts(options):
    return ctypes.byref(options) if options is not None else None


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2511_22880_amd.build` "
                              "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        for name in EXPORTS:
            fn = getattr(L, name)
            fn.restype = ctypes.c_char_p if name in ("lora_status_string", "lora_last_error") else ctypes.c_int
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != 0:
        raise LoraError(status, lib().lora_last_error().decode("utf-8", "replace"))


def _ptr(obj) -> ctypes.c_void_p:
    """Address of a torch tensor, a numpy array, or an integer address; None -> NULL."""
    if obj is None:
        return ctypes.c_void_p(None)
    if isinstance(obj, ctypes.c_void_p):
        return obj
    if isinstance(obj, int):
        return ctypes.c_void_p(obj)
    if isinstance(obj, np.ndarray):
        return ctypes.c_void_p(obj.ctypes.data)
    if hasattr(obj, "data_ptr"):
        return ctypes.c_void_p(obj.data_ptr())
    raise TypeError(f"cannot take the address of {type(obj)}")


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        return ctypes.c_void_p(None)
    if hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    return ctypes.c_void_p(int(stream) or None)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


class Pool:
    """Handle of a lora_pool_t plus the objects that must outlive it (arena tensor, desc arrays)."""

    def __init__(self, handle, in_features, out_features, ranks, scales, arena):
        self.handle = handle
        self.in_features, self.out_features = in_features, out_features
        self.ranks, self.scales = ranks, scales
        self.arena = arena

    @property
    def n_adapters(self) -> int:
        return int(self.ranks.shape[0])


class Segments:
    def __init__(self, handle, pool: Pool):
        self.handle = handle
        self.pool = pool


def _desc(in_features, out_features, ranks, scales):
    ranks = _i32(ranks)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    if ranks.shape != scales.shape:
        raise ValueError("ranks and scales differ in length")
    d = _Desc(int(in_features), int(out_features), int(ranks.shape[0]), ranks.ctypes.data, scales.ctypes.data,
              LORA_BF16)
    return d, ranks, scales


def lora_pool_bytes(in_features: int, out_features: int, ranks, scales) -> int:
    d, _r, _s = _desc(in_features, out_features, ranks, scales)
    n = ctypes.c_size_t(0)
    _check(lib().lora_pool_bytes(ctypes.byref(d), ctypes.byref(n)))
    return int(n.value)


def lora_pool_create(in_features: int, out_features: int, ranks, scales, dev_arena, arena_bytes: Optional[int] = None) -> Pool:
    """dev_arena: a torch device tensor (uint8/any dtype) or an integer device address."""
    d, r, s = _desc(in_features, out_features, ranks, scales)
    if arena_bytes is None:
        arena_bytes = dev_arena.numel() * dev_arena.element_size()
    h = ctypes.c_void_p(None)
    _check(lib().lora_pool_create(ctypes.byref(d), _ptr(dev_arena), ctypes.c_size_t(arena_bytes), ctypes.byref(h)))
    return Pool(h, int(in_features), int(out_features), r, s, dev_arena)


def lora_pool_create_live(in_features: int, out_features: int, ranks, scales, dev_arena,
                          arena_bytes: Optional[int] = None) -> Pool:
    """A pool over an arena of any size: adapters get their place when loaded (see include/lora.h)."""
    d, r, s = _desc(in_features, out_features, ranks, scales)
    if arena_bytes is None:
        arena_bytes = dev_arena.numel() * dev_arena.element_size()
    h = ctypes.c_void_p(None)
    _check(lib().lora_pool_create_live(ctypes.byref(d), _ptr(dev_arena), ctypes.c_size_t(arena_bytes), ctypes.byref(h)))
    return Pool(h, int(in_features), int(out_features), r, s, dev_arena)


def lora_pool_reserve(pool: Pool, adapter: int) -> None:
    _check(lib().lora_pool_reserve(pool.handle, ctypes.c_int32(adapter)))


def lora_pool_space(pool: Pool) -> dict:
    fr, lg = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().lora_pool_space(pool.handle, ctypes.byref(fr), ctypes.byref(lg)))
    return {"free_bytes": int(fr.value), "largest_free_bytes": int(lg.value)}


def lora_pool_compact(pool: Pool, scratch=None, stream=None, scratch_bytes: Optional[int] = None) -> int:
    """Returns the number of adapters that were moved."""
    moved = ctypes.c_int32(0)
    nbytes = (_nbytes(scratch) if scratch is not None else 0) if scratch_bytes is None else scratch_bytes
    _check(lib().lora_pool_compact(pool.handle, _ptr(scratch), ctypes.c_size_t(nbytes), _stream(stream),
                                   ctypes.byref(moved)))
    return int(moved.value)


def lora_pool_load(pool: Pool, adapter: int, A, B, src_is_device: Optional[bool] = None, stream=None) -> None:
    """A [in][rank], B [rank][out] bf16: numpy uint16 arrays (host) or torch device tensors."""
    if src_is_device is None:
        src_is_device = not isinstance(A, np.ndarray)
    if isinstance(A, np.ndarray):
        A, B = np.ascontiguousarray(A), np.ascontiguousarray(B)
        r = int(pool.ranks[adapter]) if 0 <= adapter < pool.n_adapters else -1
        if r >= 0 and (A.shape != (pool.in_features, r) or B.shape != (r, pool.out_features) or A.itemsize != 2
                       or B.itemsize != 2):
            raise ValueError(f"adapter {adapter}: A {A.shape} / B {B.shape} do not match rank {r}")
    _check(lib().lora_pool_load(pool.handle, ctypes.c_int32(adapter), _ptr(A), _ptr(B),
                                ctypes.c_int(1 if src_is_device else 0), _stream(stream)))


def lora_pool_evict(pool: Pool, adapter: int) -> None:
    _check(lib().lora_pool_evict(pool.handle, ctypes.c_int32(adapter)))


def lora_pool_mark_resident(pool: Pool, adapter: int) -> None:
    _check(lib().lora_pool_mark_resident(pool.handle, ctypes.c_int32(adapter)))


def lora_pool_adapter_info(pool: Pool, adapter: int) -> dict:
    info = _AdapterInfo()
    _check(lib().lora_pool_adapter_info(pool.handle, ctypes.c_int32(adapter), ctypes.byref(info)))
    return {k: getattr(info, k) for k, _ in _AdapterInfo._fields_}


def lora_pool_destroy(pool: Pool) -> None:
    if pool.handle:
        _check(lib().lora_pool_destroy(pool.handle))
        pool.handle = ctypes.c_void_p(None)


def lora_segments_plan(pool: Pool, token_adapter, options=None) -> Segments:
    ta = _i32(token_adapter)
    h = ctypes.c_void_p(None)
    _check(lib().lora_segments_plan_opts(pool.handle, _ptr(ta), ctypes.c_int32(ta.shape[0]), _opts(options),
                                         ctypes.byref(h)))
    return Segments(h, pool)


def lora_segments_set_options(seg: Segments, options=None) -> None:
    _check(lib().lora_segments_set_options(seg.handle, _opts(options)))


def lora_segments_table_bytes(seg: Segments) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().lora_segments_table_bytes(seg.handle, ctypes.byref(n)))
    return int(n.value)


def lora_segments_upload_to(seg: Segments, dev_table, host_staging, stream=None) -> None:
    """dev_table: device tensor; host_staging: pinned host tensor; both at least lora_segments_table_bytes long."""
    _check(lib().lora_segments_upload_to(seg.handle, _ptr(dev_table), ctypes.c_size_t(_nbytes(dev_table)),
                                         _ptr(host_staging), ctypes.c_size_t(_nbytes(host_staging)), _stream(stream)))
    seg.keepalive = (dev_table, host_staging)


def lora_pool_load_staging_bytes(pool: Pool, adapter: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().lora_pool_load_staging_bytes(pool.handle, ctypes.c_int32(adapter), ctypes.byref(n)))
    return int(n.value)


def lora_pool_load_staged(pool: Pool, adapter: int, A, B, dev_staging, stream=None) -> None:
    """A, B: host arrays (numpy uint16 or pinned torch tensors); dev_staging: device tensor of the caller's."""
    _check(lib().lora_pool_load_staged(pool.handle, ctypes.c_int32(adapter), _ptr(A), _ptr(B), _ptr(dev_staging),
                                       ctypes.c_size_t(_nbytes(dev_staging)), _stream(stream)))


def lora_segments_plan_ranges(pool: Pool, seg_start, seg_adapter) -> Segments:
    st, ad = _i32(seg_start), _i32(seg_adapter)
    if st.shape[0] != ad.shape[0] + 1:
        raise ValueError("seg_start has one more entry than seg_adapter")
    h = ctypes.c_void_p(None)
    _check(lib().lora_segments_plan_ranges(pool.handle, _ptr(st), _ptr(ad), ctypes.c_int32(ad.shape[0]), ctypes.byref(h)))
    return Segments(h, pool)


def lora_segments_upload(seg: Segments, stream=None) -> None:
    _check(lib().lora_segments_upload(seg.handle, _stream(stream)))


def lora_segments_build(pool: Pool, token_adapter, stream=None, options=None) -> Segments:
    ta = _i32(token_adapter)
    h = ctypes.c_void_p(None)
    _check(lib().lora_segments_build_opts(pool.handle, _ptr(ta), ctypes.c_int32(ta.shape[0]), _opts(options),
                                          _stream(stream), ctypes.byref(h)))
    return Segments(h, pool)


def lora_segments_build_ranges(pool: Pool, seg_start, seg_adapter, stream=None) -> Segments:
    st, ad = _i32(seg_start), _i32(seg_adapter)
    if st.shape[0] != ad.shape[0] + 1:
        raise ValueError("seg_start has one more entry than seg_adapter")
    h = ctypes.c_void_p(None)
    _check(lib().lora_segments_build_ranges(pool.handle, _ptr(st), _ptr(ad), ctypes.c_int32(ad.shape[0]),
                                            _stream(stream), ctypes.byref(h)))
    return Segments(h, pool)


def lora_segments_rebuild(seg: Segments, token_adapter, stream=None) -> None:
    ta = _i32(token_adapter)
    _check(lib().lora_segments_rebuild(seg.handle, _ptr(ta), ctypes.c_int32(ta.shape[0]), _stream(stream)))


def lora_segments_info(seg: Segments) -> dict:
    info = _SegInfo()
    _check(lib().lora_segments_info(seg.handle, ctypes.byref(info)))
    return {k: getattr(info, k) for k, _ in _SegInfo._fields_}


def lora_segments_export(seg: Segments) -> dict:
    i = lora_segments_info(seg)
    perm = np.zeros(i["n_active"], dtype=np.int32)
    start = np.zeros(i["n_segments"] + 1, dtype=np.int32)
    adapter = np.zeros(i["n_segments"], dtype=np.int32)
    voff = np.zeros(i["n_tokens"], dtype=np.int64)
    _check(lib().lora_segments_export(seg.handle, _ptr(perm), _ptr(start), _ptr(adapter), _ptr(voff)))
    return {"perm": perm, "seg_start": start, "seg_adapter": adapter, "v_offset": voff}


def lora_segments_export_units(seg: Segments) -> dict:
    i = lora_segments_info(seg)
    su = np.zeros((i["n_shrink_units"], 6), dtype=np.int32)
    eu = np.zeros((i["n_expand_units"], 6), dtype=np.int32)
    _check(lib().lora_segments_export_units(seg.handle, _ptr(su), _ptr(eu)))
    return {"shrink": su, "expand": eu}


def lora_segments_export_launch_units(seg: Segments) -> dict:
    """The one-launch decode form's lists by place in the launch, 7 int32 per place."""
    g = lora_segments_info(seg)["launch_work_groups"]
    su = np.zeros((g, 7), dtype=np.int32)
    eu = np.zeros((4 * g, 7), dtype=np.int32)
    _check(lib().lora_segments_export_launch_units(seg.handle, _ptr(su), _ptr(eu)))
    return {"shrink": su, "expand": eu}


def lora_segments_destroy(seg: Segments) -> None:
    if seg.handle:
        _check(lib().lora_segments_destroy(seg.handle))
        seg.handle = ctypes.c_void_p(None)


def lora_workspace_bytes(pool: Pool, seg: Segments) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().lora_workspace_bytes(pool.handle, seg.handle, ctypes.byref(n)))
    return int(n.value)


def lora_apply_workspace_bytes(pool: Pool, seg: Segments) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().lora_apply_workspace_bytes(pool.handle, seg.handle, ctypes.byref(n)))
    return int(n.value)


def _ld(t, ld):
    if ld is not None:
        return int(ld)
    return int(t.stride(0)) if hasattr(t, "stride") else 0


def _nbytes(ws) -> int:
    return 0 if ws is None else ws.numel() * ws.element_size()


def lora_shrink(pool: Pool, seg: Segments, x, v, workspace=None, stream=None, ldx: Optional[int] = None,
                ws_bytes: Optional[int] = None) -> None:
    """x: bf16 device tensor [T][in]; v: fp32 device tensor of info['v_floats'] elements."""
    _check(lib().lora_shrink(pool.handle, seg.handle, _ptr(x), ctypes.c_int64(_ld(x, ldx)), _ptr(v), _ptr(workspace),
                             ctypes.c_size_t(_nbytes(workspace) if ws_bytes is None else ws_bytes), _stream(stream)))


def lora_expand(pool: Pool, seg: Segments, v, y, stream=None, ldy: Optional[int] = None) -> None:
    """y: bf16 device tensor [T][out], updated in place."""
    _check(lib().lora_expand(pool.handle, seg.handle, _ptr(v), _ptr(y), ctypes.c_int64(_ld(y, ldy)), _stream(stream)))


def lora_apply(pool: Pool, seg: Segments, x, y, workspace, stream=None, ldx: Optional[int] = None,
               ldy: Optional[int] = None, ws_bytes: Optional[int] = None) -> None:
    _check(lib().lora_apply(pool.handle, seg.handle, _ptr(x), ctypes.c_int64(_ld(x, ldx)), _ptr(y),
                            ctypes.c_int64(_ld(y, ldy)), _ptr(workspace),
                            ctypes.c_size_t(_nbytes(workspace) if ws_bytes is None else ws_bytes), _stream(stream)))


def lora_linear_pack_weight(wt, in_features: int, out_features: int, dev_packed, stream=None) -> None:
    """wt: device tensor W^T [out][in] bf16; dev_packed: device tensor of in * out * 2 bytes."""
    _check(lib().lora_linear_pack_weight(_ptr(wt), ctypes.c_int32(in_features), ctypes.c_int32(out_features),
                                         _ptr(dev_packed), _stream(stream)))


def lora_linear(pool: Pool, seg: Segments, x, w_packed, y, workspace, stream=None, ldx: Optional[int] = None,
                ldy: Optional[int] = None, ws_bytes: Optional[int] = None) -> None:
    """y = bf16(x W + delta) for every token, y written once."""
    _check(lib().lora_linear(pool.handle, seg.handle, _ptr(x), ctypes.c_int64(_ld(x, ldx)), _ptr(w_packed), _ptr(y),
                             ctypes.c_int64(_ld(y, ldy)), _ptr(workspace),
                             ctypes.c_size_t(_nbytes(workspace) if ws_bytes is None else ws_bytes), _stream(stream)))


LORA_STATIC_WORKSPACE_BYTES = 32 << 20


def lora_apply_static(pool: Pool, seg: Segments, x, y, stream=None, ldx: Optional[int] = None,
                      ldy: Optional[int] = None) -> None:
    """lora_apply on the library's own static workspace: allocates nothing."""
    _check(lib().lora_apply_static(pool.handle, seg.handle, _ptr(x), ctypes.c_int64(_ld(x, ldx)), _ptr(y),
                                   ctypes.c_int64(_ld(y, ldy)), _stream(stream)))


def _pool_array(pools):
    arr = (ctypes.c_void_p * len(pools))(*[p.handle.value for p in pools])
    return arr


def lora_segments_plan_multi(pools, token_adapter, options=None) -> Segments:
    ta = _i32(token_adapter)
    h = ctypes.c_void_p(None)
    _check(lib().lora_segments_plan_multi_opts(_pool_array(pools), ctypes.c_int32(len(pools)), _ptr(ta),
                                               ctypes.c_int32(ta.shape[0]), _opts(options), ctypes.byref(h)))
    return Segments(h, pools[0])


def lora_segments_build_multi(pools, token_adapter, stream=None, options=None) -> Segments:
    ta = _i32(token_adapter)
    h = ctypes.c_void_p(None)
    _check(lib().lora_segments_build_multi_opts(_pool_array(pools), ctypes.c_int32(len(pools)), _ptr(ta),
                                                ctypes.c_int32(ta.shape[0]), _opts(options), _stream(stream),
                                                ctypes.byref(h)))
    return Segments(h, pools[0])


def lora_apply_multi(pools, seg: Segments, x, y, workspace, stream=None, ldx: Optional[int] = None,
                     ldy: Optional[int] = None, ws_bytes: Optional[int] = None) -> None:
    """y: bf16 device tensor [T][sum of the pools' out_features], updated in place."""
    _check(lib().lora_apply_multi(_pool_array(pools), ctypes.c_int32(len(pools)), seg.handle, _ptr(x),
                                  ctypes.c_int64(_ld(x, ldx)), _ptr(y), ctypes.c_int64(_ld(y, ldy)), _ptr(workspace),
                                  ctypes.c_size_t(_nbytes(workspace) if ws_bytes is None else ws_bytes),
                                  _stream(stream)))


def lora_set_fused_apply(enabled: bool) -> None:
    _check(lib().lora_set_fused_apply(ctypes.c_int(1 if enabled else 0)))


def lora_set_decode_single_launch(enabled: bool) -> None:
    _check(lib().lora_set_decode_single_launch(ctypes.c_int(1 if enabled else 0)))


def lora_set_side_stream(enabled: bool) -> None:
    _check(lib().lora_set_side_stream(ctypes.c_int(1 if enabled else 0)))


def lora_set_merged_launches(enabled: bool) -> None:
    _check(lib().lora_set_merged_launches(ctypes.c_int(1 if enabled else 0)))


def lora_set_fused_wait_limit(polls: int) -> None:
    _check(lib().lora_set_fused_wait_limit(ctypes.c_uint32(polls)))


def lora_set_whole_k_limit(max_units: int) -> None:
    _check(lib().lora_set_whole_k_limit(ctypes.c_int32(int(max_units))))


def lora_segments_check(seg: Segments, stream=None) -> None:
    _check(lib().lora_segments_check(seg.handle, _stream(stream)))


def lora_profile_next_apply(before=None, between=None, after=None) -> None:
    """hipEvent_t handles (integers) recorded around the two launches of the next lora_apply."""
    _check(lib().lora_profile_next_apply(_ptr(before), _ptr(between), _ptr(after)))


def lora_debug_clock_buffer(dev_buf, n_work_groups: int) -> None:
    """Measurement build only: 8 uint64 clock values (100 MHz) per work group of the launches that follow."""
    fn = getattr(lib(), "lora_debug_clock_buffer", None)
    if fn is None:
        raise RuntimeError("this build of the library has no device clocks: build with `python -m "
                           "paper_2511_22880_amd.build --clocks` and set LORA_GFX950_LIB to it")
    rc = fn(_ptr(dev_buf), ctypes.c_uint(int(n_work_groups)))
    if rc != 0:
        raise RuntimeError(f"lora_debug_clock_buffer: hip error {rc}")


def lora_status_string(status: int) -> str:
    return lib().lora_status_string(ctypes.c_int(status)).decode()


def lora_last_error() -> str:
    return lib().lora_last_error().decode("utf-8", "replace")


# ---- adapter placement and routing (include/lora_placement.h; host only) ----------------------------
class _PlaceProblem(ctypes.Structure):
    _fields_ = [("n_servers", ctypes.c_int32), ("n_adapters", ctypes.c_int32), ("ranks", ctypes.c_void_p),
                ("demand_tps", ctypes.c_void_p), ("n_ops", ctypes.c_int32), ("op_ranks", ctypes.c_void_p),
                ("op_tps", ctypes.c_void_p), ("prev_phi", ctypes.c_void_p)]


def lora_place_extrapolate(history, current: float) -> float:
    h = np.ascontiguousarray(history, dtype=np.float64)
    out = ctypes.c_double(0.0)
    _check(lib().lora_place_extrapolate(_ptr(h) if h.size else ctypes.c_void_p(None), ctypes.c_int32(h.size),
                                        ctypes.c_double(float(current)), ctypes.byref(out)))
    return float(out.value)


def lora_place_assign(n_servers: int, ranks, demand_tps, operating_points: dict, prev_phi=None) -> dict:
    """operating_points: {rank: tokens/s}.  Returns phi [n_adapters][n_servers], server_util,
    server_max_rank, budget {rank: servers} and target."""
    ranks = _i32(ranks)
    demand = np.ascontiguousarray(demand_tps, dtype=np.float64)
    op_r = _i32(sorted(operating_points))
    op_t = np.ascontiguousarray([operating_points[int(r)] for r in op_r], dtype=np.float64)
    prev = None if prev_phi is None else np.ascontiguousarray(prev_phi, dtype=np.float64)
    n = int(ranks.shape[0])
    phi = np.zeros((n, n_servers), dtype=np.float64)
    util = np.zeros(n_servers, dtype=np.float64)
    maxr = np.zeros(n_servers, dtype=np.int32)
    budget = np.zeros(op_r.shape[0], dtype=np.int32)
    target = ctypes.c_double(0.0)
    pr = _PlaceProblem(int(n_servers), n, ranks.ctypes.data, demand.ctypes.data, int(op_r.shape[0]), op_r.ctypes.data,
                       op_t.ctypes.data, None if prev is None else prev.ctypes.data)
    _check(lib().lora_place_assign(ctypes.byref(pr), _ptr(phi), _ptr(util), _ptr(maxr), _ptr(budget),
                                   ctypes.byref(target)))
    return {"phi": phi, "server_util": util, "server_max_rank": maxr,
            "budget": {int(r): int(b) for r, b in zip(op_r, budget)}, "target": float(target.value)}
