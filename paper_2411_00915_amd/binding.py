"""Thin ctypes binding over the C-ABI library (include/lora_abi.h).

Argument marshalling only: every step of the operator runs in the HIP kernels
of liblora_amd.so.  There is no CPU fallback; if the library has not been built
the import of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# LORA_AMD_LIBRARY names another build of the same library (instrumented or experimental builds); unset, the
# library built in-tree is the one that runs
LIB_PATH = os.environ.get("LORA_AMD_LIBRARY") or os.path.join(_HERE, "liblora_amd.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2411_00915_amd.build` "
        "(there is no fallback path)")

_lib = ctypes.CDLL(LIB_PATH)

LORA_OK, LORA_ERR_INVALID_ARG, LORA_ERR_UNSUPPORTED, LORA_ERR_NOMEM, LORA_ERR_WORKSPACE, LORA_ERR_DEVICE = range(6)
LORA_F32, LORA_BF16 = 0, 1
LORA_VARIANT_AUTO, LORA_VARIANT_GENERAL, LORA_VARIANT_TILED = 0, 1, 2
LORA_MAX_RANK = 256
LORA_TUNING_COUNT = 17
LORA_STATIC_V_BYTES = 16 << 20
LORA_STATIC_MAX_GROUPS = 4096

_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)


class BatchDesc(ctypes.Structure):
    _fields_ = [("num_tokens", ctypes.c_int32), ("num_segments", ctypes.c_int32),
                ("seg_indptr", _i32p), ("seg_adapter", _i32p),
                ("num_adapters", ctypes.c_int32), ("adapter_rank", _i32p), ("adapter_scale", _f32p),
                ("k", ctypes.c_int32), ("n", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("variant", ctypes.c_int32), ("tuning", _i32p), ("tuning_count", ctypes.c_int32),
                ("merged_adapter_plus1", ctypes.c_int32)]


class Tile(ctypes.Structure):
    _fields_ = [("adapter", ctypes.c_int32), ("row0", ctypes.c_int32), ("nrows", ctypes.c_int32),
                ("c0", ctypes.c_int32), ("cn", ctypes.c_int32), ("shape", ctypes.c_int32),
                ("reserved0", ctypes.c_int32), ("reserved1", ctypes.c_int32)]


class PlanView(ctypes.Structure):
    _fields_ = [("num_tokens", ctypes.c_int32), ("num_active", ctypes.c_int32),
                ("num_groups", ctypes.c_int32), ("v_row_stride", ctypes.c_int32),
                ("kernel_family", ctypes.c_int32), ("shrink_waves", ctypes.c_int32),
                ("v_parts", ctypes.c_int32), ("tuning_source", ctypes.c_int32),
                ("tuning", ctypes.c_int32 * LORA_TUNING_COUNT), ("shrink_kernel_family", ctypes.c_int32),
                ("token_adapter", _i32p), ("perm", _i32p), ("group_adapter", _i32p), ("group_offset", _i32p),
                ("shrink_tiles", ctypes.POINTER(Tile)), ("num_shrink_tiles", ctypes.c_int32),
                ("expand_tiles", ctypes.POINTER(Tile)), ("num_expand_tiles", ctypes.c_int32),
                ("num_gemm_rows", ctypes.c_int32), ("num_gemm_tiles", ctypes.c_int32),
                ("gemm_order", _i32p), ("gemm_stage_offset", _i32p), ("gemm_stage", _i32p),
                ("merged_adapter", ctypes.c_int32), ("num_unmerge", ctypes.c_int32),
                ("unmerge_v_row_stride", ctypes.c_int32), ("unmerge_v_parts", ctypes.c_int32),
                ("unmerge_v_offset", ctypes.c_size_t), ("unmerge_perm", _i32p),
                ("unmerge_shrink_tiles", ctypes.POINTER(Tile)), ("num_unmerge_shrink_tiles", ctypes.c_int32),
                ("unmerge_expand_tiles", ctypes.POINTER(Tile)), ("num_unmerge_expand_tiles", ctypes.c_int32)]


_vp = ctypes.c_void_p
_lib.lora_plan_create.restype = ctypes.c_int
_lib.lora_plan_create.argtypes = [ctypes.POINTER(BatchDesc), ctypes.POINTER(_vp)]
_lib.lora_plan_destroy.restype = None
_lib.lora_plan_destroy.argtypes = [_vp]
_lib.lora_plan_query.restype = ctypes.c_int
_lib.lora_plan_query.argtypes = [_vp, _i32p, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
_lib.lora_plan_export.restype = ctypes.c_int
_lib.lora_plan_export.argtypes = [_vp, ctypes.POINTER(PlanView)]
_lib.lora_plan_upload.restype = ctypes.c_int
_lib.lora_plan_upload.argtypes = [_vp, _vp]
_lib.lora_shrink.restype = ctypes.c_int
_lib.lora_shrink.argtypes = [_vp, _vp, ctypes.c_int64, _vp, _vp, _vp]
_lib.lora_expand.restype = ctypes.c_int
_lib.lora_expand.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_int64, ctypes.c_float, _vp]
_lib.lora_delta.restype = ctypes.c_int
_lib.lora_delta.argtypes = [_vp, _vp, ctypes.c_int64, _vp, _vp, _vp, _vp, ctypes.c_int64, ctypes.c_float, _vp]
_lib.lora_delta_static.restype = ctypes.c_int
_lib.lora_delta_static.argtypes = [_vp, _vp, ctypes.c_int64, _vp, _vp, _vp, ctypes.c_int64, ctypes.c_float, _vp]
_lib.lora_base_gemm.restype = ctypes.c_int
_lib.lora_base_gemm.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                _vp, ctypes.c_int64, _vp, ctypes.c_int64, _vp, ctypes.c_int64, _vp]
_lib.lora_fused_forward.restype = ctypes.c_int
_lib.lora_fused_forward.argtypes = [_vp, _vp, ctypes.c_int64, _vp, ctypes.c_int64, _vp, _vp,
                                    _vp, ctypes.c_int64, _vp, ctypes.c_size_t, _vp]
_lib.lora_merge.restype = ctypes.c_int
_lib.lora_merge.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_float, ctypes.c_int32,
                            ctypes.c_int32, _vp, ctypes.c_int64, _vp, _vp, _vp]
_lib.lora_status_str.restype = ctypes.c_char_p
_lib.lora_status_str.argtypes = [ctypes.c_int]
_lib.lora_tuning_set.restype = None
_lib.lora_tuning_set.argtypes = [_i32p, ctypes.c_int32]
_lib.lora_tuning_get.restype = None
_lib.lora_tuning_get.argtypes = [_i32p, ctypes.c_int32]



class TuningEntry(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_int32), ("k", ctypes.c_int32), ("n", ctypes.c_int32), ("max_rank", ctypes.c_int32),
                ("group_class", ctypes.c_int32), ("values", ctypes.c_int32 * LORA_TUNING_COUNT)]


_lib.lora_tuning_table_set.restype = ctypes.c_int
_lib.lora_tuning_table_set.argtypes = [ctypes.POINTER(TuningEntry), ctypes.c_int32]
_lib.lora_tuning_table_get.restype = ctypes.c_int32
_lib.lora_tuning_table_get.argtypes = [ctypes.POINTER(TuningEntry), ctypes.c_int32]
_lib.lora_probe.restype = ctypes.c_int
_lib.lora_probe.argtypes = [ctypes.c_int32, _vp, ctypes.c_size_t, ctypes.c_int32, _vp]
_lib.lora_trace_tick_khz.restype = ctypes.c_int32
_lib.lora_trace_set.restype = ctypes.c_int
_lib.lora_trace_set.argtypes = [_vp, ctypes.c_size_t]
_lib.lora_timing_begin.restype = ctypes.c_int
_lib.lora_timing_end.restype = ctypes.c_int
_lib.lora_timing_read.restype = ctypes.c_int
_lib.lora_timing_read.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double),
                                  ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
_lib.lora_kernel_name.restype = ctypes.c_char_p
_lib.lora_kernel_name.argtypes = [ctypes.c_int32]
_lib.lora_kernel_count.restype = ctypes.c_int32

EXPORTED = ["lora_timing_begin", "lora_timing_end", "lora_timing_read", "lora_kernel_name", "lora_kernel_count",
            "lora_plan_create", "lora_plan_destroy", "lora_plan_query", "lora_plan_export",
            "lora_plan_upload", "lora_shrink", "lora_expand", "lora_delta", "lora_delta_static", "lora_base_gemm",
            "lora_fused_forward", "lora_merge", "lora_status_str", "lora_tuning_set", "lora_tuning_get",
            "lora_tuning_table_set", "lora_tuning_table_get", "lora_probe", "lora_trace_set", "lora_trace_tick_khz"]

TUNING_FIELDS = ["shrink_waves", "shrink_tb2_min_rows", "shrink_max_jb", "expand_wave_bytes",
                 "expand_tb2_min_rows", "expand_tb4_min_rows", "tiled_min_tokens",
                 "shrink_small_waves", "shrink_small_jb", "shrink_target_wgs", "fused_wait_us", "fused_delay", "expand_wave_bytes_big", "shrink_tb4_min_rows",
                 "shrink_stream_min_tokens", "shrink_stream_wgs", "expand_stream_stages"]


class LoraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lora_status_str(status)} (status {status})")


def lora_status_str(status: int) -> str:
    return _lib.lora_status_str(int(status)).decode()


def _check(status: int, where: str):
    if status != LORA_OK:
        raise LoraError(status, where)


def _ptr(obj) -> Optional[int]:
    """Device/host address of a torch tensor, or an int address, or None."""
    if obj is None:
        return None
    if isinstance(obj, int):
        return obj
    return int(obj.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def lora_tuning_get() -> dict:
    buf = (ctypes.c_int32 * len(TUNING_FIELDS))()
    _lib.lora_tuning_get(buf, len(TUNING_FIELDS))
    return dict(zip(TUNING_FIELDS, list(buf)))


def lora_tuning_set(**kw) -> None:
    """Set the process's default tunables (values <= 0 or missing keep the current value)."""
    vals = _tuning_values(kw)
    buf = (ctypes.c_int32 * len(vals))(*vals)
    _lib.lora_tuning_set(buf, len(vals))


def _tuning_values(tunables: dict):
    unknown = set(tunables) - set(TUNING_FIELDS)
    if unknown:
        raise KeyError(f"unknown tuning fields: {sorted(unknown)}")
    return [int(tunables.get(f, 0)) for f in TUNING_FIELDS]


def lora_tuning_table_set(entries) -> None:
    """Replace the process's shape table.  entries: iterable of dicts with the key fields tokens, k, n, max_rank,
    group_class and `tunables` (name -> value); None or empty restores the table the library ships with."""
    entries = list(entries or [])
    arr = (TuningEntry * max(len(entries), 1))()
    for i, e in enumerate(entries):
        arr[i].tokens, arr[i].k, arr[i].n = int(e["tokens"]), int(e["k"]), int(e["n"])
        arr[i].max_rank, arr[i].group_class = int(e["max_rank"]), int(e["group_class"])
        for j, val in enumerate(_tuning_values(e["tunables"])):
            arr[i].values[j] = val
    _check(_lib.lora_tuning_table_set(arr if entries else None, len(entries)), "lora_tuning_table_set")


def lora_tuning_table_get() -> list:
    n = _lib.lora_tuning_table_get(None, 0)
    arr = (TuningEntry * max(n, 1))()
    n = min(n, _lib.lora_tuning_table_get(arr, n))
    return [dict(tokens=arr[i].tokens, k=arr[i].k, n=arr[i].n, max_rank=arr[i].max_rank, group_class=arr[i].group_class,
                 tunables={f: int(arr[i].values[j]) for j, f in enumerate(TUNING_FIELDS) if arr[i].values[j] > 0})
            for i in range(n)]


LORA_PROBE_EMPTY, LORA_PROBE_READ, LORA_PROBE_MFMA = 0, 1, 2


def lora_probe(kind: int, buffer, nbytes: int, iters: int = 1, stream=None):
    _check(_lib.lora_probe(int(kind), _ptr(buffer), int(nbytes), int(iters), _stream(stream)), "lora_probe")


def lora_trace_set(buffer=None):
    """buffer: an int64 device tensor with 8 entries per tile of the plans used while it is set; None switches off"""
    if buffer is None:
        _check(_lib.lora_trace_set(None, 0), "lora_trace_set")
    else:
        _check(_lib.lora_trace_set(_ptr(buffer), buffer.numel() * buffer.element_size()), "lora_trace_set")


def lora_trace_tick_khz() -> int:
    return int(_lib.lora_trace_tick_khz())


def lora_timing_begin():
    _check(_lib.lora_timing_begin(), "lora_timing_begin")


def lora_timing_end() -> dict:
    """Stop timing; returns {kernel name: dict(count, avg_us, min_us, max_us)} for kernels that ran."""
    _check(_lib.lora_timing_end(), "lora_timing_end")
    out = {}
    for kid in range(_lib.lora_kernel_count()):
        c, tot, mn, mx = ctypes.c_int64(), ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        _check(_lib.lora_timing_read(kid, ctypes.byref(c), ctypes.byref(tot), ctypes.byref(mn), ctypes.byref(mx)),
               "lora_timing_read")
        if c.value:
            out[_lib.lora_kernel_name(kid).decode()] = dict(count=int(c.value), avg_us=tot.value / c.value,
                                                            min_us=mn.value, max_us=mx.value)
    return out


class Plan:
    """Owner of a lora_plan handle."""

    def __init__(self, handle: int, keepalive):
        self._h = handle
        self._keep = keepalive

    @property
    def handle(self) -> int:
        return self._h

    def destroy(self):
        if self._h:
            _lib.lora_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def lora_plan(num_tokens, seg_indptr, seg_adapter, adapter_rank, adapter_scale, k, n, dtype,
              variant=LORA_VARIANT_AUTO, tuning: Optional[dict] = None, merged_adapter: Optional[int] = None) -> Plan:
    """lora_plan_create; tables are host arrays (numpy or sequences).  tuning: tunables for this plan only
    (name -> value), on top of the shape table's entry and the process defaults.  merged_adapter: mixture mode,
    the adapter that is folded into the base weight the batch runs on (None: no adapter is)."""
    indptr = np.ascontiguousarray(seg_indptr, dtype=np.int32)
    seg_ad = np.ascontiguousarray(seg_adapter, dtype=np.int32)
    rank = np.ascontiguousarray(adapter_rank, dtype=np.int32)
    scale = np.ascontiguousarray(adapter_scale, dtype=np.float32)
    desc = BatchDesc(int(num_tokens), int(seg_ad.shape[0]),
                     indptr.ctypes.data_as(_i32p), seg_ad.ctypes.data_as(_i32p),
                     int(rank.shape[0]), rank.ctypes.data_as(_i32p), scale.ctypes.data_as(_f32p),
                     int(k), int(n), int(dtype), int(variant), None, 0,
                     0 if merged_adapter is None else int(merged_adapter) + 1)
    if tuning:
        vals = (ctypes.c_int32 * LORA_TUNING_COUNT)(*_tuning_values(tuning))
        desc.tuning = ctypes.cast(vals, _i32p)
        desc.tuning_count = LORA_TUNING_COUNT
    out = _vp()
    _check(_lib.lora_plan_create(ctypes.byref(desc), ctypes.byref(out)), "lora_plan_create")
    return Plan(out.value, None)


def lora_plan_create_raw(desc: Optional[BatchDesc]):
    """Direct call for error-path tests: returns (status, handle)."""
    out = _vp()
    st = _lib.lora_plan_create(ctypes.byref(desc) if desc is not None else None, ctypes.byref(out))
    return st, out.value


def lora_plan_destroy(plan: Plan):
    plan.destroy()


def lora_plan_query(plan: Plan):
    r = ctypes.c_int32()
    vb = ctypes.c_size_t()
    ws = ctypes.c_size_t()
    _check(_lib.lora_plan_query(plan.handle, ctypes.byref(r), ctypes.byref(vb), ctypes.byref(ws)), "lora_plan_query")
    return int(r.value), int(vb.value), int(ws.value)


def lora_plan_export(plan: Plan) -> dict:
    """Copy of the plan's host tables as numpy arrays."""
    v = PlanView()
    _check(_lib.lora_plan_export(plan.handle, ctypes.byref(v)), "lora_plan_export")

    def arr(p, n):
        return np.ctypeslib.as_array(p, shape=(n,)).copy() if n > 0 else np.zeros(0, np.int32)

    def tiles(p, n):
        if n == 0:
            return np.zeros((0, 8), np.int32)
        raw = np.ctypeslib.as_array(ctypes.cast(p, _i32p), shape=(n * 8,)).copy()
        return raw.reshape(n, 8)

    return dict(num_tokens=v.num_tokens, num_active=v.num_active, num_groups=v.num_groups,
                v_row_stride=v.v_row_stride, kernel_family=v.kernel_family, shrink_kernel_family=v.shrink_kernel_family,
                shrink_waves=v.shrink_waves,
                v_parts=v.v_parts, tuning_source=v.tuning_source,
                tuning={f: int(v.tuning[j]) for j, f in enumerate(TUNING_FIELDS)},
                token_adapter=arr(v.token_adapter, v.num_tokens), perm=arr(v.perm, v.num_active),
                group_adapter=arr(v.group_adapter, v.num_groups),
                group_offset=arr(v.group_offset, v.num_groups + 1),
                shrink_tiles=tiles(v.shrink_tiles, v.num_shrink_tiles),
                expand_tiles=tiles(v.expand_tiles, v.num_expand_tiles),
                gemm_order=arr(v.gemm_order, v.num_gemm_rows),
                gemm_stage_offset=arr(v.gemm_stage_offset, v.num_gemm_tiles + 1 if v.num_gemm_tiles else 0),
                gemm_stage=(arr(v.gemm_stage, int(v.gemm_stage_offset[v.num_gemm_tiles])) if v.num_gemm_tiles
                            else np.zeros(0, np.int32)),
                merged_adapter=v.merged_adapter, num_unmerge=v.num_unmerge,
                unmerge_v_row_stride=v.unmerge_v_row_stride, unmerge_v_parts=v.unmerge_v_parts,
                unmerge_v_offset=int(v.unmerge_v_offset), unmerge_perm=arr(v.unmerge_perm, v.num_unmerge),
                unmerge_shrink_tiles=tiles(v.unmerge_shrink_tiles, v.num_unmerge_shrink_tiles),
                unmerge_expand_tiles=tiles(v.unmerge_expand_tiles, v.num_unmerge_expand_tiles))


def lora_plan_upload(plan: Plan, stream=None):
    _check(_lib.lora_plan_upload(plan.handle, _stream(stream)), "lora_plan_upload")


def lora_shrink(plan: Plan, x, ldx: int, d_At_ptrs, v, stream=None):
    _check(_lib.lora_shrink(plan.handle, _ptr(x), int(ldx), _ptr(d_At_ptrs), _ptr(v), _stream(stream)), "lora_shrink")


def lora_expand(plan: Plan, v, d_Bt_ptrs, y, ldy: int, beta: float = 1.0, stream=None):
    _check(_lib.lora_expand(plan.handle, _ptr(v), _ptr(d_Bt_ptrs), _ptr(y), int(ldy), float(beta), _stream(stream)),
           "lora_expand")


def lora_delta(plan: Plan, x, ldx: int, d_At_ptrs, d_Bt_ptrs, v, y, ldy: int, beta: float = 1.0, stream=None):
    _check(_lib.lora_delta(plan.handle, _ptr(x), int(ldx), _ptr(d_At_ptrs), _ptr(d_Bt_ptrs), _ptr(v), _ptr(y), int(ldy),
                           float(beta), _stream(stream)), "lora_delta")


def lora_delta_static(plan: Plan, x, ldx: int, d_At_ptrs, d_Bt_ptrs, y, ldy: int, beta: float = 1.0, stream=None):
    _check(_lib.lora_delta_static(plan.handle, _ptr(x), int(ldx), _ptr(d_At_ptrs), _ptr(d_Bt_ptrs), _ptr(y), int(ldy),
                                  float(beta), _stream(stream)), "lora_delta_static")


def lora_base_gemm(num_tokens: int, k: int, n: int, dtype: int, x, ldx: int, Wt, ldw: int, y, ldy: int, stream=None):
    _check(_lib.lora_base_gemm(int(num_tokens), int(k), int(n), int(dtype), _ptr(x), int(ldx), _ptr(Wt), int(ldw),
                               _ptr(y), int(ldy), _stream(stream)), "lora_base_gemm")


def lora_merge(num_layers: int, n: int, k: int, rank: int, scale: float, dtype: int, d_Wt_ptrs, ldw: int,
               d_At_ptrs, d_Bt_ptrs, variant: int = LORA_VARIANT_AUTO, stream=None):
    _check(_lib.lora_merge(int(num_layers), int(n), int(k), int(rank), float(scale), int(dtype), int(variant),
                           _ptr(d_Wt_ptrs), int(ldw), _ptr(d_At_ptrs), _ptr(d_Bt_ptrs), _stream(stream)), "lora_merge")


def lora_fused_forward(plan: Plan, x, ldx: int, Wt, ldw: int, d_At_ptrs, d_Bt_ptrs, y, ldy: int,
                       workspace, workspace_bytes: int, stream=None):
    _check(_lib.lora_fused_forward(plan.handle, _ptr(x), int(ldx), _ptr(Wt), int(ldw), _ptr(d_At_ptrs),
                                   _ptr(d_Bt_ptrs), _ptr(y), int(ldy), _ptr(workspace), int(workspace_bytes),
                                   _stream(stream)), "lora_fused_forward")
