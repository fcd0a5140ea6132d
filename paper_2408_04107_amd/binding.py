"""ctypes binding of libfdc.so: argument marshalling only.

Every function here has the name of the C entry point it forwards to
(include/fdc.h). Tensors are torch tensors used as plain device buffers: the
binding passes data_ptr() and the current HIP stream, nothing is computed in
Python. There is no fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libfdc.so")

FDC_BF16, FDC_F32, FDC_FP8, FDC_FP4 = 0, 1, 2, 3
FDC_FOLD, FDC_APPLY = 0, 1

EXPORTED_SYMBOLS = [
    "fdc_last_error", "fdc_layout_create", "fdc_layout_create_gqa", "fdc_layout_tables", "fdc_layout_destroy",
    "fdc_plan_params_default", "fdc_suggest_workers", "fdc_plan_decode", "fdc_plan_decode_paged", "fdc_plan_prefill", "fdc_plan_prefill_paged",
    "fdc_plan_export", "fdc_plan_workspace_bytes", "fdc_plan_upload", "fdc_plan_destroy",
    "fdc_project_latent_kv", "fdc_absorb_query", "fdc_latent_attn_decode",
    "fdc_latent_attn_prefill", "fdc_absorb_output", "fdc_profile_decode_events", "fdc_select_ranks",
    "fdc_rope_absorb_query", "fdc_rope_compress_keys", "fdc_project_and_absorb_query", "fdc_latent_attn_decode_at",
    "fdc_plan_decode_device", "fdc_plan_decode_run", "fdc_plan_download", "fdc_latent_attn_decode_static",
]


class FdcError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libfdc status {status}: {text}")
        self.status = status


class PlanParams(C.Structure):
    _fields_ = [("n_workers", C.c_int32), ("granule", C.c_int32), ("min_split", C.c_int32),
                ("split", C.c_int32), ("br_base", C.c_int32), ("br_cap", C.c_int32),
                ("cost_mode", C.c_int32), ("softmax_cost", C.c_int32)]


class PlanTables(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_items", C.c_int32), ("n_workers", C.c_int32),
                ("n_units", C.c_int32),
                ("item_b", C.POINTER(C.c_int32)), ("item_h", C.POINTER(C.c_int32)),
                ("item_lo", C.POINTER(C.c_int32)), ("item_hi", C.POINTER(C.c_int32)),
                ("item_cost", C.POINTER(C.c_int64)), ("unit_item_ptr", C.POINTER(C.c_int32)),
                ("worker_ptr", C.POINTER(C.c_int32)), ("worker_items", C.POINTER(C.c_int32)),
                ("worker_load", C.POINTER(C.c_int64)), ("br", C.POINTER(C.c_int32))]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with "
                               "`python -m paper_2408_04107_amd.build` (needs hipcc); there is no fallback path")
        l = C.CDLL(_LIB_PATH)
        vp, i32p, i64p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64)
        l.fdc_last_error.argtypes = [C.c_char_p, C.c_size_t]
        l.fdc_last_error.restype = None
        l.fdc_layout_create.argtypes = [C.c_int] * 4 + [i32p, i32p, C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
        l.fdc_layout_create_gqa.argtypes = [C.c_int] * 5 + [i32p, i32p, C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
        l.fdc_layout_tables.argtypes = [vp, i64p, i64p, i32p, i32p, i64p, i64p]
        l.fdc_layout_destroy.argtypes = [vp]
        l.fdc_layout_destroy.restype = None
        l.fdc_plan_params_default.argtypes = [C.POINTER(PlanParams)]
        l.fdc_plan_params_default.restype = None
        l.fdc_suggest_workers.argtypes = [C.c_int, i32p]
        l.fdc_plan_decode.argtypes = [vp, C.c_int, C.c_int, i32p, C.POINTER(PlanParams), C.POINTER(vp)]
        l.fdc_plan_decode_paged.argtypes = [vp, C.c_int, C.c_int, i32p, i32p, C.c_int, C.POINTER(PlanParams),
                                            C.POINTER(vp)]
        l.fdc_plan_prefill.argtypes = [vp, C.c_int, C.c_int, i32p, i32p, C.POINTER(PlanParams), C.POINTER(vp)]
        l.fdc_plan_prefill_paged.argtypes = [vp, C.c_int, C.c_int, i32p, i32p, i32p, C.c_int, C.POINTER(PlanParams),
                                             C.POINTER(vp)]
        l.fdc_plan_decode_device.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.POINTER(PlanParams), C.POINTER(vp)]
        l.fdc_plan_decode_run.argtypes = [C.POINTER(vp), C.POINTER(vp), C.c_int, vp, vp, vp]
        l.fdc_plan_download.argtypes = [vp, vp, vp]
        l.fdc_plan_export.argtypes = [vp, C.POINTER(PlanTables)]
        l.fdc_plan_workspace_bytes.argtypes = [vp]
        l.fdc_plan_workspace_bytes.restype = C.c_size_t
        l.fdc_plan_upload.argtypes = [vp, vp, C.c_size_t, vp]
        l.fdc_plan_destroy.argtypes = [vp]
        l.fdc_plan_destroy.restype = None
        l.fdc_project_latent_kv.argtypes = [vp, C.c_int, vp, C.c_int, vp, vp, vp, vp, vp, vp, vp]
        l.fdc_absorb_query.argtypes = [vp, C.c_int, vp, C.c_int, vp, vp, C.c_int, vp]
        l.fdc_project_and_absorb_query.argtypes = [vp, C.c_int, vp, C.c_int, vp, vp, vp, vp, vp, vp, vp, vp, C.c_int, vp, vp]
        l.fdc_latent_attn_decode.argtypes = [vp, vp, vp, vp, vp, C.c_float, vp, vp, C.c_size_t, vp]
        l.fdc_latent_attn_decode_static.argtypes = [vp, vp, vp, vp, vp, C.c_float, vp, vp]
        l.fdc_latent_attn_decode_at.argtypes = [vp, vp, vp, vp, vp, vp, C.c_float, vp, vp, C.c_size_t, vp]
        l.fdc_latent_attn_prefill.argtypes = [vp, vp, vp, vp, vp, C.c_float, C.c_int, vp, vp, C.c_size_t, vp]
        l.fdc_absorb_output.argtypes = [vp, C.c_int, C.c_int, vp, vp, vp, vp, C.c_int, C.c_int, vp, C.c_int, vp]
        l.fdc_profile_decode_events.argtypes = [vp, vp]
        l.fdc_rope_absorb_query.argtypes = [vp, C.c_int, vp, C.c_int, vp, vp, vp, C.c_int, vp, vp, C.c_int, vp, vp]
        l.fdc_rope_compress_keys.argtypes = [vp, C.c_int, vp, C.c_int, vp, vp, vp, vp, C.c_int, vp, vp, vp, vp]
        l.fdc_select_ranks.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_double), C.c_double, C.c_int, i32p]
        _lib = l
    return _lib


def _check(status: int) -> None:
    if status != 0:
        buf = C.create_string_buffer(512)
        lib().fdc_last_error(buf, 512)
        raise FdcError(status, buf.value.decode(errors="replace"))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _p32(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _p64(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int64))


def _dev(t) -> Optional[int]:
    """Device pointer of a torch tensor (or None)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libfdc takes contiguous device tensors")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is not None:
        return int(stream)
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


class Layout:
    """Owns an fdc_layout*. rk, rv: int [L, H] (H = key/value heads); q_per_kv query heads share one."""

    def __init__(self, n_layers, n_heads, d_model, d_head, rk, rv, max_batch, max_seq, dtype, q_per_kv=1):
        rk, rv = _i32(rk).reshape(-1), _i32(rv).reshape(-1)
        if rk.size != n_layers * n_heads or rv.size != n_layers * n_heads:
            raise ValueError("rk/rv must have n_layers * n_heads entries")
        self.handle = C.c_void_p()
        if q_per_kv == 1:
            _check(lib().fdc_layout_create(n_layers, n_heads, d_model, d_head, _p32(rk), _p32(rv), max_batch,
                                           max_seq, dtype, C.byref(self.handle)))
        else:
            _check(lib().fdc_layout_create_gqa(n_layers, n_heads, q_per_kv, d_model, d_head, _p32(rk), _p32(rv),
                                               max_batch, max_seq, dtype, C.byref(self.handle)))
        self.q_per_kv = q_per_kv
        self.n_layers, self.n_heads, self.d_model, self.d_head = n_layers, n_heads, d_model, d_head
        self.max_batch, self.max_seq, self.dtype = max_batch, max_seq, dtype
        self.rk = rk.reshape(n_layers, n_heads).copy()
        self.rv = rv.reshape(n_layers, n_heads).copy()

    def tables(self):
        L, H = self.n_layers, self.n_heads
        koff, voff = np.zeros(L * H, np.int64), np.zeros(L * H, np.int64)
        koff_r, voff_r = np.zeros(L * (H + 1), np.int32), np.zeros(L * (H + 1), np.int32)
        kb, vb = np.zeros(L, np.int64), np.zeros(L, np.int64)
        _check(lib().fdc_layout_tables(self.handle, _p64(koff), _p64(voff), _p32(koff_r), _p32(voff_r),
                                       _p64(kb), _p64(vb)))
        return {"koff": koff.reshape(L, H), "voff": voff.reshape(L, H),
                "koff_r": koff_r.reshape(L, H + 1), "voff_r": voff_r.reshape(L, H + 1),
                "k_bytes": kb, "v_bytes": vb}

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.fdc_layout_destroy(self.handle)
            self.handle = None


def fdc_plan_params_default() -> PlanParams:
    p = PlanParams()
    lib().fdc_plan_params_default(C.byref(p))
    return p


def fdc_suggest_workers(kind: int) -> int:
    n = C.c_int32(0)
    _check(lib().fdc_suggest_workers(kind, C.byref(n)))
    return int(n.value)


class Plan:
    """Owns an fdc_plan*. Keeps its layout alive."""

    def __init__(self, handle, layout: Layout):
        self.handle, self.layout = handle, layout

    def export(self):
        t = PlanTables()
        _check(lib().fdc_plan_export(self.handle, C.byref(t)))
        n, W, U = t.n_items, t.n_workers, t.n_units

        def arr(ptr, count, dt):
            if count == 0:
                return np.zeros(0, dt)
            return np.ctypeslib.as_array(ptr, shape=(count,)).astype(dt, copy=True)

        out = {"kind": t.kind, "n_items": n, "n_workers": W, "n_units": U,
               "item_b": arr(t.item_b, n, np.int32), "item_h": arr(t.item_h, n, np.int32),
               "item_lo": arr(t.item_lo, n, np.int32), "item_hi": arr(t.item_hi, n, np.int32),
               "item_cost": arr(t.item_cost, n, np.int64),
               "worker_ptr": arr(t.worker_ptr, W + 1, np.int32),
               "worker_items": arr(t.worker_items, n, np.int32),
               "worker_load": arr(t.worker_load, W, np.int64)}
        if t.kind == 0:
            out["unit_item_ptr"] = arr(t.unit_item_ptr, U + 1, np.int32)
        else:
            out["br"] = arr(t.br, self.layout.n_heads * self.layout.q_per_kv, np.int32)
        return out

    def workspace_bytes(self) -> int:
        return int(lib().fdc_plan_workspace_bytes(self.handle))

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.fdc_plan_destroy(self.handle)
            self.handle = None


def fdc_plan_decode(layout: Layout, layer: int, seq_len: Sequence[int], params: PlanParams) -> Plan:
    s = _i32(seq_len)
    h = C.c_void_p()
    _check(lib().fdc_plan_decode(layout.handle, layer, int(s.size), _p32(s), C.byref(params), C.byref(h)))
    return Plan(h, layout)


def fdc_plan_decode_paged(layout: Layout, layer: int, seq_len: Sequence[int], block_table, params: PlanParams) -> Plan:
    """block_table: int [batch, max_pages]; the layout's batch rows are the pages, max_seq the page size."""
    s = _i32(seq_len)
    bt = np.ascontiguousarray(np.asarray(block_table, dtype=np.int32))
    if bt.ndim != 2 or bt.shape[0] != s.size:
        raise ValueError("block_table must be [batch, max_pages]")
    h = C.c_void_p()
    _check(lib().fdc_plan_decode_paged(layout.handle, layer, int(s.size), _p32(s), _p32(bt.reshape(-1)),
                                       int(bt.shape[1]), C.byref(params), C.byref(h)))
    return Plan(h, layout)


def fdc_plan_prefill(layout: Layout, layer: int, q_len: Sequence[int], kv_len: Sequence[int],
                     params: PlanParams) -> Plan:
    q, k = _i32(q_len), _i32(kv_len)
    if q.size != k.size:
        raise ValueError("q_len and kv_len must have the same length")
    h = C.c_void_p()
    _check(lib().fdc_plan_prefill(layout.handle, layer, int(q.size), _p32(q), _p32(k), C.byref(params), C.byref(h)))
    return Plan(h, layout)


def fdc_plan_prefill_paged(layout: Layout, layer: int, q_len: Sequence[int], kv_len: Sequence[int], block_table,
                           params: PlanParams) -> Plan:
    """block_table: int [batch, max_pages]; the layout's batch rows are the pages, max_seq the page size."""
    q, k = _i32(q_len), _i32(kv_len)
    bt = np.ascontiguousarray(np.asarray(block_table, dtype=np.int32))
    if q.size != k.size or bt.ndim != 2 or bt.shape[0] != q.size:
        raise ValueError("q_len and kv_len must have the same length and block_table be [batch, max_pages]")
    h = C.c_void_p()
    _check(lib().fdc_plan_prefill_paged(layout.handle, layer, int(q.size), _p32(q), _p32(k), _p32(bt.reshape(-1)),
                                        int(bt.shape[1]), C.byref(params), C.byref(h)))
    return Plan(h, layout)


def fdc_plan_decode_device(layout: Layout, layer: int, batch: int, max_pages: int, params: PlanParams) -> Plan:
    """A decode plan whose tables the GPU computes (fdc_plan_decode_run). max_pages 0: dense cache."""
    h = C.c_void_p()
    _check(lib().fdc_plan_decode_device(layout.handle, layer, int(batch), int(max_pages), C.byref(params), C.byref(h)))
    return Plan(h, layout)


def fdc_plan_decode_run(plans: Sequence[Plan], workspaces, seq_len, block_table=None, stream=None) -> None:
    """seq_len (and block_table for paged plans): int32 device tensors; one workspace per plan."""
    n = len(plans)
    if n != len(workspaces):
        raise ValueError("one workspace per plan")
    hs = (C.c_void_p * n)(*[p.handle for p in plans])
    ws = (C.c_void_p * n)(*[_dev(w) for w in workspaces])
    _check(lib().fdc_plan_decode_run(hs, ws, n, _dev(seq_len), _dev(block_table) if block_table is not None else None,
                                     _stream(stream)))


def fdc_plan_download(plan: Plan, workspace, stream=None) -> None:
    _check(lib().fdc_plan_download(plan.handle, _dev(workspace), _stream(stream)))


def fdc_plan_upload(plan: Plan, workspace, stream=None) -> None:
    _check(lib().fdc_plan_upload(plan.handle, _dev(workspace), workspace.numel() * workspace.element_size(),
                                 _stream(stream)))


def fdc_project_latent_kv(layout: Layout, layer: int, x, tok_batch, tok_pos, A_cat, k_cache, v_cache,
                          stream=None, status=None) -> None:
    """status: device int32 tensor (one element) that collects the fault bits of skipped rows, or None."""
    T = int(x.shape[0])
    _check(lib().fdc_project_latent_kv(layout.handle, layer, _dev(x), T, _dev(tok_batch), _dev(tok_pos),
                                       _dev(A_cat), _dev(k_cache), _dev(v_cache), _dev(status), _stream(stream)))


def fdc_absorb_query(layout: Layout, layer: int, q, Bk, q_lat, q_lat_dtype: int, stream=None) -> None:
    T = int(q.shape[0])
    _check(lib().fdc_absorb_query(layout.handle, layer, _dev(q), T, _dev(Bk), _dev(q_lat), q_lat_dtype,
                                  _stream(stream)))


def fdc_project_and_absorb_query(layout: Layout, layer: int, x, tok_batch, tok_pos, A_cat, k_cache, v_cache,
                                 q, Bk, q_lat, q_lat_dtype: int, stream=None, status=None) -> None:
    T = int(x.shape[0])
    _check(lib().fdc_project_and_absorb_query(layout.handle, layer, _dev(x), T, _dev(tok_batch), _dev(tok_pos),
                                              _dev(A_cat), _dev(k_cache), _dev(v_cache), _dev(q), _dev(Bk),
                                              _dev(q_lat), q_lat_dtype, _dev(status), _stream(stream)))


def fdc_latent_attn_decode(layout: Layout, plan: Plan, q_lat, k_cache, v_cache, scale: float, o_lat,
                           workspace, stream=None) -> None:
    _check(lib().fdc_latent_attn_decode(layout.handle, plan.handle, _dev(q_lat), _dev(k_cache), _dev(v_cache),
                                        float(scale), _dev(o_lat), _dev(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)))


def fdc_latent_attn_decode_static(layout: Layout, plan: Plan, q_lat, k_cache, v_cache, scale: float, o_lat,
                                  stream=None) -> None:
    """fdc_latent_attn_decode on the workspace built into the library (no allocation, no upload)."""
    _check(lib().fdc_latent_attn_decode_static(layout.handle, plan.handle, _dev(q_lat), _dev(k_cache),
                                               _dev(v_cache), float(scale), _dev(o_lat), _stream(stream)))


def fdc_latent_attn_decode_at(layout: Layout, plan: Plan, seq_len, q_lat, k_cache, v_cache, scale: float, o_lat,
                              workspace, stream=None) -> None:
    """seq_len: device int32 tensor [batch], the actual lengths inside the planned lengths' last granule."""
    _check(lib().fdc_latent_attn_decode_at(layout.handle, plan.handle, _dev(seq_len), _dev(q_lat), _dev(k_cache),
                                           _dev(v_cache), float(scale), _dev(o_lat), _dev(workspace),
                                           workspace.numel() * workspace.element_size(), _stream(stream)))


def fdc_latent_attn_prefill(layout: Layout, plan: Plan, q_lat, k_cache, v_cache, scale: float, causal: bool,
                            o_lat, workspace, stream=None) -> None:
    _check(lib().fdc_latent_attn_prefill(layout.handle, plan.handle, _dev(q_lat), _dev(k_cache), _dev(v_cache),
                                         float(scale), int(bool(causal)), _dev(o_lat), _dev(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)))


def fdc_absorb_output(layout: Layout, layer: int, mode: int, Bv, Wo, M, o_lat, o_lat_dtype: int, T: int, y,
                      y_dtype: int, stream=None) -> None:
    _check(lib().fdc_absorb_output(layout.handle, layer, mode, _dev(Bv), _dev(Wo), _dev(M), _dev(o_lat),
                                   o_lat_dtype, int(T), _dev(y), y_dtype, _stream(stream)))


def fdc_profile_decode_events(start_event: Optional[int], stop_event: Optional[int]) -> None:
    """start_event / stop_event: raw hipEvent_t handles (ints) or None."""
    _check(lib().fdc_profile_decode_events(start_event, stop_event))


def fdc_select_ranks(theta, r: float, multiple: int = 16) -> np.ndarray:
    """theta: float64 [n, d_head] singular values per head (descending). Returns int32 [n]."""
    th = np.ascontiguousarray(np.asarray(theta, dtype=np.float64))
    if th.ndim != 2:
        raise ValueError("theta must be [n, d_head]")
    out = np.zeros(th.shape[0], dtype=np.int32)
    _check(lib().fdc_select_ranks(th.shape[0], th.shape[1], th.ctypes.data_as(C.POINTER(C.c_double)), float(r),
                                  int(multiple), _p32(out)))
    return out


def fdc_rope_absorb_query(layout: Layout, layer: int, q, tok_pos, cos_t, sin_t, R_t, q_lat, q_lat_dtype: int,
                          stream=None, status=None) -> None:
    _check(lib().fdc_rope_absorb_query(layout.handle, layer, _dev(q), int(q.shape[0]), _dev(tok_pos), _dev(cos_t),
                                       _dev(sin_t), int(cos_t.shape[0]), _dev(R_t), _dev(q_lat), q_lat_dtype,
                                       _dev(status), _stream(stream)))


def fdc_rope_compress_keys(layout: Layout, layer: int, k, tok_batch, tok_pos, cos_t, sin_t, R_t, k_cache,
                           stream=None, status=None) -> None:
    _check(lib().fdc_rope_compress_keys(layout.handle, layer, _dev(k), int(k.shape[0]), _dev(tok_batch),
                                        _dev(tok_pos), _dev(cos_t), _dev(sin_t), int(cos_t.shape[0]), _dev(R_t),
                                        _dev(k_cache), _dev(status), _stream(stream)))
