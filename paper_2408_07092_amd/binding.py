"""Thin ctypes binding of libdsattn.so: argument marshalling only.

Every function has the name and semantics of the C entry point declared in
``include/ds_attn.h``; torch tensors supply device memory and the current
stream, nothing is computed here.  The library must have been built
(``python -m paper_2408_07092_amd.build``); there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch  # imported first so that the HIP runtime torch ships is the one the library binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdsattn.so")

DS_OK = 0
DS_ERR_NULL, DS_ERR_SHAPE, DS_ERR_ALIGN, DS_ERR_WORKSPACE, DS_ERR_UNSUPPORTED, DS_ERR_HIP = -1, -2, -3, -4, -5, -6
DS_CALIB_Q, DS_CALIB_K, DS_CALIB_QK = 0, 1, 2
DS_KV_SPLIT, DS_KV_INTERLEAVED = 0, 1

EXPORTS = [
    "ds_strerror", "ds_version", "ds_calibrate_channels", "ds_build_label", "ds_append_label",
    "ds_workspace_bytes", "ds_workspace_init", "ds_workspace_errors", "ds_sparse_decode", "ds_sparse_decode_nolabel",
    "ds_static_scratch_bytes", "ds_static_init", "ds_sparse_decode_static",
    "ds_sparse_decode_kv", "ds_append_kv", "ds_build_label_kv", "ds_build_label_q4",
    "ds_append_label_q4", "ds_sparse_decode_q4", "ds_predict_query", "ds_dense_decode", "ds_select",
    "ds_gather_rows_host", "ds_attend_rows", "ds_probe_stream_read", "ds_profile_kernel_count",
    "ds_profile_kernel_name", "ds_profile_enable", "ds_profile_reset", "ds_profile_read",
    "ds_tune_set", "ds_tune_get", "ds_plan_describe", "ds_pretend_device",
]


class DsShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "Hq", "Hkv", "d", "L", "L_max", "r", "k")]


class DsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2408_07092_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        shp = ctypes.POINTER(DsShape)
        L.ds_strerror.restype = ctypes.c_char_p
        L.ds_strerror.argtypes = [ctypes.c_int]
        L.ds_version.restype = ctypes.c_int
        L.ds_calibrate_channels.argtypes = [vp, vp, i32, i32, i32, i32, i32, ctypes.c_int, vp]
        L.ds_build_label.argtypes = [vp, vp, vp, shp, vp]
        L.ds_append_label.argtypes = [vp, vp, vp, shp, i32, i32, vp]
        L.ds_workspace_bytes.restype = sz
        L.ds_workspace_bytes.argtypes = [shp]
        L.ds_workspace_init.argtypes = [vp, sz, vp]
        L.ds_workspace_errors.argtypes = [vp, sz, shp, vp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        L.ds_sparse_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, shp, vp]
        L.ds_static_scratch_bytes.restype = sz
        L.ds_static_scratch_bytes.argtypes = []
        L.ds_static_init.argtypes = []
        L.ds_sparse_decode_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, shp, vp]
        L.ds_sparse_decode_nolabel.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, shp, vp]
        L.ds_sparse_decode_kv.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, shp, vp]
        L.ds_append_kv.argtypes = [vp, vp, vp, vp, vp, vp, shp, i32, i32, ctypes.c_int, vp]
        L.ds_build_label_kv.argtypes = [vp, vp, vp, shp, vp]
        L.ds_predict_query.argtypes = [vp, vp, vp, i32, i32, i32, vp]
        L.ds_build_label_q4.argtypes = [vp, vp, vp, vp, shp, vp]
        L.ds_append_label_q4.argtypes = [vp, vp, vp, vp, shp, i32, i32, vp]
        L.ds_sparse_decode_q4.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, shp, vp]
        L.ds_dense_decode.argtypes = [vp, vp, vp, vp, vp, sz, shp, vp]
        L.ds_select.argtypes = [vp, vp, vp, vp, vp, sz, shp, vp]
        L.ds_gather_rows_host.argtypes = [vp, vp, vp, vp, shp, vp]
        L.ds_attend_rows.argtypes = [vp, vp, vp, vp, sz, shp, vp]
        L.ds_probe_stream_read.argtypes = [vp, sz, vp, vp]
        L.ds_profile_kernel_name.restype = ctypes.c_char_p
        L.ds_profile_kernel_name.argtypes = [ctypes.c_int]
        L.ds_profile_enable.argtypes = [ctypes.c_int]
        L.ds_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_int64)]
        L.ds_tune_set.argtypes = [ctypes.c_int, ctypes.c_int]
        L.ds_tune_get.argtypes = [ctypes.c_int]
        L.ds_plan_describe.argtypes = [shp, i32, ctypes.POINTER(ctypes.c_int32)]
        L.ds_pretend_device.argtypes = [i32, i32, i32]
        for name in EXPORTS:
            getattr(L, name)  # AttributeError names a missing export
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().ds_strerror(status).decode()


def _check(status: int, where: str):
    if status != DS_OK:
        raise DsError(status, where)


def shape(B, Hq, Hkv, d, L, L_max, r, k) -> DsShape:
    return DsShape(B, Hq, Hkv, d, L, L_max, r, k)


def _dp(t):
    """Device (or pinned-host) pointer of a contiguous tensor, or NULL."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def ds_version() -> int:
    return lib().ds_version()


def ds_calibrate_channels(q_calib: np.ndarray, k_calib: np.ndarray, r: int, mode: int) -> np.ndarray:
    """Host arrays: q_calib [N,Hq,d], k_calib [N,Hkv,d] float16 -> channels [Hkv,r] int32."""
    q_calib = np.ascontiguousarray(q_calib); k_calib = np.ascontiguousarray(k_calib)
    if q_calib.dtype != np.float16 or k_calib.dtype != np.float16:
        raise TypeError("calibration samples must be float16")
    N, Hq, d = q_calib.shape
    Hkv = k_calib.shape[1]
    out = np.empty((Hkv, max(r, 0)), dtype=np.int32)
    st = lib().ds_calibrate_channels(q_calib.ctypes.data, k_calib.ctypes.data, N, Hq, Hkv, d, r, mode,
                                     out.ctypes.data)
    _check(st, "ds_calibrate_channels")
    return out


def ds_build_label(K, channels, label, shp: DsShape, stream=None):
    _check(lib().ds_build_label(_dp(K), _dp(channels), _dp(label), ctypes.byref(shp), _stream(stream)),
           "ds_build_label")


def ds_append_label(K, channels, label, shp: DsShape, t0: int, n_new: int, stream=None):
    _check(lib().ds_append_label(_dp(K), _dp(channels), _dp(label), ctypes.byref(shp), t0, n_new,
                                 _stream(stream)), "ds_append_label")


def ds_workspace_bytes(shp: DsShape) -> int:
    return int(lib().ds_workspace_bytes(ctypes.byref(shp)))


def ds_workspace_init(workspace, stream=None):
    _check(lib().ds_workspace_init(_dp(workspace), workspace.numel() * workspace.element_size(),
                                   _stream(stream)), "ds_workspace_init")


def ds_workspace_errors(workspace, shp: DsShape, stream=None):
    """(units whose bounded wait gave up, first error code); waits for the stream."""
    n, first = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().ds_workspace_errors(_dp(workspace), workspace.numel() * workspace.element_size(),
                                     ctypes.byref(shp), _stream(stream), ctypes.byref(n), ctypes.byref(first)),
           "ds_workspace_errors")
    return n.value, first.value


def ds_workspace_alloc(shp: DsShape, device="cuda") -> "torch.Tensor":
    """torch-allocated, cleared workspace for `shp` (convenience of the binding).  The clearing
    runs on the current stream and is waited for, so the workspace may be used on any stream."""
    n = ds_workspace_bytes(shp)
    if n == 0:
        raise DsError(DS_ERR_SHAPE, "ds_workspace_bytes")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    ds_workspace_init(ws)
    torch.cuda.current_stream(ws.device).synchronize()
    return ws


def ds_sparse_decode(q, label, K, V, channels, out, idx_out, workspace, shp: DsShape, stream=None):
    _check(lib().ds_sparse_decode(_dp(q), _dp(label), _dp(K), _dp(V), _dp(channels), _dp(out),
                                  _dp(idx_out), _dp(workspace),
                                  workspace.numel() * workspace.element_size(),
                                  ctypes.byref(shp), _stream(stream)), "ds_sparse_decode")


def ds_static_scratch_bytes() -> int:
    return int(lib().ds_static_scratch_bytes())


def ds_static_init():
    _check(lib().ds_static_init(), "ds_static_init")


def ds_sparse_decode_static(q, label, K, V, channels, out, idx_out, shp: DsShape, stream=None):
    _check(lib().ds_sparse_decode_static(_dp(q), _dp(label), _dp(K), _dp(V), _dp(channels), _dp(out),
                                         _dp(idx_out), ctypes.byref(shp), _stream(stream)),
           "ds_sparse_decode_static")


def ds_sparse_decode_nolabel(q, K, V, channels, out, idx_out, workspace, shp: DsShape, stream=None):
    _check(lib().ds_sparse_decode_nolabel(_dp(q), _dp(K), _dp(V), _dp(channels), _dp(out),
                                          _dp(idx_out), _dp(workspace),
                                          workspace.numel() * workspace.element_size(),
                                          ctypes.byref(shp), _stream(stream)), "ds_sparse_decode_nolabel")


def ds_sparse_decode_kv(q, label, KV, channels, out, idx_out, workspace, shp: DsShape, stream=None):
    _check(lib().ds_sparse_decode_kv(_dp(q), _dp(label), _dp(KV), _dp(channels), _dp(out),
                                     _dp(idx_out), _dp(workspace),
                                     workspace.numel() * workspace.element_size(),
                                     ctypes.byref(shp), _stream(stream)), "ds_sparse_decode_kv")


def ds_append_kv(k_new, v_new, K, V, channels, label, shp: DsShape, t0, n_new, layout=DS_KV_SPLIT, stream=None):
    _check(lib().ds_append_kv(_dp(k_new), _dp(v_new), _dp(K), _dp(V), _dp(channels), _dp(label),
                              ctypes.byref(shp), int(t0), int(n_new), int(layout), _stream(stream)),
           "ds_append_kv")


def ds_build_label_kv(KV, channels, label, shp: DsShape, stream=None):
    _check(lib().ds_build_label_kv(_dp(KV), _dp(channels), _dp(label), ctypes.byref(shp), _stream(stream)),
           "ds_build_label_kv")


def ds_build_label_q4(K, channels, label_q4, amax, shp: DsShape, stream=None):
    _check(lib().ds_build_label_q4(_dp(K), _dp(channels), _dp(label_q4), _dp(amax), ctypes.byref(shp),
                                   _stream(stream)), "ds_build_label_q4")


def ds_append_label_q4(K, channels, label_q4, amax, shp: DsShape, t0, n_new, stream=None):
    _check(lib().ds_append_label_q4(_dp(K), _dp(channels), _dp(label_q4), _dp(amax), ctypes.byref(shp),
                                    int(t0), int(n_new), _stream(stream)), "ds_append_label_q4")


def ds_sparse_decode_q4(q, label_q4, amax, K, V, channels, out, idx_out, workspace, shp: DsShape, stream=None):
    _check(lib().ds_sparse_decode_q4(_dp(q), _dp(label_q4), _dp(amax), _dp(K), _dp(V), _dp(channels),
                                     _dp(out), _dp(idx_out), _dp(workspace),
                                     workspace.numel() * workspace.element_size(),
                                     ctypes.byref(shp), _stream(stream)), "ds_sparse_decode_q4")


def ds_predict_query(x, Wq, q_out, stream=None):
    """x [B, Dm], Wq [N, Dm], q_out [B, ...] with N elements per batch row (all fp16)."""
    B, Dm = x.shape
    N = Wq.shape[0]
    assert Wq.shape[1] == Dm and q_out.numel() == B * N
    _check(lib().ds_predict_query(_dp(x), _dp(Wq), _dp(q_out), B, Dm, N, _stream(stream)), "ds_predict_query")


def ds_dense_decode(q, K, V, out, workspace, shp: DsShape, stream=None):
    _check(lib().ds_dense_decode(_dp(q), _dp(K), _dp(V), _dp(out), _dp(workspace),
                                 workspace.numel() * workspace.element_size(),
                                 ctypes.byref(shp), _stream(stream)), "ds_dense_decode")


def ds_select(q, label, channels, idx_out, workspace, shp: DsShape, stream=None):
    _check(lib().ds_select(_dp(q), _dp(label), _dp(channels), _dp(idx_out), _dp(workspace),
                           workspace.numel() * workspace.element_size(),
                           ctypes.byref(shp), _stream(stream)), "ds_select")


def ds_gather_rows_host(K_host, V_host, idx, KV_rows, shp: DsShape, stream=None):
    _check(lib().ds_gather_rows_host(_dp(K_host), _dp(V_host), _dp(idx), _dp(KV_rows),
                                     ctypes.byref(shp), _stream(stream)), "ds_gather_rows_host")


def ds_attend_rows(q, KV_rows, out, workspace, shp: DsShape, stream=None):
    _check(lib().ds_attend_rows(_dp(q), _dp(KV_rows), _dp(out), _dp(workspace),
                                workspace.numel() * workspace.element_size(),
                                ctypes.byref(shp), _stream(stream)), "ds_attend_rows")


def ds_probe_stream_read(src, sink, stream=None, nbytes: int | None = None):
    n = src.numel() * src.element_size() if nbytes is None else nbytes
    _check(lib().ds_probe_stream_read(_dp(src), n, _dp(sink), _stream(stream)), "ds_probe_stream_read")


def ds_profile_enable(on: bool):
    _check(lib().ds_profile_enable(1 if on else 0), "ds_profile_enable")


def ds_profile_reset():
    _check(lib().ds_profile_reset(), "ds_profile_reset")


def ds_profile_read() -> dict:
    """{kernel name: (total_ms, launches)} for kernels launched since the last reset."""
    L = lib()
    out = {}
    for i in range(L.ds_profile_kernel_count()):
        ms, n = ctypes.c_double(0), ctypes.c_int64(0)
        _check(L.ds_profile_read(i, ctypes.byref(ms), ctypes.byref(n)), "ds_profile_read")
        if n.value:
            out[L.ds_profile_kernel_name(i).decode()] = (ms.value, n.value)
    return out


def ds_tune_set(knob: int, value: int):
    _check(lib().ds_tune_set(knob, value), "ds_tune_set")


def ds_tune_get(knob: int) -> int:
    return lib().ds_tune_get(knob)


def ds_plan_describe(shp: DsShape, label_kind: int = 0) -> dict:
    out = (ctypes.c_int32 * 8)()
    _check(lib().ds_plan_describe(ctypes.byref(shp), label_kind, out), "ds_plan_describe")
    keys = ("launches_planned", "launches", "tokens_per_workgroup", "workgroups_per_unit", "workgroups",
            "compute_units", "scores_itself", "heads_per_kv_head")
    return dict(zip(keys, list(out)))


def ds_pretend_device(cus: int, xccs: int, lds_per_cu: int):
    _check(lib().ds_pretend_device(cus, xccs, lds_per_cu), "ds_pretend_device")
