"""Thin ctypes binding of libattnpred.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in include/attnpred.h.
Tensors are torch CUDA(ROCm) tensors used purely as device memory; the current torch stream is
passed as the hipStream_t.  There is no CPU fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libattnpred.so")

AP_F32, AP_BF16 = 0, 1
AP_PRED_REBASE, AP_PRED_ADVANCE, AP_PRED_HOLD, AP_PRED_SKIP = 0, 1, 2, 3
AP_STEP_REUSE_SELECTION = 16
AP_FLAG_PREDICTOR_FP32 = 1
AP_OK, AP_ERR_ARG, AP_ERR_ALIGN, AP_ERR_RANGE, AP_ERR_HIP, AP_ERR_UNSUPPORTED, AP_ERR_STATE = 0, -1, -2, -3, -4, -5, -6

EXPORTS = [
    "ap_create", "ap_destroy", "ap_workspace_bytes", "ap_hist_slots", "ap_nb_cap", "ap_set_weights", "ap_score_offset", "ap_set_block_table",
    "ap_predict", "ap_predict_incremental", "ap_select_topk", "ap_refresh_selection", "ap_sparse_decode", "ap_sparse_decode_noalloc", "ap_calibrate", "ap_update_history", "ap_step",
    "ap_prefetch_state_bytes", "ap_prefetch_blocks", "ap_append_kv", "ap_offload_begin", "ap_offload_step", "ap_stream_read", "ap_stream_copy", "ap_strerror",
]


class ap_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_inst", "g", "head_dim", "block", "hist_len", "t_cap", "k_blocks", "n_sink", "n_local",
        "c1", "c2", "kv_dtype", "flags")]


class ApError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"attnpred error {code}: {what}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Loads the HIP library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2502_04077_amd.build` "
            "(or __graft_entry__.build()); this package has no other execution path")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    lib.ap_create.argtypes = [C.POINTER(ap_config), C.POINTER(vp)]
    lib.ap_destroy.argtypes = [vp]
    lib.ap_workspace_bytes.argtypes = [vp]
    lib.ap_workspace_bytes.restype = sz
    lib.ap_hist_slots.argtypes = [vp]
    lib.ap_hist_slots.restype = i32
    lib.ap_nb_cap.argtypes = [vp]
    lib.ap_nb_cap.restype = i32
    lib.ap_set_weights.argtypes = [vp, vp, sz, vp]
    lib.ap_score_offset.argtypes = [vp]
    lib.ap_score_offset.restype = C.c_double
    lib.ap_set_block_table.argtypes = [vp, vp, i32]
    lib.ap_predict.argtypes = [vp, vp, i64, i32, vp, vp, vp]
    lib.ap_predict_incremental.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp, vp, vp]
    lib.ap_select_topk.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    lib.ap_refresh_selection.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.ap_sparse_decode.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.ap_sparse_decode_noalloc.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.ap_calibrate.argtypes = [vp, vp, vp, i32, vp, vp, vp]
    lib.ap_update_history.argtypes = [vp, vp, i64, vp, vp]
    lib.ap_step.argtypes = [vp, vp, i64, vp, vp, vp, i32, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.ap_prefetch_state_bytes.argtypes = [vp]
    lib.ap_prefetch_state_bytes.restype = sz
    lib.ap_prefetch_blocks.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.ap_append_kv.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.ap_offload_begin.argtypes = [vp, vp, i64, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.ap_offload_step.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp,
                                    vp, vp, vp, vp]
    lib.ap_stream_read.argtypes = [vp, sz, vp, i32, vp]
    lib.ap_stream_copy.argtypes = [vp, sz, vp, i32, vp]
    lib.ap_strerror.argtypes = [C.c_int]
    lib.ap_strerror.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("ap_workspace_bytes", "ap_prefetch_state_bytes", "ap_hist_slots", "ap_nb_cap", "ap_strerror",
                        "ap_score_offset"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise ApError(rc, load_library().ap_strerror(rc).decode())


def _ptr(t: torch.Tensor) -> int:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


def _rptr(t: torch.Tensor) -> int:
    """A tensor a kernel may read: device memory, or pinned (device-mapped) host memory."""
    if not (t.is_cuda or t.is_pinned()) or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor or pinned host tensor")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def stream_read(src: torch.Tensor, sink: torch.Tensor, n_workgroups: int) -> None:
    _check(load_library().ap_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), n_workgroups,
                                         _stream()))


def stream_copy(src: torch.Tensor, dst: torch.Tensor, n_workgroups: int) -> None:
    _check(load_library().ap_stream_copy(_ptr(src), src.numel() * src.element_size(), _ptr(dst), n_workgroups,
                                         _stream()))


class Context:
    """Owns one ap_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, *, n_inst, g, head_dim, block, hist_len, t_cap, k_blocks, n_sink, n_local, c1, c2,
                 kv_dtype, flags=0):
        lib = load_library()
        self.cfg = ap_config(n_inst, g, head_dim, block, hist_len, t_cap, k_blocks, n_sink, n_local, c1, c2,
                             AP_BF16 if kv_dtype in ("bf16", AP_BF16) else AP_F32, flags)
        h = C.c_void_p()
        _check(lib.ap_create(C.byref(self.cfg), C.byref(h)))
        self._h = h
        self._lib = lib

    def close(self):
        if getattr(self, "_h", None):
            self._lib.ap_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- sizes ------------------------------------------------------------------------------
    def workspace_bytes(self) -> int:
        return int(self._lib.ap_workspace_bytes(self._h))

    def hist_slots(self) -> int:
        return int(self._lib.ap_hist_slots(self._h))

    def nb_cap(self) -> int:
        return int(self._lib.ap_nb_cap(self._h))

    # -- calls ------------------------------------------------------------------------------
    def set_weights(self, blob: np.ndarray) -> None:
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        _check(self._lib.ap_set_weights(self._h, blob.ctypes.data, blob.size, _stream()))

    def score_offset(self) -> float:
        """P0: pred holds the predictor's output minus this constant (see ap_predict in attnpred.h)."""
        return float(self._lib.ap_score_offset(self._h))

    def set_block_table(self, table, n_phys_blocks: int = 0) -> None:
        """table: device int32 [n_inst][nb_cap] (kept alive by the caller), or None for the contiguous layout."""
        _check(self._lib.ap_set_block_table(self._h, None if table is None else _ptr(table), n_phys_blocks))

    def predict(self, hist, n_pushed, nb_cur, pred, ws) -> None:
        _check(self._lib.ap_predict(self._h, _ptr(hist), n_pushed, nb_cur, _ptr(pred), _ptr(ws), _stream()))

    def predict_incremental(self, hist, n_pushed, nb_cur, nb_prev, mode, pstate, pred, ws) -> None:
        _check(self._lib.ap_predict_incremental(self._h, _ptr(hist), n_pushed, nb_cur, nb_prev, mode, _ptr(pstate),
                                                _ptr(pred), _ptr(ws), _stream()))

    def select_topk(self, pred, nb_cur, idx, cnt, ws) -> None:
        _check(self._lib.ap_select_topk(self._h, _ptr(pred), nb_cur, _ptr(idx), _ptr(cnt), _ptr(ws), _stream()))

    def refresh_selection(self, nb_prev, nb_cur, idx, cnt) -> None:
        _check(self._lib.ap_refresh_selection(self._h, nb_prev, nb_cur, _ptr(idx), _ptr(cnt), _stream()))

    def sparse_decode(self, q, K, V, t_cur, idx, cnt, out, row, ws) -> None:
        _check(self._lib.ap_sparse_decode(self._h, _ptr(q), _ptr(K), _ptr(V), t_cur, _ptr(idx), _ptr(cnt),
                                          _ptr(out), _ptr(row), _ptr(ws), _stream()))

    def sparse_decode_noalloc(self, q, K, V, t_cur, idx, cnt, out, row) -> None:
        _check(self._lib.ap_sparse_decode_noalloc(self._h, _ptr(q), _ptr(K), _ptr(V), t_cur, _ptr(idx), _ptr(cnt),
                                                  _ptr(out), _ptr(row), _stream()))

    def calibrate(self, q, K, t_cur, row, ws) -> None:
        _check(self._lib.ap_calibrate(self._h, _ptr(q), _rptr(K), t_cur, _ptr(row), _ptr(ws), _stream()))

    def prefetch_state_bytes(self) -> int:
        return int(self._lib.ap_prefetch_state_bytes(self._h))

    def prefetch_blocks(self, K_src, V_src, t_avail, nb_cur, idx, cnt, pool_K, pool_V, table, state) -> None:
        _check(self._lib.ap_prefetch_blocks(self._h, _rptr(K_src), _rptr(V_src), t_avail, nb_cur, _ptr(idx), _ptr(cnt),
                                            _ptr(pool_K), _ptr(pool_V), _ptr(table), _ptr(state), _stream()))

    def offload_begin(self, hist, n_pushed, K_src, V_src, t_first, idx, cnt, pred, pstate, pool_K, pool_V, table, state,
                      ws, copy_stream) -> None:
        _check(self._lib.ap_offload_begin(self._h, _ptr(hist), n_pushed, _rptr(K_src), _rptr(V_src), t_first, _ptr(idx),
                                          _ptr(cnt), _ptr(pred), _ptr(pstate), _ptr(pool_K), _ptr(pool_V), _ptr(table),
                                          _ptr(state), _ptr(ws), _stream(), copy_stream.cuda_stream))

    def offload_step(self, hist, n_pushed, q, k_new, v_new, K_src, V_src, t_cur, calibrate, out, idx, cnt, pred, pstate,
                     pred_mode, pool_K, pool_V, table, state, row, ws, copy_stream) -> None:
        _check(self._lib.ap_offload_step(self._h, _ptr(hist), n_pushed, _ptr(q), _ptr(k_new), _ptr(v_new), _rptr(K_src),
                                         _rptr(V_src), t_cur, int(bool(calibrate)), _ptr(out), _ptr(idx), _ptr(cnt),
                                         _ptr(pred), _ptr(pstate), pred_mode, _ptr(pool_K), _ptr(pool_V), _ptr(table),
                                         _ptr(state), _ptr(row), _ptr(ws), _stream(), copy_stream.cuda_stream))

    def append_kv(self, k_new, v_new, t_pos, table, state, pool_K, pool_V) -> None:
        _check(self._lib.ap_append_kv(self._h, _ptr(k_new), _ptr(v_new), t_pos, _ptr(table), _ptr(state), _ptr(pool_K),
                                      _ptr(pool_V), _stream()))

    def update_history(self, hist, n_pushed, row) -> None:
        _check(self._lib.ap_update_history(self._h, _ptr(hist), n_pushed, _ptr(row), _stream()))

    def step(self, hist, n_pushed, q, K, V, t_cur, out, idx, cnt, pred, pstate, pred_mode, ws) -> None:
        _check(self._lib.ap_step(self._h, _ptr(hist), n_pushed, _ptr(q), _ptr(K), _ptr(V), t_cur, _ptr(out),
                                 _ptr(idx), _ptr(cnt), _ptr(pred), None if pstate is None else _ptr(pstate),
                                 pred_mode, _ptr(ws), _stream()))
