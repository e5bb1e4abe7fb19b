"""ctypes binding of libmllm_stage.so: same names as the C ABI, argument marshalling only.

Tensors are anything with `.data_ptr()` (PyTorch device tensors: PyTorch only provides device
memory and the stream) or plain integer device addresses.  Every step of the path runs inside
the library's kernels; there is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmllm_stage.so")

MLLM_OK = 0
STATUS_NAMES = ["MLLM_OK", "MLLM_ERR_NULL", "MLLM_ERR_DESC", "MLLM_ERR_SHAPE", "MLLM_ERR_CU_SEQLENS",
                "MLLM_ERR_MASK_KIND", "MLLM_ERR_INDEX", "MLLM_ERR_WORKSPACE", "MLLM_ERR_UNSUPPORTED",
                "MLLM_ERR_HIP"]

EXPORTS = ["mllm_stage_create", "mllm_stage_destroy", "mllm_stage_param_count", "mllm_stage_param_info",
           "mllm_stage_sizes", "mllm_stage_fwd", "mllm_stage_bwd", "mllm_last_error", "mllm_op_gemm",
           "mllm_op_gemm_swiglu", "mllm_op_gemm_swiglu_bwd", "mllm_op_attn_workspace_bytes", "mllm_attn_work_list", "mllm_op_attn_fwd", "mllm_op_attn_bwd", "mllm_op_norm_fwd",
           "mllm_op_norm_bwd_partial_bytes", "mllm_op_norm_bwd", "mllm_op_norm_bwd_colsum", "mllm_op_rope", "mllm_op_rope_table", "mllm_op_gemm_rope", "mllm_op_attn_bwd_rope", "mllm_op_act_fwd",
           "mllm_op_act_bwd", "mllm_op_colsum_partial_bytes", "mllm_op_colsum", "mllm_op_colsum_static_max_bytes", "mllm_op_colsum_static", "mllm_profile_begin",
           "mllm_profile_end", "mllm_schedule_lpt", "mllm_schedule", "mllm_interp", "mllm_item_durations",
           "mllm_find_combs", "mllm_evaluate_parallelism", "mllm_optimize_parallelism"]

PROFILE_CLASSES = ["gemm_fwd", "gemm_dx", "gemm_dw", "attn_fwd", "attn_bwd", "elementwise", "gemm_small",
                   "gemm_rows192"]


class MllmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status, message))
        self.status = status


class LayerDescC(C.Structure):
    _fields_ = [("kind", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ff", C.c_int32),
                ("d_out", C.c_int32), ("act", C.c_int32), ("has_bias", C.c_int32),
                ("norm_eps", C.c_float), ("rope_base", C.c_float), ("pool", C.c_int32),
                ("merge", C.c_int32), ("qk_norm", C.c_int32)]


class StageDescC(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(LayerDescC))]


class CurveC(C.Structure):
    _fields_ = [("n", C.c_int32), ("x", C.POINTER(C.c_double)), ("y", C.POINTER(C.c_double))]


class ModuleProfileC(C.Structure):
    _fields_ = [("n_tp", C.c_int32), ("tp", C.POINTER(C.c_int32)), ("n_x", C.c_int32),
                ("x", C.POINTER(C.c_double)), ("thr", C.POINTER(C.c_double)),
                ("layers_lo", C.c_double), ("layers_hi", C.c_double),
                ("model_state", C.POINTER(C.c_double)), ("act_state", C.POINTER(C.c_double)),
                ("n_layers", C.c_int32), ("flop_per_item", C.c_double)]


class PackC(C.Structure):
    _fields_ = [("total_tokens", C.c_int32), ("n_segments", C.c_int32), ("max_seqlen", C.c_int32),
                ("cu_seqlens_host", C.POINTER(C.c_int32)), ("mask_kind_host", C.POINTER(C.c_uint8))]


class BatchC(C.Structure):
    _fields_ = [("img", PackC), ("seq", PackC), ("img_to_seq_row_host", C.POINTER(C.c_int32))]


_lib = None


def lib() -> C.CDLL:
    """Load the HIP library; raise if it was not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: build it with `python -m paper_2603_25120_amd.build`" % LIB_PATH)
    # One process, one HIP runtime: PyTorch (which owns the device memory handed to the library)
    # ships its own libamdhip64 with the same soname as the system one this library links to.
    # Loading PyTorch first makes the dynamic linker bind both to the same copy; the other order
    # would put two runtimes in the process, and the second cannot see the GPU.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.mllm_last_error.restype = C.c_char_p
    L.mllm_stage_create.argtypes = [C.POINTER(StageDescC), C.POINTER(vp)]
    L.mllm_stage_destroy.argtypes = [vp]
    L.mllm_stage_destroy.restype = None
    L.mllm_stage_param_count.argtypes = [vp]
    L.mllm_stage_param_count.restype = sz
    L.mllm_stage_param_info.argtypes = [vp, sz, C.POINTER(C.c_char_p), C.POINTER(i32), C.POINTER(i64), C.POINTER(i64)]
    L.mllm_stage_sizes.argtypes = [vp, C.POINTER(BatchC), C.POINTER(sz), C.POINTER(sz)]
    L.mllm_stage_fwd.argtypes = [vp, C.POINTER(BatchC), C.POINTER(vp), vp, vp, vp, vp, sz, vp, sz, vp]
    L.mllm_stage_bwd.argtypes = [vp, C.POINTER(BatchC), C.POINTER(vp), vp, vp, sz, vp, vp, C.POINTER(vp), C.c_int, vp, sz, vp]
    L.mllm_op_gemm.argtypes = [vp, vp, vp, i64, i64, i64, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp, vp]
    L.mllm_op_gemm_swiglu.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp]
    L.mllm_op_gemm_swiglu_bwd.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp]
    L.mllm_op_attn_workspace_bytes.argtypes = [i32, i32, i32]
    L.mllm_op_attn_workspace_bytes.restype = sz
    L.mllm_attn_work_list.argtypes = [C.POINTER(PackC), i32, i32, i32, i32, vp, sz, C.POINTER(sz), C.POINTER(i32)]
    L.mllm_op_attn_fwd.argtypes = [vp, vp, vp, vp, vp, C.POINTER(PackC), i32, i32, i32, i64, i64, i64, vp, sz, vp]
    L.mllm_op_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.POINTER(PackC), i32, i32, i32, i64, i64, i64, vp, sz, vp]
    L.mllm_op_norm_fwd.argtypes = [C.c_int, vp, vp, vp, vp, vp, i64, i64, C.c_float, vp]
    L.mllm_op_norm_bwd_partial_bytes.argtypes = [i64, i64]
    L.mllm_op_norm_bwd_partial_bytes.restype = sz
    L.mllm_op_norm_bwd.argtypes = [C.c_int, vp, vp, vp, vp, vp, vp, vp, vp, C.c_int, vp, i64, i64, vp]
    L.mllm_op_norm_bwd_colsum.argtypes = [C.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_int, vp, i64, i64, vp]
    L.mllm_op_rope.argtypes = [vp, vp, i64, i64, i64, i32, i32, C.c_float, C.c_int, vp]
    L.mllm_op_rope_table.argtypes = [vp, i64, i32, C.c_float, vp]
    L.mllm_op_gemm_rope.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp, i64, i32, vp]
    L.mllm_op_attn_bwd_rope.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.POINTER(PackC), i32, i32, i32, i64, i64, i64, vp, vp, sz, vp]
    L.mllm_op_act_fwd.argtypes = [C.c_int, vp, vp, i64, i64, vp]
    L.mllm_op_act_bwd.argtypes = [C.c_int, vp, vp, vp, i64, i64, vp]
    L.mllm_op_colsum_partial_bytes.argtypes = [i64, i64]
    L.mllm_op_colsum_partial_bytes.restype = sz
    L.mllm_op_colsum.argtypes = [vp, vp, C.c_int, vp, i64, i64, vp]
    L.mllm_op_colsum_static_max_bytes.argtypes = []
    L.mllm_op_colsum_static_max_bytes.restype = sz
    L.mllm_op_colsum_static.argtypes = [vp, vp, C.c_int, i64, i64, vp]
    L.mllm_profile_begin.argtypes = [i32]
    L.mllm_profile_end.argtypes = [C.POINTER(i64), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(i64)]
    dp, ip = C.POINTER(C.c_double), C.POINTER(i32)
    L.mllm_schedule_lpt.argtypes = [i64, dp, dp, i32, ip]
    L.mllm_schedule.argtypes = [i64, dp, dp, i32, i64, ip, dp, ip]
    cp, mp = C.POINTER(CurveC), C.POINTER(ModuleProfileC)
    L.mllm_interp.argtypes = [cp, i64, dp, i32, dp]
    L.mllm_item_durations.argtypes = [i64, dp, dp, dp, dp, dp, cp, cp, cp, dp, dp]
    L.mllm_find_combs.argtypes = [i32, i32, i32, i64, ip, C.POINTER(i64)]
    L.mllm_evaluate_parallelism.argtypes = [mp, mp, ip, C.c_double, i32, C.c_double, C.c_double, dp, dp, dp, ip]
    L.mllm_optimize_parallelism.argtypes = [mp, mp, i32, i32, C.c_double, i32, C.c_double, C.c_double, ip, dp, ip]
    for name in EXPORTS:
        getattr(L, name)          # every declared entry point must be exported
    _lib = L
    return L


def _check(status: int):
    if status != MLLM_OK:
        raise MllmError(status, lib().mllm_last_error().decode())


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _nbytes(t) -> int:
    return int(t.numel() * t.element_size())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


class _PackKeep:
    """ctypes view of a packed token space; keeps the NumPy arrays alive."""

    def __init__(self, pack):
        self.c = PackC()
        if pack is None:
            self.cu = np.zeros(1, dtype=np.int32)
            self.mk = np.zeros(0, dtype=np.uint8)
            n_seg, total, longest = 0, 0, 0
        else:
            self.cu = np.ascontiguousarray(pack.cu_seqlens, dtype=np.int32)
            self.mk = np.ascontiguousarray(pack.mask_kind, dtype=np.uint8)
            n_seg = len(self.mk)
            total = int(getattr(pack, "total_tokens_override", self.cu[-1]))
            longest = getattr(pack, "max_seqlen_override", None)
            if longest is None:
                longest = int(np.max(np.diff(self.cu))) if n_seg else 0
        self.c.total_tokens, self.c.n_segments, self.c.max_seqlen = total, n_seg, int(longest)
        self.c.cu_seqlens_host = self.cu.ctypes.data_as(C.POINTER(C.c_int32))
        self.c.mask_kind_host = self.mk.ctypes.data_as(C.POINTER(C.c_uint8))


class _BatchKeep:
    def __init__(self, batch):
        self.img = _PackKeep(getattr(batch, "img", None))
        self.seq = _PackKeep(getattr(batch, "seq", None))
        self.c = BatchC()
        self.c.img, self.c.seq = self.img.c, self.seq.c
        rows = getattr(batch, "img_to_seq_row", None)
        if rows is not None:
            self.rows = np.ascontiguousarray(rows, dtype=np.int32)
            self.c.img_to_seq_row_host = self.rows.ctypes.data_as(C.POINTER(C.c_int32))


def _ptr_array(tensors: Sequence):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = _ptr(t)
    return arr


# -------------------------------------------------------------------------------------------
# stage entry points
# -------------------------------------------------------------------------------------------
def mllm_stage_create(layers: Sequence) -> int:
    """layers: objects with the fields of mllm_layer_desc_t.  Returns the opaque handle."""
    arr = (LayerDescC * len(layers))()
    for i, l in enumerate(layers):
        for f, _ in LayerDescC._fields_:
            setattr(arr[i], f, getattr(l, f, 0) if f == "qk_norm" else getattr(l, f))
    desc = StageDescC(len(layers), arr)
    out = C.c_void_p()
    _check(lib().mllm_stage_create(C.byref(desc), C.byref(out)))
    return out.value


def mllm_stage_destroy(handle: int) -> None:
    lib().mllm_stage_destroy(handle)


def mllm_stage_param_count(handle: int) -> int:
    return int(lib().mllm_stage_param_count(handle))


def mllm_stage_param_info(handle: int, i: int):
    name, layer, rows, cols = C.c_char_p(), C.c_int32(), C.c_int64(), C.c_int64()
    _check(lib().mllm_stage_param_info(handle, i, C.byref(name), C.byref(layer), C.byref(rows), C.byref(cols)))
    return name.value.decode(), layer.value, rows.value, cols.value


def mllm_stage_sizes(handle: int, batch):
    bk = _BatchKeep(batch)
    a, b = C.c_size_t(), C.c_size_t()
    _check(lib().mllm_stage_sizes(handle, C.byref(bk.c), C.byref(a), C.byref(b)))
    return a.value, b.value


def mllm_stage_fwd(handle, batch, params, x_img, x_seq, y, saved, workspace, stream=None,
                   saved_bytes=None, workspace_bytes=None) -> None:
    bk = _BatchKeep(batch)
    _check(lib().mllm_stage_fwd(handle, C.byref(bk.c), _ptr_array(params), _ptr(x_img), _ptr(x_seq), _ptr(y),
                                _ptr(saved), _nbytes(saved) if saved_bytes is None else saved_bytes,
                                _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes,
                                _stream(stream)))


def mllm_stage_bwd(handle, batch, params, dy, saved, dx_img, dx_seq, dparams, accumulate, workspace,
                   stream=None, saved_bytes=None, workspace_bytes=None) -> None:
    bk = _BatchKeep(batch)
    _check(lib().mllm_stage_bwd(handle, C.byref(bk.c), _ptr_array(params), _ptr(dy), _ptr(saved),
                                _nbytes(saved) if saved_bytes is None else saved_bytes, _ptr(dx_img), _ptr(dx_seq),
                                _ptr_array(dparams), int(accumulate), _ptr(workspace),
                                _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream)))


def mllm_last_error() -> str:
    return lib().mllm_last_error().decode()


# -------------------------------------------------------------------------------------------
# single operations
# -------------------------------------------------------------------------------------------
def mllm_op_gemm(a, b, c, m, n, k, a_layout=0, b_layout=0, out_fp32=0, accumulate=0, bias=None,
                 residual=None, stream=None) -> None:
    _check(lib().mllm_op_gemm(_ptr(a), _ptr(b), _ptr(c), m, n, k, a_layout, b_layout, out_fp32, accumulate,
                              _ptr(bias), _ptr(residual), _stream(stream)))


def mllm_op_gemm_swiglu(x, w_gu, pre, act, m, f, k, stream=None) -> None:
    _check(lib().mllm_op_gemm_swiglu(_ptr(x), _ptr(w_gu), _ptr(pre), _ptr(act), m, f, k, _stream(stream)))


def mllm_op_gemm_swiglu_bwd(dy, w_d, pre, dpre, m, f, k, stream=None) -> None:
    _check(lib().mllm_op_gemm_swiglu_bwd(_ptr(dy), _ptr(w_d), _ptr(pre), _ptr(dpre), m, f, k, _stream(stream)))


def mllm_op_attn_workspace_bytes(n_segments: int, total_tokens: int, n_q_heads: int) -> int:
    return int(lib().mllm_op_attn_workspace_bytes(n_segments, total_tokens, n_q_heads))


def mllm_attn_work_list(pack, kv_major: bool, n_q_heads: int, n_kv_heads: int, head_dim: int) -> np.ndarray:
    """The launch's entries [grid, 5] = seg_start, seg_len, tile0, causal, head (seg_len 0: empty entry)."""
    pk = _PackKeep(pack)
    need, grid = C.c_size_t(), C.c_int32()
    _check(lib().mllm_attn_work_list(C.byref(pk.c), int(kv_major), n_q_heads, n_kv_heads, head_dim, None, 0,
                                     C.byref(need), C.byref(grid)))
    buf = np.zeros(max(need.value // 4, 5), dtype=np.int32)
    _check(lib().mllm_attn_work_list(C.byref(pk.c), int(kv_major), n_q_heads, n_kv_heads, head_dim,
                                     buf.ctypes.data_as(C.c_void_p), buf.nbytes, C.byref(need), C.byref(grid)))
    return buf[:5 * grid.value].reshape(-1, 5).copy()


def mllm_op_attn_fwd(q, k, v, o, lse, pack, n_q_heads, n_kv_heads, head_dim, q_stride, kv_stride, o_stride,
                     workspace, stream=None) -> None:
    pk = _PackKeep(pack)
    _check(lib().mllm_op_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), C.byref(pk.c), n_q_heads,
                                  n_kv_heads, head_dim, q_stride, kv_stride, o_stride, _ptr(workspace),
                                  _nbytes(workspace), _stream(stream)))


def mllm_op_attn_bwd(q, k, v, o, lse, d_o, dq, dk, dv, delta, pack, n_q_heads, n_kv_heads, head_dim, q_stride,
                     kv_stride, o_stride, workspace, stream=None) -> None:
    pk = _PackKeep(pack)
    _check(lib().mllm_op_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq), _ptr(dk),
                                  _ptr(dv), _ptr(delta), C.byref(pk.c), n_q_heads, n_kv_heads, head_dim,
                                  q_stride, kv_stride, o_stride, _ptr(workspace), _nbytes(workspace),
                                  _stream(stream)))


def mllm_op_norm_fwd(kind, x, gamma, beta, y, stats, t, d, eps, stream=None) -> None:
    _check(lib().mllm_op_norm_fwd(kind, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(stats), t, d, eps,
                                  _stream(stream)))


def mllm_op_norm_bwd_partial_bytes(t: int, d: int) -> int:
    return int(lib().mllm_op_norm_bwd_partial_bytes(t, d))


def mllm_op_norm_bwd_colsum(kind, dy, x, gamma, stats, dres, dx, dgamma, dbeta, dx_colsum, accumulate, partial, t, d,
                            stream=None) -> None:
    _check(lib().mllm_op_norm_bwd_colsum(kind, _ptr(dy), _ptr(x), _ptr(gamma), _ptr(stats), _ptr(dres), _ptr(dx),
                                         _ptr(dgamma), _ptr(dbeta), _ptr(dx_colsum), int(accumulate), _ptr(partial), t, d,
                                         _stream(stream)))


def mllm_op_norm_bwd(kind, dy, x, gamma, stats, dres, dx, dgamma, dbeta, accumulate, partial, t, d,
                     stream=None) -> None:
    _check(lib().mllm_op_norm_bwd(kind, _ptr(dy), _ptr(x), _ptr(gamma), _ptr(stats), _ptr(dres), _ptr(dx),
                                  _ptr(dgamma), _ptr(dbeta), int(accumulate), _ptr(partial), t, d,
                                  _stream(stream)))


def mllm_op_rope(qk, pos, t, row_stride, col0, n_heads, head_dim, rope_base, inverse=0, stream=None) -> None:
    _check(lib().mllm_op_rope(_ptr(qk), _ptr(pos), t, row_stride, col0, n_heads, head_dim, rope_base,
                              int(inverse), _stream(stream)))


def mllm_op_rope_table(table, n_pos, head_dim, rope_base, stream=None) -> None:
    _check(lib().mllm_op_rope_table(_ptr(table), n_pos, head_dim, rope_base, _stream(stream)))


def mllm_op_gemm_rope(x, w, bias, y, m, n, k, pos, rope_table, rope_cols, head_dim, stream=None) -> None:
    _check(lib().mllm_op_gemm_rope(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), m, n, k, _ptr(pos), _ptr(rope_table),
                                   rope_cols, head_dim, _stream(stream)))


def mllm_op_attn_bwd_rope(q, k, v, o, lse, d_o, dq, dk, dv, delta, pack, n_q_heads, n_kv_heads, head_dim, q_stride,
                          kv_stride, o_stride, rope_table, workspace, stream=None) -> None:
    pk = _PackKeep(pack)
    _check(lib().mllm_op_attn_bwd_rope(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq), _ptr(dk),
                                       _ptr(dv), _ptr(delta), C.byref(pk.c), n_q_heads, n_kv_heads, head_dim,
                                       q_stride, kv_stride, o_stride, _ptr(rope_table), _ptr(workspace),
                                       _nbytes(workspace), _stream(stream)))


def mllm_op_act_fwd(act, pre, a, t, f, stream=None) -> None:
    _check(lib().mllm_op_act_fwd(act, _ptr(pre), _ptr(a), t, f, _stream(stream)))


def mllm_op_act_bwd(act, da, pre, dpre, t, f, stream=None) -> None:
    _check(lib().mllm_op_act_bwd(act, _ptr(da), _ptr(pre), _ptr(dpre), t, f, _stream(stream)))


def mllm_op_colsum_partial_bytes(t: int, n: int) -> int:
    return int(lib().mllm_op_colsum_partial_bytes(t, n))


def mllm_op_colsum(x, out, accumulate, partial, t, n, stream=None) -> None:
    _check(lib().mllm_op_colsum(_ptr(x), _ptr(out), int(accumulate), _ptr(partial), t, n, _stream(stream)))


def mllm_op_colsum_static_max_bytes() -> int:
    return int(lib().mllm_op_colsum_static_max_bytes())


def mllm_op_colsum_static(x, out, accumulate, t, n, stream=None) -> None:
    _check(lib().mllm_op_colsum_static(_ptr(x), _ptr(out), int(accumulate), t, n, _stream(stream)))


def mllm_profile_begin(max_records: int) -> None:
    _check(lib().mllm_profile_begin(max_records))


def mllm_profile_end():
    """Returns {class: (launches, milliseconds, work)} and the number of dropped records."""
    n = len(PROFILE_CLASSES)
    launches, ms, work, dropped = (C.c_int64 * n)(), (C.c_double * n)(), (C.c_double * n)(), C.c_int64()
    _check(lib().mllm_profile_end(launches, ms, work, C.byref(dropped)))
    return {PROFILE_CLASSES[i]: (int(launches[i]), float(ms[i]), float(work[i])) for i in range(n)}, int(dropped.value)


def _dvec(x):
    a = np.ascontiguousarray(x, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def mllm_schedule_lpt(e_dur, l_dur, n_buckets: int) -> np.ndarray:
    """Bucket index per item by longest-processing-time-first."""
    e, ep = _dvec(e_dur)
    l, lp = _dvec(l_dur)
    out = np.zeros(len(e), dtype=np.int32)
    _check(lib().mllm_schedule_lpt(len(e), ep, lp, n_buckets, out.ctypes.data_as(C.POINTER(C.c_int32))))
    return out


def mllm_schedule(e_dur, l_dur, n_buckets: int, node_limit: int = 1_000_000):
    """(bucket index per item, C_max of that assignment, whether it is proven optimal)."""
    e, ep = _dvec(e_dur)
    l, lp = _dvec(l_dur)
    out = np.zeros(len(e), dtype=np.int32)
    cmax, optimal = C.c_double(), C.c_int32()
    _check(lib().mllm_schedule(len(e), ep, lp, n_buckets, node_limit, out.ctypes.data_as(C.POINTER(C.c_int32)),
                               C.byref(cmax), C.byref(optimal)))
    return out, cmax.value, bool(optimal.value)


def _curve(xy):
    """(x, y) -> CurveC plus the arrays that must outlive the call."""
    x, xp = _dvec(xy[0])
    y, yp = _dvec(xy[1])
    if x.ndim != 1 or x.shape != y.shape:
        raise ValueError("a curve is two equally long 1-d arrays")
    return CurveC(len(x), xp, yp), (x, y)


def mllm_interp(x, y, q, extrapolate: bool = False) -> np.ndarray:
    """Piecewise-linear function through (x, y) at the points q."""
    c, keep = _curve((x, y))
    qa, qp = _dvec(np.atleast_1d(q))
    out = np.zeros(len(qa), dtype=np.float64)
    _check(lib().mllm_interp(C.byref(c), len(qa), qp, int(bool(extrapolate)), out.ctypes.data_as(C.POINTER(C.c_double))))
    return out


def mllm_item_durations(b, s, e_flop, l_lin_flop, l_attn_flop, e_thr, l_lin_thr, l_attn_thr):
    """(e_dur, l_dur) per item from the three profiled throughput curves, each given as (x, y)."""
    arrs = [_dvec(a) for a in (b, s, e_flop, l_lin_flop, l_attn_flop)]
    n = len(arrs[0][0])
    if any(len(a) != n for a, _ in arrs):
        raise ValueError("item arrays differ in length")
    curves = [_curve(c) for c in (e_thr, l_lin_thr, l_attn_thr)]
    e_dur, l_dur = np.zeros(n), np.zeros(n)
    _check(lib().mllm_item_durations(n, *[p for _, p in arrs], *[C.byref(c) for c, _ in curves],
                                     e_dur.ctypes.data_as(C.POINTER(C.c_double)),
                                     l_dur.ctypes.data_as(C.POINTER(C.c_double))))
    return e_dur, l_dur


def mllm_find_combs(gpus: int, n_gpu_node: int, max_pp: int) -> np.ndarray:
    """All (tp, pp, dp) with product `gpus`, as an [n, 3] int32 array."""
    count = C.c_int64()
    _check(lib().mllm_find_combs(gpus, n_gpu_node, max_pp, 0, None, C.byref(count)))
    out = np.zeros((count.value, 3), dtype=np.int32)
    _check(lib().mllm_find_combs(gpus, n_gpu_node, max_pp, count.value,
                                 out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(count)))
    return out


def _module_profile(prof: dict):
    """dict with tp, x, thr [n_tp][n_x], layers_lo, layers_hi, model_state [n_tp][2],
    act_state [n_tp][2][n_x], n_layers, flop_per_item -> ModuleProfileC plus its arrays."""
    tp = np.ascontiguousarray(prof["tp"], dtype=np.int32)
    x, xp = _dvec(prof["x"])
    thr, tp_ = _dvec(prof["thr"])
    ms, msp = _dvec(prof["model_state"])
    act, actp = _dvec(prof["act_state"])
    if thr.shape != (len(tp), len(x)) or ms.shape != (len(tp), 2) or act.shape != (len(tp), 2, len(x)):
        raise ValueError("module profile tables have the wrong shape")
    c = ModuleProfileC(len(tp), tp.ctypes.data_as(C.POINTER(C.c_int32)), len(x), xp, tp_,
                       float(prof["layers_lo"]), float(prof["layers_hi"]), msp, actp,
                       int(prof["n_layers"]), float(prof["flop_per_item"]))
    return c, (tp, x, thr, ms, act)


def mllm_evaluate_parallelism(enc: dict, llm: dict, theta, m_gpu: float, gbs: int, mean_bsz: float,
                              mean_seq_len: float):
    """(makespan, encoder memory, LLM memory, feasible) of one configuration theta."""
    e, keep_e = _module_profile(enc)
    l, keep_l = _module_profile(llm)
    th = (C.c_int32 * 7)(*[int(v) for v in theta])
    t, em, lm, ok = C.c_double(), C.c_double(), C.c_double(), C.c_int32()
    _check(lib().mllm_evaluate_parallelism(C.byref(e), C.byref(l), th, m_gpu, gbs, mean_bsz, mean_seq_len,
                                           C.byref(t), C.byref(em), C.byref(lm), C.byref(ok)))
    return t.value, em.value, lm.value, bool(ok.value)


def mllm_optimize_parallelism(enc: dict, llm: dict, n_gpus: int, n_gpu_node: int, m_gpu: float, gbs: int,
                              mean_bsz: float, mean_seq_len: float):
    """(theta*, min_T) or (None, inf); theta* = (E_tp, E_pp, E_dp, L_tp, L_pp, L_dp, N_mb)."""
    e, keep_e = _module_profile(enc)
    l, keep_l = _module_profile(llm)
    th = (C.c_int32 * 7)()
    t, found = C.c_double(), C.c_int32()
    _check(lib().mllm_optimize_parallelism(C.byref(e), C.byref(l), n_gpus, n_gpu_node, m_gpu, gbs, mean_bsz,
                                           mean_seq_len, th, C.byref(t), C.byref(found)))
    return (tuple(int(v) for v in th) if found.value else None), t.value
