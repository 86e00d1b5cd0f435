"""Thin ctypes binding of libmquant.so: argument marshalling only.

Every function has the name of the C entry point it calls (without the
``mquant_`` prefix) and does no arithmetic of the method: tensors are handed
over as device pointers, the stream is torch's current HIP stream.  PyTorch is
used for device memory and streams only.  There is no CPU fallback: if the HIP
library is missing or cannot be loaded the import of this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np
# torch before libmquant.so: the ROCm wheel of torch carries its own HIP runtime under the
# same soname.  Loaded second, libmquant binds to that copy and shares torch's streams and
# memory; loaded first, it would pull in the system runtime as a second one in the process,
# and a second runtime may find no device to open.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libmquant.so")

EXPORTS = (
    "mquant_version", "mquant_status_string", "mquant_aifs_build_perm", "mquant_aifs_permute",
    "mquant_aifs_remap_mask", "mquant_hadamard_quant_act", "mquant_hadamard_absmax",
    "mquant_w4_prepacked_bytes", "mquant_w4_prepack", "mquant_w4a8_workspace_bytes",
    "mquant_w4a8_gemm", "mquant_w4a8_linear_prefill_workspace_bytes", "mquant_w4a8_linear_prefill",
    "mquant_hadamard_dynquant_act", "mquant_w4a8_gemm_rowscale", "mquant_w4a8_gemm_rms",
    "mquant_rope_apply", "mquant_aifs_attention_workspace_bytes", "mquant_aifs_attention",
    "mquant_hadamard_quant_act_bits", "mquant_static_scale_from_absmax", "mquant_tune_set",
    "mquant_build_id",
    "mquant_w4a8_linear_decode", "mquant_w4a8_linear_prefill_static", "mquant_w4a8_gemv_grouped",
    "mquant_w4a8_linear_decode_grouped",
    "mquant_w4g128_prepacked_bytes", "mquant_w4g128_prepack", "mquant_w4g128_gemm",
)

OK, ERR_NULL, ERR_BAD_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_ALIGNMENT = 0, -1, -2, -3, -4, -5, -6


class MQuantError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class Span(ctypes.Structure):
    _fields_ = [("start", ctypes.c_int32), ("len", ctypes.c_int32)]


class Linear(ctypes.Structure):
    _fields_ = [("w_prepacked_dev", ctypes.c_void_p), ("w_scale_dev", ctypes.c_void_p),
                ("y_dev", ctypes.c_void_p), ("ldy", ctypes.c_int64), ("N", ctypes.c_int32)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2502_00425_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i32, i64, f32, p = ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p
    lib.mquant_version.restype = ctypes.c_int
    lib.mquant_status_string.restype = ctypes.c_char_p
    lib.mquant_status_string.argtypes = [ctypes.c_int]
    lib.mquant_build_id.restype = ctypes.c_char_p
    lib.mquant_build_id.argtypes = []
    lib.mquant_static_scale_from_absmax.argtypes = [f32, i32, i32, p]
    lib.mquant_tune_set.argtypes = [i32, i32]
    lib.mquant_aifs_build_perm.argtypes = [i32, p, i32, p, p, p]
    lib.mquant_aifs_permute.argtypes = [p, i64, p, i64, p, i32, i32, p]
    lib.mquant_aifs_remap_mask.argtypes = [p, p, p, i32, p]
    lib.mquant_hadamard_quant_act.argtypes = [p, i64, p, p, i32, i32, i32, f32, f32, i32, p]
    lib.mquant_hadamard_absmax.argtypes = [p, i64, i32, i32, i32, p, p]
    lib.mquant_hadamard_quant_act_bits.argtypes = [p, i64, p, p, i32, i32, i32, f32, f32, i32, i32, p]
    lib.mquant_hadamard_dynquant_act.argtypes = [p, i64, p, p, p, i32, i32, i32, p]
    lib.mquant_w4a8_gemm_rowscale.argtypes = [p, p, p, p, p, i64, p, i32, i32, i32, p, i64, p]
    lib.mquant_w4a8_gemm_rms.argtypes = [p, p, p, p, i64, p, i32, i32, i32, i32, f32, f32, p, p, p, i32,
                                         p, i64, p]
    lib.mquant_w4_prepacked_bytes.restype = i64
    lib.mquant_w4_prepacked_bytes.argtypes = [i32, i32]
    lib.mquant_w4_prepack.argtypes = [p, p, i32, i32, p]
    lib.mquant_w4a8_workspace_bytes.restype = i64
    lib.mquant_w4a8_workspace_bytes.argtypes = [i32, i32, i32]
    lib.mquant_w4a8_gemm.argtypes = [p, p, p, p, i64, p, i32, i32, i32, i32, f32, f32, p, i64, p]
    lib.mquant_w4a8_linear_prefill_workspace_bytes.restype = i64
    lib.mquant_w4a8_linear_prefill_workspace_bytes.argtypes = [i32, i32, i32]
    lib.mquant_w4a8_linear_prefill.argtypes = [p, i64, p, p, p, p, i64, i32, i32, i32, i32, f32, f32,
                                               i32, p, i64, p]
    lib.mquant_w4a8_linear_prefill_static.argtypes = [p, i64, p, p, p, p, i64, i32, i32, i32, i32, f32, f32,
                                                      i32, p]
    lib.mquant_w4a8_gemv_grouped.argtypes = [p, i32, i32, i32, f32, f32, p, i32, p]
    lib.mquant_w4a8_linear_decode_grouped.argtypes = [p, i64, i32, i32, i32, f32, f32, i32, p, i32, p]
    lib.mquant_rope_apply.argtypes = [p, i64, p, i32, i32, i32, ctypes.c_double, p]
    lib.mquant_aifs_attention_workspace_bytes.restype = i64
    lib.mquant_aifs_attention_workspace_bytes.argtypes = [i32, i32, i32]
    lib.mquant_aifs_attention.argtypes = [p, i64, p, i64, p, i64, p, i64, p, i32, i32, i32, i32, p, i64, p]
    lib.mquant_w4a8_linear_decode.argtypes = [p, i64, p, p, p, i64, i32, i32, i32, i32, f32, f32, i32, p]
    lib.mquant_w4g128_prepacked_bytes.restype = i64
    lib.mquant_w4g128_prepacked_bytes.argtypes = [i32, i32]
    lib.mquant_w4g128_prepack.argtypes = [p, p, p, i32, i32, p]
    lib.mquant_w4g128_gemm.argtypes = [p, i64, p, p, i64, i32, i32, i32, p]
    for name in EXPORTS:
        if name not in ("mquant_status_string", "mquant_w4_prepacked_bytes", "mquant_aifs_attention_workspace_bytes",
                        "mquant_build_id", "mquant_w4g128_prepacked_bytes",
                        "mquant_w4a8_workspace_bytes", "mquant_w4a8_linear_prefill_workspace_bytes",
                        "mquant_version"):
            getattr(lib, name).restype = ctypes.c_int
    return lib


lib = _load()


def status_string(status: int) -> str:
    return lib.mquant_status_string(int(status)).decode()


def version() -> int:
    return int(lib.mquant_version())


def build_id() -> str:
    return lib.mquant_build_id().decode()


TUNE_GEMM_TILE, TUNE_GEMM_NOSPLIT, TUNE_G128_TILE, TUNE_GEMV_VARIANT = 0, 1, 2, 3


def tune_set(key: int, value: int) -> None:
    _check(lib.mquant_tune_set(int(key), int(value)), "mquant_tune_set")


def static_scale_from_absmax(absmax_u: float, had_block: int, act_bits: int = 8) -> float:
    """Eq. (2)'s static scale from the statistic of ``hadamard_absmax`` (computed by the library)."""
    out = ctypes.c_float(0.0)
    _check(lib.mquant_static_scale_from_absmax(float(absmax_u), int(had_block), int(act_bits),
                                               ctypes.cast(ctypes.byref(out), ctypes.c_void_p)),
           "mquant_static_scale_from_absmax")
    return float(out.value)


def _check(status: int, where: str) -> None:
    if status != OK:
        raise MQuantError(int(status), where)


def _dp(t) -> Optional[int]:
    """Device (or host) address of a torch tensor; None stays NULL."""
    return None if t is None else t.data_ptr()


def _rows(t, what: str) -> None:
    """A 2-D operand the ABI addresses through a leading dimension: unit stride along a row."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1) or (t.shape[0] > 1 and t.stride(0) < t.shape[1]):
        raise MQuantError(ERR_BAD_SHAPE, f"{what}: expected a 2-D tensor with unit column stride")


def _dense(t, what: str) -> None:
    """An operand the ABI takes without a leading dimension."""
    if t is not None and not t.is_contiguous():
        raise MQuantError(ERR_BAD_SHAPE, f"{what}: expected a contiguous tensor")


def _stream() -> Optional[int]:
    import torch
    return torch.cuda.current_stream().cuda_stream or None


# ------------------------------------------------------------------- host

def aifs_build_perm(T: int, vis_spans: Sequence[Tuple[int, int]]):
    """-> (perm int32[T], inv_perm int32[T], n_vis) as numpy arrays (host)."""
    n = len(vis_spans)
    arr = (Span * max(n, 1))()
    for i, (s, l) in enumerate(vis_spans):
        arr[i].start, arr[i].len = int(s), int(l)
    perm = np.empty(max(T, 0), dtype=np.int32)
    inv = np.empty(max(T, 0), dtype=np.int32)
    n_vis = ctypes.c_int32(0)
    st = lib.mquant_aifs_build_perm(T, ctypes.cast(arr, ctypes.c_void_p) if n else None, n,
                                    perm.ctypes.data, inv.ctypes.data,
                                    ctypes.cast(ctypes.byref(n_vis), ctypes.c_void_p))
    _check(st, "mquant_aifs_build_perm")
    return perm, inv, int(n_vis.value)


# ----------------------------------------------------------------- device

def aifs_permute(x, perm_dev, out=None):
    import torch
    T, K = x.shape
    if out is None:
        out = torch.empty((T, K), dtype=x.dtype, device=x.device)
    _rows(x, "aifs_permute x"), _rows(out, "aifs_permute out"), _dense(perm_dev, "perm")
    _check(lib.mquant_aifs_permute(_dp(x), x.stride(0), _dp(out), out.stride(0), _dp(perm_dev),
                                   T, K, _stream()), "mquant_aifs_permute")
    return out


def aifs_remap_mask(mask, perm_dev, out=None):
    import torch
    T = mask.shape[0]
    if out is None:
        out = torch.empty((T, T), dtype=torch.uint8, device=mask.device)
    _dense(mask, "mask"), _dense(out, "mask_u"), _dense(perm_dev, "perm")
    _check(lib.mquant_aifs_remap_mask(_dp(mask), _dp(out), _dp(perm_dev), T, _stream()),
           "mquant_aifs_remap_mask")
    return out


def hadamard_quant_act(x, n_vis: int, s_vis: float, s_txt: float, had_block: int,
                       perm_dev=None, out=None, T: Optional[int] = None, act_bits: Optional[int] = None):
    import torch
    rows, K = x.shape
    T = rows if T is None else T
    if out is None:
        out = torch.empty((T, K), dtype=torch.int8, device=x.device)
    _rows(x, "hadamard_quant_act x"), _dense(out, "xq"), _dense(perm_dev, "perm")
    if act_bits is None:
        _check(lib.mquant_hadamard_quant_act(_dp(x), x.stride(0), _dp(perm_dev), _dp(out), T, K, n_vis,
                                             s_vis, s_txt, had_block, _stream()),
               "mquant_hadamard_quant_act")
    else:
        _check(lib.mquant_hadamard_quant_act_bits(_dp(x), x.stride(0), _dp(perm_dev), _dp(out), T, K,
                                                  n_vis, s_vis, s_txt, had_block, act_bits, _stream()),
               "mquant_hadamard_quant_act_bits")
    return out


def hadamard_absmax(x, had_block: int, absmax_dev):
    T, K = x.shape
    _rows(x, "hadamard_absmax x")
    _check(lib.mquant_hadamard_absmax(_dp(x), x.stride(0), T, K, had_block, _dp(absmax_dev),
                                      _stream()), "mquant_hadamard_absmax")
    return absmax_dev


def w4_prepacked_bytes(N: int, K: int) -> int:
    n = int(lib.mquant_w4_prepacked_bytes(N, K))
    if n < 0:
        raise MQuantError(n, "mquant_w4_prepacked_bytes")
    return n


def w4_prepack(w_canonical, out=None):
    import torch
    N, K2 = w_canonical.shape
    K = 2 * K2
    if out is None:
        out = torch.empty(w4_prepacked_bytes(N, K), dtype=torch.uint8, device=w_canonical.device)
    _dense(w_canonical, "w_canonical"), _dense(out, "w_prepacked")
    _check(lib.mquant_w4_prepack(_dp(w_canonical), _dp(out), N, K, _stream()), "mquant_w4_prepack")
    return out


def w4a8_workspace_bytes(T: int, N: int, K: int) -> int:
    n = int(lib.mquant_w4a8_workspace_bytes(T, N, K))
    if n < 0:
        raise MQuantError(n, "mquant_w4a8_workspace_bytes")
    return n


def w4a8_gemm(xq, w_prepacked, w_scale, N: int, n_vis: int, s_vis: float, s_txt: float,
              out=None, acc_out=None, workspace=None):
    import torch
    T, K = xq.shape
    if out is None:
        out = torch.empty((T, N), dtype=torch.float16, device=xq.device)
    if workspace is None:
        need = w4a8_workspace_bytes(T, N, K)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=xq.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _dense(xq, "xq"), _rows(out, "y"), _dense(acc_out, "acc_out"), _dense(w_scale, "w_scale")
    _check(lib.mquant_w4a8_gemm(_dp(xq), _dp(w_prepacked), _dp(w_scale), _dp(out), out.stride(0),
                                _dp(acc_out), T, N, K, n_vis, s_vis, s_txt, _dp(workspace),
                                ws_bytes, _stream()), "mquant_w4a8_gemm")
    return out


def hadamard_dynquant_act(x, had_block: int, perm_dev=None, out=None, row_scale=None):
    import torch
    T, K = x.shape
    if out is None:
        out = torch.empty((T, K), dtype=torch.int8, device=x.device)
    if row_scale is None:
        row_scale = torch.empty((T,), dtype=torch.float32, device=x.device)
    _rows(x, "x"), _dense(out, "xq"), _dense(row_scale, "row_scale"), _dense(perm_dev, "perm")
    _check(lib.mquant_hadamard_dynquant_act(_dp(x), x.stride(0), _dp(perm_dev), _dp(out),
                                            _dp(row_scale), T, K, had_block, _stream()),
           "mquant_hadamard_dynquant_act")
    return out, row_scale


def w4a8_gemm_rowscale(xq, w_prepacked, w_scale, row_scale, N: int, out=None, acc_out=None,
                       workspace=None):
    import torch
    T, K = xq.shape
    if out is None:
        out = torch.empty((T, N), dtype=torch.float16, device=xq.device)
    if workspace is None:
        need = w4a8_workspace_bytes(T, N, K)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=xq.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _dense(xq, "xq"), _rows(out, "y"), _dense(acc_out, "acc_out"), _dense(row_scale, "row_scale")
    _check(lib.mquant_w4a8_gemm_rowscale(_dp(xq), _dp(w_prepacked), _dp(w_scale), _dp(row_scale),
                                         _dp(out), out.stride(0), _dp(acc_out), T, N, K,
                                         _dp(workspace), ws_bytes, _stream()),
           "mquant_w4a8_gemm_rowscale")
    return out


def w4a8_gemm_rms(xq, w_prepacked, w_scale, N: int, n_vis: int, s_vis: float, s_txt: float,
                  split_idx, split_w, split_scale, out=None, acc_out=None, workspace=None):
    """split_idx (int32) and split_scale (fp32) are HOST arrays (per-layer constants),
    split_w is a device tensor int8 [n_split, N]."""
    import torch
    T, K = xq.shape
    if split_idx is None:
        n_split, idx_p, sc_p = 0, None, None
    else:
        idx = np.ascontiguousarray(split_idx, dtype=np.int32)
        sc = np.ascontiguousarray(split_scale, dtype=np.float32)
        n_split = int(idx.shape[0])
        idx_p, sc_p = idx.ctypes.data_as(ctypes.c_void_p), sc.ctypes.data_as(ctypes.c_void_p)
    if out is None:
        out = torch.empty((T, N), dtype=torch.float16, device=xq.device)
    if workspace is None:
        need = w4a8_workspace_bytes(T, N, K)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=xq.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _dense(xq, "xq"), _rows(out, "y"), _dense(acc_out, "acc_out"), _dense(split_w, "split_w")
    _check(lib.mquant_w4a8_gemm_rms(_dp(xq), _dp(w_prepacked), _dp(w_scale), _dp(out), out.stride(0),
                                    _dp(acc_out), T, N, K, n_vis, s_vis, s_txt, idx_p,
                                    _dp(split_w), sc_p, n_split, _dp(workspace),
                                    ws_bytes, _stream()), "mquant_w4a8_gemm_rms")
    return out


def w4a8_linear_prefill_workspace_bytes(T: int, N: int, K: int) -> int:
    n = int(lib.mquant_w4a8_linear_prefill_workspace_bytes(T, N, K))
    if n < 0:
        raise MQuantError(n, "mquant_w4a8_linear_prefill_workspace_bytes")
    return n


def w4a8_linear_prefill(x, perm_dev, w_prepacked, w_scale, N: int, n_vis: int, s_vis: float,
                        s_txt: float, had_block: int, workspace, out=None):
    import torch
    T, K = x.shape
    if out is None:
        out = torch.empty((T, N), dtype=torch.float16, device=x.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _rows(x, "x"), _rows(out, "y"), _dense(perm_dev, "perm"), _dense(w_scale, "w_scale")
    _check(lib.mquant_w4a8_linear_prefill(_dp(x), x.stride(0), _dp(perm_dev), _dp(w_prepacked),
                                          _dp(w_scale), _dp(out), out.stride(0), T, N, K, n_vis,
                                          s_vis, s_txt, had_block, _dp(workspace), ws_bytes,
                                          _stream()), "mquant_w4a8_linear_prefill")
    return out


def w4a8_gemv_grouped(xq, linears, n_vis: int, s_vis: float, s_txt: float):
    """linears: sequence of (w_prepacked, w_scale, N, out) sharing the input xq [T, K];
    one launch computes every out [T, N]."""
    T, K = xq.shape
    _dense(xq, "xq")
    arr = (Linear * max(len(linears), 1))()
    for i, (wp, ws, N, out) in enumerate(linears):
        _rows(out, "y"), _dense(ws, "w_scale")
        arr[i].w_prepacked_dev, arr[i].w_scale_dev, arr[i].y_dev = _dp(wp), _dp(ws), _dp(out)
        arr[i].ldy, arr[i].N = out.stride(0), N
    _check(lib.mquant_w4a8_gemv_grouped(_dp(xq), T, K, n_vis, s_vis, s_txt,
                                        ctypes.cast(arr, ctypes.c_void_p), len(linears), _stream()),
           "mquant_w4a8_gemv_grouped")
    return [l[3] for l in linears]


STATIC_SCRATCH_BYTES = 128 << 20


def w4a8_linear_prefill_static(x, perm_dev, w_prepacked, w_scale, N: int, n_vis: int, s_vis: float,
                               s_txt: float, had_block: int, out):
    """The fused prefill entry on the library's own scratch array; `out` is required (the
    point of the entry is that nothing gets allocated)."""
    T, K = x.shape
    _rows(x, "x"), _rows(out, "y"), _dense(perm_dev, "perm"), _dense(w_scale, "w_scale")
    _check(lib.mquant_w4a8_linear_prefill_static(_dp(x), x.stride(0), _dp(perm_dev), _dp(w_prepacked),
                                                 _dp(w_scale), _dp(out), out.stride(0), T, N, K, n_vis,
                                                 s_vis, s_txt, had_block, _stream()),
           "mquant_w4a8_linear_prefill_static")
    return out


def rope_apply(x, pos_dev, n_heads: int, head_dim: int = 128, base: float = 10000.0):
    """In place on x [T, >= n_heads*head_dim] fp16."""
    T = x.shape[0]
    _check(lib.mquant_rope_apply(_dp(x), x.stride(0), _dp(pos_dev), T, n_heads, head_dim,
                                 float(base), _stream()), "mquant_rope_apply")
    return x


def aifs_attention_workspace_bytes(T: int, n_kv_heads: int, head_dim: int = 128) -> int:
    n = int(lib.mquant_aifs_attention_workspace_bytes(T, n_kv_heads, head_dim))
    if n < 0:
        raise MQuantError(n, "mquant_aifs_attention_workspace_bytes")
    return n


def aifs_attention(q, k, v, pos_dev, n_q_heads: int, n_kv_heads: int, head_dim: int = 128,
                   out=None, workspace=None):
    """q [T, >= Hq*D], k, v [T, >= Hkv*D] fp16 views (row strides are passed on)."""
    import torch
    T = q.shape[0]
    if out is None:
        out = torch.empty((T, n_q_heads * head_dim), dtype=torch.float16, device=q.device)
    if workspace is None:
        workspace = torch.empty(max(aifs_attention_workspace_bytes(T, n_kv_heads, head_dim), 256),
                                dtype=torch.uint8, device=q.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib.mquant_aifs_attention(_dp(q), q.stride(0), _dp(k), k.stride(0), _dp(v), v.stride(0),
                                     _dp(out), out.stride(0), _dp(pos_dev), T, n_q_heads, n_kv_heads,
                                     head_dim, _dp(workspace), ws_bytes, _stream()),
           "mquant_aifs_attention")
    return out


def w4a8_linear_decode(x, w_prepacked, w_scale, N: int, n_vis: int, s_vis: float, s_txt: float,
                       had_block: int, out=None):
    """x fp16 [T <= 4, K] -> y fp16 [T, N]: rotate, quantize, GEMV and dequant in one launch."""
    import torch
    T, K = x.shape
    if out is None:
        out = torch.empty((T, N), dtype=torch.float16, device=x.device)
    _check(lib.mquant_w4a8_linear_decode(_dp(x), x.stride(0), _dp(w_prepacked), _dp(w_scale), _dp(out),
                                         out.stride(0), T, N, K, n_vis, s_vis, s_txt, had_block,
                                         _stream()), "mquant_w4a8_linear_decode")
    return out


def w4a8_linear_decode_grouped(x, linears, n_vis: int, s_vis: float, s_txt: float, had_block: int):
    """x fp16 [T <= 4, K]; linears: sequence of (w_prepacked, w_scale, N, out) sharing x.
    One launch rotates and quantizes x and computes every out [T, N]."""
    T, K = x.shape
    _rows(x, "x")
    arr = (Linear * max(len(linears), 1))()
    for i, (wp, ws, N, out) in enumerate(linears):
        _rows(out, "y"), _dense(ws, "w_scale")
        arr[i].w_prepacked_dev, arr[i].w_scale_dev, arr[i].y_dev = _dp(wp), _dp(ws), _dp(out)
        arr[i].ldy, arr[i].N = out.stride(0), N
    _check(lib.mquant_w4a8_linear_decode_grouped(_dp(x), x.stride(0), T, K, n_vis, s_vis, s_txt, had_block,
                                                 ctypes.cast(arr, ctypes.c_void_p), len(linears),
                                                 _stream()), "mquant_w4a8_linear_decode_grouped")
    return [l[3] for l in linears]


def w4g128_prepacked_bytes(N: int, K: int) -> int:
    n = int(lib.mquant_w4g128_prepacked_bytes(N, K))
    if n < 0:
        raise MQuantError(n, "mquant_w4g128_prepacked_bytes")
    return n


def w4g128_prepack(w_canonical, scales, out=None):
    """w_canonical uint8 [N, K/2], scales fp16 [N, K/128] -> the weight-only kernel's layout."""
    import torch
    N, K2 = w_canonical.shape
    K = 2 * K2
    if out is None:
        out = torch.empty(w4g128_prepacked_bytes(N, K), dtype=torch.uint8, device=w_canonical.device)
    if tuple(scales.shape) != (N, K // 128) or not scales.is_contiguous():
        raise MQuantError(ERR_BAD_SHAPE, "w4g128_prepack: scales must be contiguous [N, K/128]")
    _check(lib.mquant_w4g128_prepack(_dp(w_canonical), _dp(scales), _dp(out), N, K, _stream()),
           "mquant_w4g128_prepack")
    return out


def w4g128_gemm(x, w_prepacked, N: int, out=None):
    """x fp16 [T, K] (row stride in elements) -> y fp16 [T, N] = x W~^T, group-wise dequantised weight."""
    import torch
    T, K = x.shape
    if out is None:
        out = torch.empty((T, N), dtype=torch.float16, device=x.device)
    _check(lib.mquant_w4g128_gemm(_dp(x), x.stride(0) if T > 0 else K, _dp(w_prepacked), _dp(out),
                                  out.stride(0) if T > 0 else N, T, N, K, _stream()), "mquant_w4g128_gemm")
    return out
