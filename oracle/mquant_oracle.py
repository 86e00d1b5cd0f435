"""CPU oracle for the MQuant W4A8 linear hot path -- TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct implementation of what the hot path computes,
written from the MQuant paper (arXiv 2502.00425).  Index work, masks and the
attention check are numpy; the per-element arithmetic (Hadamard butterflies,
quantizer, int4 unpack, integer GEMM, dequant) is the C file next to this one,
loaded with ctypes.  Nothing here imports, links or shares code with the HIP
library, and the product path never imports this module.

Notation follows the paper: a mixed sequence E of length L (here T rows) with
visual segment(s); s_v / s_t are the static per-tensor scales of visual / text
tokens; E^u is the AIFS order (all visual tokens, then all text tokens); M^u is
the unified causal mask.  0-based half-open spans are used in the API; the one
function that restates Eq. (6) keeps the paper's 1-based m, n.

Pins (tests/test_oracle_*.py) fix every function to something other than
itself: H H^T = B I, closed forms, brute force, hand-computed fixtures under
tests/golden/, the attention-invariance claim of Sec. 3.1.  The paper prints no
numeric worked example, so there is no paper-printed value to reproduce.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import Iterable, Sequence, Tuple

import numpy as np

from . import build as _build

_LIB = None


def _lib() -> ctypes.CDLL:
    global _LIB
    if _LIB is None:
        path = _build.build()
        lib = ctypes.CDLL(path)
        i64, i32, f32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_float
        p = ctypes.c_void_p
        lib.orc_num_threads.restype = ctypes.c_int
        lib.orc_fwht_block_f32.argtypes = [p, i32]
        lib.orc_hadamard_rows_f32.argtypes = [p, i64, i64, i32]
        lib.orc_msq_quantize.argtypes = [p, i64, i64, i64, f32, f32, p]
        lib.orc_msq_quantize_bits.argtypes = [p, i64, i64, i64, f32, f32, i32, p]
        lib.orc_absmax_f32.argtypes = [p, i64]
        lib.orc_absmax_f32.restype = f32
        lib.orc_unpack_w4.argtypes = [p, i64, i64, p]
        lib.orc_gemm_i8_i4_i32.argtypes = [p, p, i64, i64, i64, p]
        lib.orc_dequant_f32.argtypes = [p, i64, i64, i64, f32, f32, p, p]
        lib.orc_dequant_rms_f32.argtypes = [p, p, i64, i64, i64, i64, f32, f32, p, p, p, p, i64, p]
        lib.orc_dyn_quantize.argtypes = [p, i64, i64, ctypes.c_double, p, p]
        lib.orc_dequant_rows_f32.argtypes = [p, i64, i64, p, p, p]
        _LIB = lib
    return _LIB


def num_threads() -> int:
    """Host threads the row-parallel loops of the C part use."""
    return int(_lib().orc_num_threads())


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _c(a: np.ndarray, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


# --------------------------------------------------------------------------
# AIFS: token reorder, unified causal mask (Sec. 3.1, Eq. (5), Eq. (6);
# index form in the appendix on rotary position embedding)
# --------------------------------------------------------------------------

def aifs_build_perm(T: int, vis_spans: Iterable[Tuple[int, int]]):
    """Stable partition of row indices: visual rows first, then text rows.

    ``vis_spans`` are 0-based (start, length) pairs.  Returns (perm, inv_perm,
    V): row i of E^u is row perm[i] of E, V is the number of visual rows.  With
    one span [m, n] this is the index vector (m..n, 1..m-1, n+1..L) the paper
    prints; with several spans each modality keeps its original order, which is
    the natural extension of E^u to "text-image-text-image-..." sequences.
    """
    is_vis = np.zeros(T, dtype=bool)
    for start, length in vis_spans:
        if length < 0 or start < 0 or start + length > T:
            raise ValueError("span outside [0, T)")
        if is_vis[start:start + length].any():
            raise ValueError("overlapping visual spans")
        is_vis[start:start + length] = True
    vis = [i for i in range(T) if is_vis[i]]
    txt = [i for i in range(T) if not is_vis[i]]
    perm = np.array(vis + txt, dtype=np.int32).reshape(T)
    inv = np.empty(T, dtype=np.int32)
    for new, old in enumerate(perm):
        inv[old] = new
    return perm, inv, len(vis)


def aifs_permute_rows(x: np.ndarray, perm: np.ndarray) -> np.ndarray:
    """E^u: row i of the result is row perm[i] of x (a pure copy)."""
    return np.ascontiguousarray(x[np.asarray(perm, dtype=np.int64)])


def causal_mask(T: int) -> np.ndarray:
    """Eq. (5) as a boolean matrix: entry (i, j) is True (value 0, attend)
    iff j <= i, False (value -inf) otherwise."""
    i = np.arange(T).reshape(T, 1)
    j = np.arange(T).reshape(1, T)
    return j <= i


def aifs_remap_mask(mask: np.ndarray, perm: np.ndarray) -> np.ndarray:
    """M^u[i, j] = M[perm[i], perm[j]]: token i of E^u may attend token j of
    E^u exactly when the same two tokens could attend in the original order."""
    p = np.asarray(perm, dtype=np.int64)
    return np.ascontiguousarray(mask[p][:, p])


def unified_mask_eq6(L: int, m: int, n: int) -> np.ndarray:
    """Eq. (6) for one visual segment, in the paper's 1-based m..n notation.

    The printed conditions use (n - m) as the number of visual tokens; the
    segment e^v_m..e^v_n holds n - m + 1 of them, so V = n - m + 1 is used
    where the paper writes (n - m).  The second bound, n, then equals
    V + (m - 1): the end of the moved-forward text e^t_1..e^t_{m-1}.
    Returns a boolean [L, L] matrix (True = 0 = attend) indexed 0-based.
    """
    V = n - m + 1
    out = np.zeros((L, L), dtype=bool)
    for i in range(1, L + 1):
        for j in range(1, L + 1):
            if i <= V:
                ok = (j <= i) or (V < j <= n)
            elif i <= n:
                ok = V < j <= i
            else:
                ok = j <= i
            out[i - 1, j - 1] = ok
    return out


def causal_attention_f64(Q, K, Vv, mask) -> np.ndarray:
    """Single-head softmax(Q K^T / sqrt(D) + M) V in fp64 with a boolean mask
    (Eq. (5)); used only to check the attention-invariance claim of AIFS."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    Vv = np.asarray(Vv, dtype=np.float64)
    D = Q.shape[1]
    s = Q @ K.T / math.sqrt(D)
    s = np.where(mask, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    a = e / e.sum(axis=1, keepdims=True)
    return a @ Vv


def aifs_attention_f64(q, k, v, pos, n_q_heads: int, n_kv_heads: int, rows=None) -> np.ndarray:
    """Multi-head causal attention on AIFS-ordered tokens (Sec. 3.1, Eq. (5)-(6)).

    q is [T, n_q_heads*D], k and v are [T, n_kv_heads*D] (token-major, heads side
    by side; query head h reads key/value head h // (n_q_heads // n_kv_heads)),
    pos[i] is the position token i had in the original sequence (the AIFS index
    vector).  Token i attends token j exactly when pos[j] <= pos[i]: the unified
    mask M^u[i,j] = M[pos[i], pos[j]] of the causal M, which for one visual segment
    is the three-region rule of Eq. (6).  softmax(q k^T / sqrt(D) + M^u) v per head,
    everything in fp64.  `rows` restricts the queries (for spot checks)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    pos = np.asarray(pos, dtype=np.int64)
    T = q.shape[0]
    D = q.shape[1] // n_q_heads
    assert k.shape == (T, n_kv_heads * D) and v.shape == k.shape and n_q_heads % n_kv_heads == 0
    sel = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)
    allowed = pos[None, :] <= pos[sel][:, None]
    out = np.empty((len(sel), n_q_heads * D), dtype=np.float64)
    group = n_q_heads // n_kv_heads
    for h in range(n_q_heads):
        g = h // group
        out[:, h * D:(h + 1) * D] = causal_attention_f64(
            q[sel, h * D:(h + 1) * D], k[:, g * D:(g + 1) * D], v[:, g * D:(g + 1) * D], allowed)
    return out


def rope_inv_freq(D: int, base: float = 10000.0) -> np.ndarray:
    """theta_i = base^(-2(i-1)/D), i = 1..D/2 (appendix "Rotary Position Embedding for AIFS")."""
    return np.asarray([base ** (-2.0 * i / D) for i in range(D // 2)], dtype=np.float64)


def rope_apply_f64(x, pos, n_heads: int, base: float = 10000.0) -> np.ndarray:
    """Rotary position embedding with the reordered position ids (appendix "Rotary
    Position Embedding for AIFS"): for token i at original position p = pos[i],
    every head's channel pair (2j, 2j+1) is rotated by the angle p * theta_j,
        x'[2j]   = x[2j] cos - x[2j+1] sin,   x'[2j+1] = x[2j] sin + x[2j+1] cos
    (the block-diagonal rotation matrix printed there).  x is [T, n_heads*D]; fp64."""
    x = np.asarray(x, dtype=np.float64)
    pos = np.asarray(pos, dtype=np.float64)
    T = x.shape[0]
    D = x.shape[1] // n_heads
    ang = pos[:, None] * rope_inv_freq(D, base)[None, :]          # [T, D/2]
    c, s_ = np.cos(ang), np.sin(ang)
    xr = x.reshape(T, n_heads, D // 2, 2)
    out = np.empty_like(xr)
    out[..., 0] = xr[..., 0] * c[:, None, :] - xr[..., 1] * s_[:, None, :]
    out[..., 1] = xr[..., 0] * s_[:, None, :] + xr[..., 1] * c[:, None, :]
    return out.reshape(T, n_heads * D)


# --------------------------------------------------------------------------
# Online Hadamard rotation (Sec. 3.2; appendix on the Walsh-Hadamard matrix)
# --------------------------------------------------------------------------

def hadamard_matrix(B: int) -> np.ndarray:
    """The +-1 Walsh-Hadamard matrix by the Kronecker recursion
    H_{2^n} = H_2 (x) H_{2^{n-1}} without the 1/sqrt(2) factors (int64)."""
    if B < 1 or (B & (B - 1)) != 0:
        raise ValueError("B must be a power of two")
    H2 = np.array([[1, 1], [1, -1]], dtype=np.int64)
    H = np.array([[1]], dtype=np.int64)
    while H.shape[0] < B:
        H = np.kron(H2, H)
    return H


def fwht_block_f32(v: np.ndarray) -> np.ndarray:
    """v * H_B for one block, fp32 butterflies in stage order h = 1, 2, ..."""
    out = _c(v, np.float32).copy()
    _lib().orc_fwht_block_f32(_ptr(out), out.shape[0])
    return out


def hadamard_rotate(x: np.ndarray, B: int) -> np.ndarray:
    """Unnormalised block-diagonal rotation u = x (I (x) H_B) of a [T, K]
    matrix.  fp16 input is widened to fp32 exactly; the result is fp32.  The
    orthonormal transform of the paper is u / sqrt(B); that factor is folded
    into the quantizer's multiplier."""
    x = np.asarray(x)
    T, K = x.shape
    if K % B != 0:
        raise ValueError("B must divide K")
    u = np.array(x, dtype=np.float32, order="C", copy=True)
    _lib().orc_hadamard_rows_f32(_ptr(u), T, K, B)
    return u


# --------------------------------------------------------------------------
# Quantizer (Eq. (2)) with modality-specific static scales (Eq. (3))
# --------------------------------------------------------------------------

def quant_multiplier(s: float, B: int) -> np.float32:
    """c = fp32(1 / (s sqrt(B))), evaluated in double and rounded once."""
    return np.float32(1.0 / (float(np.float32(s)) * math.sqrt(float(B))))


def msq_quantize(u: np.ndarray, V: int, s_vis: float, s_txt: float, B: int) -> np.ndarray:
    """int8 codes clamp(round_half_even(u / (sqrt(B) s_i)), -128, 127) with
    s_i = s_v for rows below V (visual) and s_t for the rest (text)."""
    u = _c(u, np.float32)
    T, K = u.shape
    xq = np.empty((T, K), dtype=np.int8)
    _lib().orc_msq_quantize(_ptr(u), T, K, V,
                            quant_multiplier(s_vis, B), quant_multiplier(s_txt, B), _ptr(xq))
    return xq


def msq_quantize_bits(u: np.ndarray, V: int, s_vis: float, s_txt: float, B: int, bits: int) -> np.ndarray:
    """msq_quantize at activation bit-width `bits` (Eq. (2) with b = bits; W4A4 is
    bits = 4, codes in [-8, 7]); one int8 per code."""
    if not 2 <= bits <= 8:
        raise ValueError("bits must be in 2..8")
    u = _c(u, np.float32)
    T, K = u.shape
    xq = np.empty((T, K), dtype=np.int8)
    _lib().orc_msq_quantize_bits(_ptr(u), T, K, V, quant_multiplier(s_vis, B),
                                 quant_multiplier(s_txt, B), bits, _ptr(xq))
    return xq


def static_scale_from_absmax_bits(absmax_u: float, B: int, bits: int) -> np.float32:
    """s = max|x_rot| / (2^{b-1} - 1) of Eq. (2) for bit-width b."""
    return np.float32(float(np.float32(absmax_u)) / math.sqrt(float(B)) / float((1 << (bits - 1)) - 1))


def rotated_absmax(x_calib: np.ndarray, B: int) -> np.float32:
    """max |u| over the unnormalised rotation of calibration rows."""
    u = hadamard_rotate(x_calib, B)
    return np.float32(_lib().orc_absmax_f32(_ptr(u), u.size))


def static_scale_from_absmax(absmax_u: float, B: int) -> np.float32:
    """s = max|x_rot| / (2^{b-1} - 1) with b = 8 (Eq. (2)); x_rot = u/sqrt(B)."""
    return np.float32(float(np.float32(absmax_u)) / math.sqrt(float(B)) / 127.0)


def calibrate_static_scale(x_calib: np.ndarray, B: int) -> np.float32:
    """Static per-tensor scale of one modality from its calibration rows."""
    return static_scale_from_absmax(rotated_absmax(x_calib, B), B)


# --------------------------------------------------------------------------
# W4A8 integer GEMM and dequantisation
# --------------------------------------------------------------------------

def unpack_w4(packed: np.ndarray) -> np.ndarray:
    """Canonical [N, K/2] bytes -> int8 [N, K] in [-8, 7] (even k = low nibble,
    two's complement)."""
    packed = _c(packed, np.uint8)
    N, K2 = packed.shape
    wq = np.empty((N, 2 * K2), dtype=np.int8)
    _lib().orc_unpack_w4(_ptr(packed), N, 2 * K2, _ptr(wq))
    return wq


def gemm_i8_i4_i32(xq: np.ndarray, wq: np.ndarray) -> np.ndarray:
    """acc[i, n] = sum_k xq[i, k] wq[n, k], exact int32."""
    xq = _c(xq, np.int8)
    wq = _c(wq, np.int8)
    T, K = xq.shape
    N, K2 = wq.shape
    if K != K2:
        raise ValueError("K mismatch")
    acc = np.empty((T, N), dtype=np.int32)
    _lib().orc_gemm_i8_i4_i32(_ptr(xq), _ptr(wq), T, N, K, _ptr(acc))
    return acc


def dequant(acc: np.ndarray, V: int, s_vis: float, s_txt: float, w_scale: np.ndarray):
    """(fp32 reference, fp16 output): ref = (float(acc) s_i) w_scale[n]."""
    acc = _c(acc, np.int32)
    T, N = acc.shape
    ws = np.asarray(w_scale).astype(np.float32)   # fp16 -> fp32 is exact
    ws = _c(ws, np.float32)
    ref = np.empty((T, N), dtype=np.float32)
    _lib().orc_dequant_f32(_ptr(acc), T, N, V, np.float32(s_vis), np.float32(s_txt),
                           _ptr(ws), _ptr(ref))
    return ref, ref.astype(np.float16)


# ------------------------------------------------ Rotation Magnitude Suppression

def rotate_weight(W: np.ndarray, B: int) -> np.ndarray:
    """H^T W for W [K, N] (input channels down the rows) with the orthonormal
    block-diagonal Hadamard matrix, in float64: the weight the rotated
    activations x H meet, so that (x H)(H^T W) = x W (Sec. 3.2, computational
    invariance; appendix on weight outliers after the online transform)."""
    W = np.asarray(W, dtype=np.float64)
    K, N = W.shape
    if K % B:
        raise ValueError("block size must divide K")
    Hn = hadamard_matrix(B).astype(np.float64) / math.sqrt(float(B))
    out = np.empty_like(W)
    for b in range(K // B):
        out[b * B:(b + 1) * B] = Hn.T @ W[b * B:(b + 1) * B]
    return out


def rms_flag_channels(W: np.ndarray, B: int) -> np.ndarray:
    """Input channels of the rotated weight that carry a channel-mean outlier
    (the condition sqrt(n) mean(w_:j) > max_i w_ij of Sec. 3.2, taken in
    magnitude and per Hadamard block of n = B rows): the first row of block b is
    flagged when for some output column j the block's column mean times sqrt(B)
    exceeds the largest magnitude of that column inside the block.  Returns the
    sorted row indices b*B of the flagged blocks."""
    W = np.asarray(W, dtype=np.float64)
    K, N = W.shape
    flagged = []
    for b in range(K // B):
        blk = W[b * B:(b + 1) * B]
        lhs = math.sqrt(float(B)) * np.abs(blk.mean(axis=0))
        rhs = np.abs(blk).max(axis=0)
        if (lhs > rhs).any():
            flagged.append(b * B)
    return np.asarray(flagged, dtype=np.int32)


def quantize_weight_rows_int4(Wt: np.ndarray):
    """Per-output-channel symmetric int4 (Eq. (2) with b = 4, z = 0, round to
    nearest even): Wt is [N, K]; returns (codes int8 in [-8,7], scale fp16 [N]).
    The scale max|w|/7 is rounded to fp16 first and the codes use that value."""
    Wt = np.asarray(Wt, dtype=np.float64)
    amax = np.abs(Wt).max(axis=1)
    scale = np.where(amax > 0, amax / 7.0, 1.0).astype(np.float16)
    q = np.clip(np.rint(Wt / scale.astype(np.float64)[:, None]), -8, 7).astype(np.int8)
    return q, scale


def rms_split_weight(W_rot: np.ndarray, flagged: np.ndarray):
    """Offline side of RMS for one linear (Sec. 3.2 steps 1-2): the flagged rows
    of the rotated weight [K, N] are taken out and quantized on their own (int4,
    one scale per row), the main matrix keeps zeros there and is quantized per
    output channel.  Returns (wq_main int8 [N,K], w_scale fp16 [N],
    wsplit int8 [S,N], ssplit fp32 [S])."""
    W_rot = np.asarray(W_rot, dtype=np.float64)
    flagged = np.asarray(flagged, dtype=np.int64)
    main = W_rot.copy()
    main[flagged] = 0.0
    wq_main, w_scale = quantize_weight_rows_int4(main.T)
    rows = W_rot[flagged]
    amax = np.abs(rows).max(axis=1) if len(flagged) else np.zeros(0)
    ssplit = np.where(amax > 0, amax / 7.0, 1.0).astype(np.float32)
    wsplit = np.clip(np.rint(rows / ssplit.astype(np.float64)[:, None]), -8, 7).astype(np.int8)
    return wq_main, w_scale, wsplit.reshape(len(flagged), W_rot.shape[1]), ssplit


def dequant_rms(acc: np.ndarray, xq: np.ndarray, V: int, s_vis: float, s_txt: float,
                w_scale: np.ndarray, split_idx: np.ndarray, wsplit: np.ndarray, ssplit: np.ndarray):
    """Main-path dequantisation plus the split GEMV of the flagged channels, added
    before the store (Sec. 3.2 step 3).  (fp32 reference, fp16 output)."""
    acc = _c(acc, np.int32)
    xq = _c(xq, np.int8)
    T, N = acc.shape
    K = xq.shape[1]
    ws = _c(np.asarray(w_scale).astype(np.float32), np.float32)
    idx = _c(split_idx, np.int32)
    S = idx.shape[0]
    wsp = _c(np.asarray(wsplit).reshape(S, N), np.int8)
    ssp = _c(ssplit, np.float32)
    assert xq.shape[0] == T and ssp.shape == (S,)
    assert ((idx >= 0) & (idx < K)).all()
    ref = np.empty((T, N), dtype=np.float32)
    _lib().orc_dequant_rms_f32(_ptr(acc), _ptr(xq), T, N, K, V, np.float32(s_vis), np.float32(s_txt),
                               _ptr(ws), _ptr(idx), _ptr(wsp), _ptr(ssp), S, _ptr(ref))
    return ref, ref.astype(np.float16)


def dyn_quantize(u: np.ndarray, B: int):
    """Per-token dynamic int8 quantization of the unnormalised rotation u
    (Sec. 2.2 "dynamic quantization"; one scale per token as in the appendix on
    granularity): returns (codes int8 [T,K], s fp32 [T]) with
    s_i = fp32(max_k|u_ik| / sqrt(B) / 127); an all-zero row gets s_i = 1."""
    u = _c(u, np.float32)
    T, K = u.shape
    xq = np.empty((T, K), dtype=np.int8)
    s_rows = np.empty(T, dtype=np.float32)
    _lib().orc_dyn_quantize(_ptr(u), T, K, math.sqrt(float(B)), _ptr(xq), _ptr(s_rows))
    return xq, s_rows


def dequant_rows(acc: np.ndarray, s_rows: np.ndarray, w_scale: np.ndarray):
    """(fp32 reference, fp16 output): ref = (float(acc) s_i) w_scale[n], s_i per token."""
    acc = _c(acc, np.int32)
    T, N = acc.shape
    ws = _c(np.asarray(w_scale).astype(np.float32), np.float32)
    sr = _c(s_rows, np.float32)
    assert sr.shape == (T,)
    ref = np.empty((T, N), dtype=np.float32)
    _lib().orc_dequant_rows_f32(_ptr(acc), T, N, _ptr(sr), _ptr(ws), _ptr(ref))
    return ref, ref.astype(np.float16)


def w4a8_linear_dynamic(x_u: np.ndarray, w_packed: np.ndarray, w_scale: np.ndarray, B: int,
                        rows=None, cols=None) -> dict:
    """The per-token dynamic baseline on one linear: rotate, per-row scale and
    codes, integer GEMM, per-row dequant.  x_u is fp16 [T, K] (row order is
    irrelevant to this scheme: every row carries its own scale)."""
    u = hadamard_rotate(x_u, B)
    xq, s_rows = dyn_quantize(u, B)
    xs, sr = (xq, s_rows) if rows is None else (xq[np.asarray(rows)], s_rows[np.asarray(rows)])
    wp = w_packed if cols is None else w_packed[np.asarray(cols)]
    ws = w_scale if cols is None else np.asarray(w_scale)[np.asarray(cols)]
    acc = gemm_i8_i4_i32(xs, unpack_w4(wp))
    ref, y = dequant_rows(acc, sr, ws)
    return {"xq": xq, "s_rows": s_rows, "acc": acc, "ref": ref, "y": y}


# --------------------------------------------------------------------------
# Weight-only setting (Table 13: W4 with a group size of 128, activations kept in
# the 16-bit type; group-wise weight granularity of the appendix on quantization
# granularity).  The weight is dequantised to the 16-bit type and the GEMM runs in
# it (the "dequant W" pipeline that Table 3 lists for weight-only methods); fp16 is the 16-bit type of this path.

def quantize_weight_groups_int4(Wt: np.ndarray, group: int = 128):
    """Group-wise symmetric int4 (Eq. (2), b = 4, z = 0, round to nearest even):
    Wt is [N, K]; every run of `group` input channels of an output channel has its
    own scale max|w|/7, rounded to fp16 before the codes are taken (all-zero group:
    scale 1).  Returns (codes int8 [N, K] in [-8, 7], scales fp16 [N, K/group])."""
    Wt = np.asarray(Wt, dtype=np.float64)
    N, K = Wt.shape
    assert K % group == 0
    Wg = Wt.reshape(N, K // group, group)
    amax = np.abs(Wg).max(axis=2)
    scale = np.where(amax > 0, amax / 7.0, 1.0).astype(np.float16)
    q = np.clip(np.rint(Wg / scale.astype(np.float64)[:, :, None]), -8, 7).astype(np.int8)
    return q.reshape(N, K), scale


def dequant_weight_groups_f16(wq: np.ndarray, scales: np.ndarray, group: int = 128) -> np.ndarray:
    """fp16 weight W~[n, k] = fp16(wq[n, k] * scales[n, k // group]): the product of
    an int4 code and an fp16 scale is exact in double; one rounding to fp16."""
    wq = np.asarray(wq)
    N, K = wq.shape
    sc = np.asarray(scales)
    assert sc.dtype == np.float16 and sc.shape == (N, K // group)
    prod = wq.astype(np.float64) * np.repeat(sc.astype(np.float64), group, axis=1)
    return prod.astype(np.float16)


def w4g128_linear(x: np.ndarray, wq: np.ndarray, scales: np.ndarray, group: int = 128):
    """y = x W~^T with fp16 x [T, K] and the dequantised fp16 weight, summed in
    double.  Returns (ref fp64 [T, N], mag fp64 [T, N]) where mag = sum_k |x_k W~_nk|
    is the magnitude a floating-point accumulation error is measured against."""
    x = np.asarray(x)
    assert x.dtype == np.float16
    Wd = dequant_weight_groups_f16(wq, scales, group).astype(np.float64)
    xd = x.astype(np.float64)
    return xd @ Wd.T, np.abs(xd) @ np.abs(Wd).T


def w4a8_linear(x: np.ndarray, vis_spans: Sequence[Tuple[int, int]], w_packed: np.ndarray,
                w_scale: np.ndarray, s_vis: float, s_txt: float, B: int,
                rows=None, cols=None) -> dict:
    """The whole path on one linear, every intermediate kept.

    x is fp16 [T, K] in ORIGINAL token order.  ``rows`` / ``cols`` (index
    arrays into the AIFS-ordered rows and the output channels) restrict the
    GEMM and dequant to a sub-matrix so large shapes can be spot-checked; the
    permutation, rotation and quantization always cover every row.
    """
    T, K = x.shape
    perm, inv, V = aifs_build_perm(T, vis_spans)
    x_u = aifs_permute_rows(x, perm)
    u = hadamard_rotate(x_u, B)
    xq = msq_quantize(u, V, s_vis, s_txt, B)
    out = {"perm": perm, "inv_perm": inv, "V": V, "x_u": x_u, "xq": xq}
    xs = xq if rows is None else xq[np.asarray(rows)]
    wp = w_packed if cols is None else w_packed[np.asarray(cols)]
    ws = w_scale if cols is None else np.asarray(w_scale)[np.asarray(cols)]
    acc = gemm_i8_i4_i32(xs, unpack_w4(wp))
    if rows is None:
        ref, y = dequant(acc, V, s_vis, s_txt, ws)
    else:
        # per-row scale choice must follow the AIFS row index, not the position
        # inside the sample: dequantise visual and text samples separately.
        r = np.asarray(rows)
        ref = np.empty(acc.shape, dtype=np.float32)
        isv = r < V
        if isv.any():
            ref[isv], _ = dequant(acc[isv], int(isv.sum()), s_vis, s_txt, ws)
        if (~isv).any():
            ref[~isv], _ = dequant(acc[~isv], 0, s_vis, s_txt, ws)
        y = ref.astype(np.float16)
    out.update({"acc": acc, "ref": ref, "y": y})
    return out
