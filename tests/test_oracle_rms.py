"""Pins for the Rotation Magnitude Suppression functions of the oracle (Sec. 3.2:
channel-mean outliers in the first row of H W, split / zero-out / add-back;
appendix on weight outliers after the online Hadamard transform)."""
import math
import os

import numpy as np
import pytest

from oracle import mquant_oracle as orc


def _load(path):
    d = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tag, rest = line.split(None, 1)
            d.setdefault(tag, []).append([float(v) for v in rest.split()])
    return {k: np.array(v) for k, v in d.items()}


def test_hand_worked_split(golden_dir):
    g = _load(os.path.join(golden_dir, "rms_split_2x4x2.txt"))
    xq = g["xq"].astype(np.int8)
    wmain = g["wmain"].astype(np.int8)
    acc = orc.gemm_i8_i4_i32(xq, wmain)
    assert (acc == g["acc"].astype(np.int32)).all()
    ref, y = orc.dequant_rms(acc, xq, 1, 0.5, 0.25, g["wscale"][0].astype(np.float16),
                             np.array([0], dtype=np.int32), g["wsplit"].astype(np.int8),
                             g["ssplit"][0].astype(np.float32))
    assert (ref == g["y"].astype(np.float32)).all()
    assert (y == g["y"].astype(np.float16)).all()


def test_first_row_of_rotated_weight_is_sqrt_n_times_column_mean():
    """(H W)_{0j} = sqrt(n) mean(w_:j): the identity the outlier argument rests on."""
    rng = np.random.default_rng(0)
    for B in (4, 64, 512):
        W = rng.standard_normal((2 * B, 5)) + rng.uniform(-1, 1, size=(1, 5))
        R = orc.rotate_weight(W, B)
        for b in range(2):
            blk = W[b * B:(b + 1) * B]
            assert np.allclose(R[b * B], math.sqrt(B) * blk.mean(axis=0), rtol=1e-12, atol=1e-12)
        # orthonormal rotation keeps the Frobenius norm
        assert np.isclose(np.linalg.norm(R), np.linalg.norm(W), rtol=1e-12)


def test_rotation_pair_cancels():
    """(x H)(H^T W) = x W: rotating activations online and weights offline changes nothing."""
    rng = np.random.default_rng(1)
    B, K, N = 16, 64, 7
    x = rng.integers(-8, 9, size=(3, K)).astype(np.float16)
    W = rng.standard_normal((K, N))
    u = orc.hadamard_rotate(x, B).astype(np.float64) / math.sqrt(B)
    assert np.allclose(u @ orc.rotate_weight(W, B), x.astype(np.float64) @ W, rtol=1e-10, atol=1e-10)


def test_flagging_follows_the_mean_condition():
    rng = np.random.default_rng(2)
    B, N = 64, 6
    zero_mean = rng.standard_normal((B, N))
    zero_mean -= zero_mean.mean(axis=0, keepdims=True)
    big_mean = rng.standard_normal((B, N)) * 0.1
    big_mean[:, 2] += 1.0                           # sqrt(64) * 1.0 = 8 > max|w| ~ 1.3
    W = np.vstack([zero_mean, big_mean, zero_mean])
    assert orc.rms_flag_channels(W, B).tolist() == [B]
    assert orc.rms_flag_channels(np.vstack([zero_mean, zero_mean]), B).tolist() == []
    # the boundary: a constant column of value v has sqrt(B) v > v for B > 1, equality never flags
    const = np.ones((B, 1))
    assert orc.rms_flag_channels(const, B).tolist() == [0]
    assert orc.rms_flag_channels(np.ones((1, 1)), 1).tolist() == []


def test_split_plus_main_equals_unsplit_in_integers():
    """With unit scales everything is an integer: zeroing the flagged rows in the main
    matrix and adding the split products back must reproduce the full product exactly
    (nothing dropped, nothing counted twice)."""
    rng = np.random.default_rng(3)
    T, K, N = 9, 96, 11
    xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
    w_full = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    idx = np.array([0, 32, 64], dtype=np.int32)
    w_main = w_full.copy()
    w_main[:, idx] = 0
    wsplit = np.ascontiguousarray(w_full[:, idx].T)
    ones_n, ones_s = np.ones(N, dtype=np.float16), np.ones(3, dtype=np.float32)
    ref, _ = orc.dequant_rms(orc.gemm_i8_i4_i32(xq, w_main), xq, 4, 1.0, 1.0, ones_n, idx, wsplit, ones_s)
    full = orc.gemm_i8_i4_i32(xq, w_full)
    assert (ref == full.astype(np.float32)).all()


def test_no_split_reduces_to_plain_dequant():
    rng = np.random.default_rng(4)
    acc = rng.integers(-10 ** 6, 10 ** 6, size=(5, 8), dtype=np.int32)
    xq = rng.integers(-128, 128, size=(5, 16), dtype=np.int8)
    ws = rng.uniform(0.005, 0.02, size=8).astype(np.float16)
    a, _ = orc.dequant_rms(acc, xq, 2, 0.3, 0.02, ws, np.zeros(0, np.int32), np.zeros((0, 8), np.int8),
                           np.zeros(0, np.float32))
    b, _ = orc.dequant(acc, 2, 0.3, 0.02, ws)
    assert (a == b).all()


def test_split_suppresses_the_weight_scale_and_the_error():
    """What RMS is for: a weight whose columns have a large common mean gets a first-row
    outlier after rotation; taking that row out shrinks the per-channel int4 step of the main
    matrix and the end-to-end error of the quantized linear."""
    rng = np.random.default_rng(5)
    B, K, N, T = 64, 128, 24, 16
    W = rng.standard_normal((K, N)) * 0.05 + rng.uniform(0.3, 0.6, size=(1, N))
    R = orc.rotate_weight(W, B)
    flagged = orc.rms_flag_channels(W, B)
    assert flagged.tolist() == [0, B]
    wq0, s0 = orc.quantize_weight_rows_int4(R.T)
    wq1, s1, wsplit, ssplit = orc.rms_split_weight(R, flagged)
    assert (wq1[:, flagged] == 0).all()
    assert (s1.astype(np.float64) < 0.5 * s0.astype(np.float64)).all()
    x = rng.standard_normal((T, K)).astype(np.float16)
    u = orc.hadamard_rotate(x, B)
    s_act = float(orc.static_scale_from_absmax(np.abs(u).max(), B))
    xq = orc.msq_quantize(u, 0, s_act, s_act, B)
    want = x.astype(np.float64) @ W
    y0, _ = orc.dequant(orc.gemm_i8_i4_i32(xq, wq0), 0, s_act, s_act, s0)
    y1, _ = orc.dequant_rms(orc.gemm_i8_i4_i32(xq, wq1), xq, 0, s_act, s_act, s1, flagged, wsplit, ssplit)
    e0 = np.abs(y0 - want).mean()
    e1 = np.abs(y1 - want).mean()
    assert e1 < 0.6 * e0
