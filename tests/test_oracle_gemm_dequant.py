"""Pins for the integer side of the oracle: int4 unpack, exact int32 GEMM,
fp32 dequant with per-channel x per-modality scales, and end-to-end sanity
against the unquantized product (Sec. 4; Eq. (2), Eq. (3))."""
import math
import os

import numpy as np

from oracle import mquant_oracle as orc


def _pack_canonical(wq):
    """Test-side packer (independent of both implementations): even k low nibble."""
    wq = np.asarray(wq, dtype=np.int64)
    lo = wq[:, 0::2] & 0xF
    hi = wq[:, 1::2] & 0xF
    return (lo | (hi << 4)).astype(np.uint8)


def test_unpack_all_256_bytes(golden_dir):
    table = {}
    with open(os.path.join(golden_dir, "int4_nibbles.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            h, v = line.split()
            table[int(h, 16)] = int(v)
    assert len(table) == 16
    packed = np.arange(256, dtype=np.uint8).reshape(2, 128)     # N=2, K=256
    wq = orc.unpack_w4(packed)
    assert wq.shape == (2, 256) and wq.dtype == np.int8
    for n in range(2):
        for j in range(128):
            byte = int(packed[n, j])
            assert wq[n, 2 * j] == table[byte & 0xF]            # even k: low nibble
            assert wq[n, 2 * j + 1] == table[byte >> 4]         # odd k: high nibble


def test_gemm_hand_worked_2x4_4x3(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "gemm_2x4_4x3.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            rows.append([int(t) for t in line.split()])
    X = np.array(rows[0:2], dtype=np.int8)
    W = np.array(rows[2:5], dtype=np.int8)
    want = np.array(rows[5:7], dtype=np.int32)
    assert (orc.gemm_i8_i4_i32(X, W) == want).all()
    # through the canonical packing as well
    assert (orc.gemm_i8_i4_i32(X, orc.unpack_w4(_pack_canonical(W))) == want).all()


def test_gemm_extremes_no_overflow():
    K = 29568
    X = np.full((2, K), -128, dtype=np.int8)
    X[1] = 127
    W = np.full((2, K), -8, dtype=np.int8)
    W[1] = 7
    acc = orc.gemm_i8_i4_i32(X, W)
    assert acc.dtype == np.int32
    assert acc.tolist() == [[K * 1024, -K * 896], [-K * 1016, K * 889]]
    assert K * 1024 == 30277632


def test_gemm_identity_like_weights_copy_codes():
    rng = np.random.default_rng(1)
    K = 64
    X = rng.integers(-128, 128, size=(5, K), dtype=np.int8)
    W = np.eye(K, dtype=np.int8)
    assert (orc.gemm_i8_i4_i32(X, W) == X.astype(np.int32)).all()
    assert (orc.gemm_i8_i4_i32(X, -W[::-1]) == -X[:, ::-1].astype(np.int32)).all()


def test_gemm_matches_library_int64_matmul():
    rng = np.random.default_rng(2)
    for (T, N, K) in [(3, 5, 8), (17, 33, 130), (64, 512, 512)]:
        X = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
        packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
        W = orc.unpack_w4(packed)
        assert W.min() >= -8 and W.max() <= 7
        want = X.astype(np.int64) @ W.astype(np.int64).T
        assert (orc.gemm_i8_i4_i32(X, W).astype(np.int64) == want).all()


def test_dequant_power_of_two_scales_and_span_choice():
    acc = np.array([[3, -5, 0], [3, -5, 0], [1000, 1, -1]], dtype=np.int32)
    w_scale = np.array([0.5, 0.25, 2.0], dtype=np.float16)
    ref, y = orc.dequant(acc, 1, 0.125, 2.0, w_scale)          # row 0 visual, rows 1-2 text
    assert ref.dtype == np.float32 and y.dtype == np.float16
    assert ref[0].tolist() == [3 * 0.125 * 0.5, -5 * 0.125 * 0.25, 0.0]
    assert ref[1].tolist() == [3 * 2.0 * 0.5, -5 * 2.0 * 0.25, 0.0]
    assert ref[2].tolist() == [1000.0, 0.5, -4.0]
    assert (y.astype(np.float32) == ref).all()                   # all exactly representable


def test_dequant_fp16_rounding_is_nearest_even():
    # acc * 2^-11: 2049 -> 1 + 2^-11 is a tie between 1 and 1+2^-10 -> 1 (even);
    # 2051 -> 1 + 3*2^-11 is a tie between 1+2^-10 and 1+2^-9 -> 1+2^-9 (even mantissa)
    acc = np.array([[2049, 2051, 2050]], dtype=np.int32)
    ref, y = orc.dequant(acc, 0, 1.0, 2.0 ** -11, np.ones(3, dtype=np.float16))
    assert y[0, 0] == np.float16(1.0)
    assert y[0, 1] == np.float16(1.0 + 2.0 ** -9)
    assert y[0, 2] == np.float16(1.0 + 2.0 ** -10)


def test_w4a8_linear_tracks_unquantized_product_and_msq_beats_shared_scale():
    """End-to-end sanity (not parity): the quantized path approximates
    (X_u H/sqrt(B)) (W diag(w_scale))^T with error of the order of the
    quantisation noise, and one shared scale inflates the text-row error by
    about s_vis / s_txt -- the paper's Table 8 observation that a single
    per-tensor static scale collapses while MSQ does not."""
    rng = np.random.default_rng(21)
    T, K, N, B = 48, 256, 40, 128
    spans = [(8, 24)]
    is_vis = np.zeros(T, dtype=bool)
    is_vis[8:32] = True
    x = rng.standard_normal((T, K)).astype(np.float32)
    x[is_vis] *= 20.0
    x = x.astype(np.float16)
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    s_vis = orc.calibrate_static_scale(x[is_vis], B)
    s_txt = orc.calibrate_static_scale(x[~is_vis], B)
    assert 10 < float(s_vis) / float(s_txt) < 40
    out = orc.w4a8_linear(x, spans, packed, w_scale, s_vis, s_txt, B)
    V = out["V"]
    assert V == 24

    Hn = np.kron(np.eye(K // B), orc.hadamard_matrix(B)).astype(np.float64) / math.sqrt(B)
    Wd = orc.unpack_w4(packed).astype(np.float64) * w_scale.astype(np.float64).reshape(N, 1)
    exact = (out["x_u"].astype(np.float64) @ Hn) @ Wd.T

    def rel(a, b):
        return np.linalg.norm(a - b) / np.linalg.norm(b)

    e_vis = rel(out["ref"][:V], exact[:V])
    e_txt = rel(out["ref"][V:], exact[V:])
    # noise/signal of a uniform quantizer with step s on data of rms r: s/(sqrt(12) r)
    r_vis = np.sqrt(((out["x_u"][:V].astype(np.float64)) ** 2).mean())
    r_txt = np.sqrt(((out["x_u"][V:].astype(np.float64)) ** 2).mean())
    assert 0.3 < e_vis / (float(s_vis) / math.sqrt(12) / r_vis) < 3.0
    assert 0.3 < e_txt / (float(s_txt) / math.sqrt(12) / r_txt) < 3.0

    shared = orc.w4a8_linear(x, spans, packed, w_scale, s_vis, s_vis, B)
    e_txt_shared = rel(shared["ref"][V:], exact[V:])
    assert e_txt_shared > 5 * e_txt
    assert abs(rel(shared["ref"][:V], exact[:V]) - e_vis) < 1e-12

    # y is the fp16 rounding of ref
    assert (out["y"] == out["ref"].astype(np.float16)).all()
    # sampled rows/cols give the same numbers as the full run
    rows = np.array([0, 5, 23, 24, 47])
    cols = np.array([0, 7, 39])
    sub = orc.w4a8_linear(x, spans, packed, w_scale, s_vis, s_txt, B, rows=rows, cols=cols)
    assert (sub["acc"] == out["acc"][np.ix_(rows, cols)]).all()
    assert (sub["ref"] == out["ref"][np.ix_(rows, cols)]).all()
