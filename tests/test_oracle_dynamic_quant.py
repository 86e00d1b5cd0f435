"""Pins for the per-token dynamic quantization baseline of the oracle (Sec. 2.2:
the scale of Eq. (2) from runtime statistics; appendix on quantization
granularity: one scale per token; "per token scale" column of the scheme table)."""
import math
import os

import numpy as np
import pytest

from oracle import mquant_oracle as orc


def _load_cases(path):
    cases, cur = [], {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tag, rest = line.split(None, 1)
            cur[tag] = np.array(rest.split(), dtype=np.float64)
            if tag == "q":
                cases.append(cur)
                cur = {}
    return cases


def test_hand_worked_rows(golden_dir):
    cases = _load_cases(os.path.join(golden_dir, "dyn_quant_rows.txt"))
    assert len(cases) == 4
    for c in cases:
        xq, s = orc.dyn_quantize(c["x"].astype(np.float32)[None, :], 1)
        assert s[0] == np.float32(c["s"][0])
        assert (xq[0].astype(np.int64) == c["q"].astype(np.int64)).all()


@pytest.mark.parametrize("B", [1, 16, 128, 512])
def test_largest_element_maps_to_127_and_error_is_at_most_half_a_step(B):
    """By construction of s_i nothing is clipped, so |x_rot - s q| <= s/2 everywhere
    (plus fp32 rounding of the product) and the largest magnitude of every row
    lands on +-127."""
    rng = np.random.default_rng(B)
    T, K = 37, 4 * max(B, 8)
    x = (rng.standard_normal((T, K)) * rng.uniform(0.01, 30.0, size=(T, 1))).astype(np.float16)
    u = orc.hadamard_rotate(x, B)
    xq, s = orc.dyn_quantize(u, B)
    assert (np.abs(xq.astype(np.int64)).max(axis=1) == 127).all()
    xrot = u.astype(np.float64) / math.sqrt(B)
    err = np.abs(xrot - s.astype(np.float64)[:, None] * xq.astype(np.float64))
    assert (err <= 0.5 * s.astype(np.float64)[:, None] * (1 + 1e-5) + 1e-12).all()
    want_s = np.abs(xrot).max(axis=1) / 127.0
    assert np.allclose(s, want_s, rtol=2e-7, atol=0)


def test_power_of_two_row_scaling_changes_only_the_scale():
    rng = np.random.default_rng(7)
    u = rng.standard_normal((5, 256)).astype(np.float32)
    f = np.array([1.0, 2.0, 0.5, 1024.0, 2.0 ** -10], dtype=np.float32)[:, None]
    q0, s0 = orc.dyn_quantize(u, 64)
    q1, s1 = orc.dyn_quantize(u * f, 64)
    assert (q0 == q1).all()
    assert (s1 == s0 * f[:, 0]).all()


def test_rows_are_independent_and_zero_row_gets_unit_scale():
    rng = np.random.default_rng(8)
    u = rng.standard_normal((6, 128)).astype(np.float32) * 50
    u[3] = 0.0
    q, s = orc.dyn_quantize(u, 128)
    assert s[3] == 1.0 and (q[3] == 0).all()
    for i in (0, 5):
        qi, si = orc.dyn_quantize(u[i:i + 1], 128)
        assert si[0] == s[i] and (qi[0] == q[i]).all()


def test_agrees_with_static_quantizer_given_the_same_scale():
    """A token quantized dynamically equals the static quantizer of Eq. (2)/(3)
    run with that token's own scale for both modalities."""
    rng = np.random.default_rng(9)
    B = 32
    u = (rng.standard_normal((4, 96)) * 17).astype(np.float32)
    q, s = orc.dyn_quantize(u, B)
    for i in range(4):
        qs = orc.msq_quantize(u[i:i + 1], 1, float(s[i]), float(s[i]), B)
        assert (qs[0] == q[i]).all()


def test_dequant_rows_by_hand():
    acc = np.array([[100, -3, 0], [7, 8, -9]], dtype=np.int32)
    s_rows = np.array([0.5, 0.25], dtype=np.float32)
    w_scale = np.array([2.0, 0.125, 1.0], dtype=np.float16)
    ref, y = orc.dequant_rows(acc, s_rows, w_scale)
    want = np.array([[100.0, -0.1875, 0.0], [3.5, 0.25, -2.25]], dtype=np.float32)
    assert (ref == want).all() and (y == want.astype(np.float16)).all()


def test_dequant_rows_reduces_to_two_scale_dequant():
    rng = np.random.default_rng(10)
    acc = rng.integers(-10 ** 6, 10 ** 6, size=(9, 33), dtype=np.int32)
    w_scale = rng.uniform(0.005, 0.02, size=33).astype(np.float16)
    V, sv, st = 4, np.float32(0.37), np.float32(0.011)
    s_rows = np.where(np.arange(9) < V, sv, st).astype(np.float32)
    a, _ = orc.dequant_rows(acc, s_rows, w_scale)
    b, _ = orc.dequant(acc, V, sv, st, w_scale)
    assert (a == b).all()


def test_dynamic_linear_tracks_the_float_product():
    """End to end: with 8-bit tokens and exact int4 weights the dynamic path must
    reproduce x W^T to within the activation rounding error bound
    sum_k |w_nk| s_w s_i / 2 per output."""
    rng = np.random.default_rng(11)
    T, K, N, B = 6, 256, 10, 64
    x = (rng.standard_normal((T, K)) * 3).astype(np.float16)
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    out = orc.w4a8_linear_dynamic(x, packed, w_scale, B)
    wq = orc.unpack_w4(packed).astype(np.float64)
    H = np.kron(np.eye(K // B), orc.hadamard_matrix(B)).astype(np.float64) / math.sqrt(B)
    xrot = x.astype(np.float64) @ H
    want = (xrot @ wq.T) * w_scale.astype(np.float64)[None, :]
    bound = 0.5 * out["s_rows"].astype(np.float64)[:, None] * (np.abs(wq).sum(axis=1) * w_scale.astype(np.float64))[None, :]
    assert (np.abs(out["ref"].astype(np.float64) - want) <= bound * (1 + 1e-4) + 1e-6).all()
