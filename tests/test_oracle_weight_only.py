"""Pins for the weight-only functions of the oracle (Table 13: W4 with a group
size of 128 and 16-bit activations; group-wise granularity of the appendix on
quantization granularity; Eq. (2) with z = 0)."""
import os
from fractions import Fraction

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


def _fp16_rne(fr: Fraction) -> Fraction:
    """Round a rational to the nearest normal fp16 value, ties to even, with integer arithmetic."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = 0
    while a >= 2:
        a /= 2
        e += 1
    while a < 1:
        a *= 2
        e -= 1
    assert -14 <= e <= 15
    scaled = a * 1024                       # 10 fraction bits
    lo = scaled.numerator // scaled.denominator
    rem = scaled - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return sign * Fraction(lo, 1024) * Fraction(2) ** e


def test_hand_worked_group_linear(golden_dir):
    g = _load(os.path.join(golden_dir, "w4_group_linear_2x4.txt"))
    group = int(g["group"][0][0])
    x = g["x"].astype(np.float16)
    wq = g["wq"].astype(np.int8)
    s = g["s"].astype(np.float16)
    wd = orc.dequant_weight_groups_f16(wq, s, group)
    assert wd.dtype == np.float16 and (wd.astype(np.float64) == g["wd"]).all()
    ref, mag = orc.w4g128_linear(x, wq, s, group)
    assert (ref == g["y"]).all() and (mag == g["mag"]).all()
    codes, sc = orc.quantize_weight_groups_int4(g["qrow"], group=4)
    assert (codes == g["qcodes"].astype(np.int8)).all() and sc.tolist() == [[1.0]]


def test_dequantised_weight_is_rounded_once_to_fp16():
    """7 * fp16(0.1) = 0.6998291015625 is not an fp16 value: it becomes 1433 * 2^-11."""
    s = np.array([[0.1]], dtype=np.float16)
    assert Fraction(float(s[0, 0])) == Fraction(0.0999755859375)
    wd = orc.dequant_weight_groups_f16(np.array([[7]], dtype=np.int8), s, group=1)
    assert float(wd[0, 0]) == 1433 * 2.0 ** -11
    rng = np.random.default_rng(5)
    sc = rng.uniform(0.001, 0.05, size=(3, 4)).astype(np.float16)
    wq = rng.integers(-8, 8, size=(3, 8), dtype=np.int8)
    got = orc.dequant_weight_groups_f16(wq, sc, group=2)
    for n in range(3):
        for k in range(8):
            want = _fp16_rne(Fraction(int(wq[n, k])) * Fraction(float(sc[n, k // 2])))
            assert Fraction(float(got[n, k])) == want, (n, k)


def test_unit_scales_reduce_to_the_integer_product():
    rng = np.random.default_rng(6)
    T, N, K = 3, 5, 256
    x = rng.integers(-20, 21, size=(T, K)).astype(np.float16)
    wq = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    ref, mag = orc.w4g128_linear(x, wq, np.ones((N, 2), dtype=np.float16))
    want = [[sum(int(x[t, k]) * int(wq[n, k]) for k in range(K)) for n in range(N)] for t in range(T)]
    assert (ref == np.array(want, dtype=np.float64)).all()
    assert (mag >= np.abs(ref)).all()


def test_scale_of_a_group_weighs_only_its_own_channels():
    """With power-of-two scales the result is sum_g s[n,g] * (x_g . wq[n,g]) exactly; raising one
    scale changes exactly one term.  N != K/group, so a transposed scale table cannot pass."""
    rng = np.random.default_rng(7)
    T, N, K, G = 2, 5, 384, 128
    x = rng.integers(-9, 10, size=(T, K)).astype(np.float16)
    wq = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    expo = rng.integers(-6, 1, size=(N, K // G))
    s = (2.0 ** expo).astype(np.float16)
    ref, _ = orc.w4g128_linear(x, wq, s)
    for t in range(T):
        for n in range(N):
            tot = Fraction(0)
            for g in range(K // G):
                part = sum(int(x[t, k]) * int(wq[n, k]) for k in range(g * G, (g + 1) * G))
                tot += Fraction(float(s[n, g])) * part
            assert Fraction(float(ref[t, n])) == tot, (t, n)
    s2 = s.copy()
    s2[3, 1] *= 2
    ref2, _ = orc.w4g128_linear(x, wq, s2)
    delta = ref2 - ref
    assert (np.delete(delta, 3, axis=1) == 0).all()
    for t in range(T):
        part = sum(int(x[t, k]) * int(wq[3, k]) for k in range(G, 2 * G))
        assert delta[t, 3] == float(s[3, 1]) * part


def test_group_quantiser_scale_codes_and_error_bound():
    rng = np.random.default_rng(8)
    N, K, G = 7, 512, 128
    W = rng.standard_normal((N, K)) * 0.03
    W[2, 128:256] = 0.0                                   # an all-zero group
    W[4, 300] = 0.9                                        # an outlier only widens its own group
    q, s = orc.quantize_weight_groups_int4(W)
    assert q.dtype == np.int8 and s.dtype == np.float16 and s.shape == (N, K // G)
    assert q.min() >= -8 and q.max() <= 7
    assert s[2, 1] == 1.0 and (q[2, 128:256] == 0).all()
    for n in range(N):
        for g in range(K // G):
            blk = W[n, g * G:(g + 1) * G]
            if np.abs(blk).max() > 0:
                assert s[n, g] == np.float16(np.abs(blk).max() / 7.0)
    assert s[4, 2] > 4 * s[4, 1] and s[4, 2] > 4 * s[4, 3]
    sd = np.repeat(s.astype(np.float64), G, axis=1)
    # inside the clamp range the code is the nearest integer to w / s
    assert (np.abs(W / sd - q) <= 0.5 + 1e-12).all() or (np.abs(W / sd) > 7.5).any()
    wd = orc.dequant_weight_groups_f16(q, s).astype(np.float64)
    assert (np.abs(wd - W) <= sd * (0.5 + 8 * 2.0 ** -11) + 1e-12).all()
    # codes of an exactly representable grid are recovered
    q2, s2 = orc.quantize_weight_groups_int4(q.astype(np.float64) * 0.25)
    full = np.abs(q.reshape(N, K // G, G)).max(axis=2) == 7
    assert (q2.reshape(N, K // G, G)[full] == q.reshape(N, K // G, G)[full]).all()
    assert (s2[full] == np.float16(0.25)).all()


def test_planted_mistakes_are_caught(golden_dir):
    """A scale taken per input-channel stripe of the wrong group, or a missing fp16 rounding of the
    dequantised weight, changes the hand-worked / rounding cases above."""
    g = _load(os.path.join(golden_dir, "w4_group_linear_2x4.txt"))
    x = g["x"][0]
    wq = g["wq"]
    s = g["s"]
    wrong = (wq * np.repeat(s[:, ::-1], 2, axis=1)) @ x      # groups swapped
    assert not (wrong == g["y"][0]).all()
    assert 7 * float(np.float16(0.1)) != float(orc.dequant_weight_groups_f16(
        np.array([[7]], dtype=np.int8), np.array([[0.1]], dtype=np.float16), group=1)[0, 0])
