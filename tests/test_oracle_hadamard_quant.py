"""Pins for the rotation and the quantizer of the oracle: Walsh-Hadamard matrix
and butterflies (appendix on the Hadamard transform, Sec. 3.2), uniform signed
quantizer (Eq. (2)), modality-specific static scales (Eq. (3))."""
import math
import os

import numpy as np
import pytest

from oracle import mquant_oracle as orc


def _popcount_hadamard(B):
    p = np.arange(B).reshape(B, 1)
    q = np.arange(B).reshape(1, B)
    bits = np.zeros((B, B), dtype=np.int64)
    x = p & q
    while x.any():
        bits += x & 1
        x = x >> 1
    return 1 - 2 * (bits & 1)


# ------------------------------------------------------------------ H matrix

@pytest.mark.parametrize("B", [1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024])
def test_H_Ht_is_B_I_and_closed_form(B):
    H = orc.hadamard_matrix(B)
    assert H.shape == (B, B) and set(np.unique(H).tolist()) <= {-1, 1}
    assert (H @ H.T == B * np.eye(B, dtype=np.int64)).all()
    assert (H == H.T).all()
    assert (H == _popcount_hadamard(B)).all()
    assert (H[0] == 1).all() and (H[:, 0] == 1).all()
    if B > 1:
        assert (H[1:].sum(axis=1) == 0).all()      # "other rows sum to zero"


def test_H4_matches_hand_written_kronecker(golden_dir):
    H4 = np.loadtxt(os.path.join(golden_dir, "h4_sylvester.txt"), dtype=np.int64)
    assert (orc.hadamard_matrix(4) == H4).all()


def test_hadamard_matrix_rejects_non_power_of_two():
    with pytest.raises(ValueError):
        orc.hadamard_matrix(12)


# ---------------------------------------------------------------- butterflies

@pytest.mark.parametrize("B", [2, 4, 8, 16, 64, 128, 512, 1024])
def test_fwht_equals_dense_product_on_small_integers(B):
    """Small integers keep every partial sum exact in fp32, so the butterflies
    must equal x H bit for bit whatever the order."""
    rng = np.random.default_rng(B)
    x = rng.integers(-64, 65, size=B).astype(np.float32)
    got = orc.fwht_block_f32(x)
    want = (x.astype(np.int64) @ orc.hadamard_matrix(B)).astype(np.float32)
    assert (got == want).all()


def test_fwht_unit_vectors_give_rows_of_H():
    B = 16
    H = orc.hadamard_matrix(B)
    for p in range(B):
        e = np.zeros(B, dtype=np.float32)
        e[p] = 1.0
        assert (orc.fwht_block_f32(e) == H[p].astype(np.float32)).all()


def test_fwht_involution_first_element_and_norm():
    B = 512
    rng = np.random.default_rng(7)
    xi = rng.integers(-100, 101, size=B).astype(np.float32)
    u = orc.fwht_block_f32(xi)
    assert (orc.fwht_block_f32(u) == B * xi).all()                  # H H = B I
    assert u[0] == xi.sum()                                         # first row all ones
    x = rng.standard_normal(B).astype(np.float32)
    u = orc.fwht_block_f32(x)
    # normalised: sqrt(B) * mean (Sec. 3.2) and norm preservation
    assert abs(u[0] / math.sqrt(B) - math.sqrt(B) * x.astype(np.float64).mean()) < 1e-4
    n0 = np.linalg.norm(x.astype(np.float64))
    n1 = np.linalg.norm(u.astype(np.float64) / math.sqrt(B))
    assert abs(n1 / n0 - 1.0) < 1e-6


def test_fwht_stage_order_is_h_1_2_4():
    """The fp32 result depends on the stage order; pin it with an input where
    the orders differ: stage h=1 first absorbs the tiny partner of the huge value."""
    x = np.array([2.0 ** 24, 1.0, 1.0, 1.0], dtype=np.float32)
    got = orc.fwht_block_f32(x)
    # h=1: (2^24+1 -> 2^24 (tie to even), 2^24-1, 2, 0); h=2: (2^24+2, 2^24-1, 2^24-2, 2^24-1)
    want = np.array([2.0 ** 24 + 2, 2.0 ** 24 - 1, 2.0 ** 24 - 2, 2.0 ** 24 - 1], dtype=np.float32)
    assert (got == want).all()
    # the other order (h=2 first) gives (2^24+2, 2^24-2, 2^24-1, 2^24-1): slots 1, 2 differ
    other = np.array([x[0] + x[2], x[1] + x[3], x[0] - x[2], x[1] - x[3]], dtype=np.float32)
    other = np.array([other[0] + other[1], other[0] - other[1], other[2] + other[3], other[2] - other[3]],
                     dtype=np.float32)
    assert not (other == want).all()


def test_rotate_is_close_to_exact_fp64_product_on_workload_like_rows():
    """fp16 inputs are multiples of 2^-24 below 2^16, so the fp64 dense product
    is exact; the fp32 butterflies must agree with it to ~1e-6 of the row norm."""
    rng = np.random.default_rng(11)
    B, T = 512, 6
    x = rng.standard_normal((T, 2 * B)).astype(np.float32) * 20.0
    x[:, [3, 97, 200, 411]] *= 50.0
    x = x.astype(np.float16)
    u = orc.hadamard_rotate(x, B)
    H = orc.hadamard_matrix(B).astype(np.float64)
    for b in range(2):
        exact = x[:, b * B:(b + 1) * B].astype(np.float64) @ H
        err = np.abs(u[:, b * B:(b + 1) * B] - exact).max(axis=1)
        scale = np.abs(x[:, b * B:(b + 1) * B].astype(np.float64)).sum(axis=1)
        assert (err <= 1e-6 * scale).all()


def test_rotate_block_structure_and_identity_block():
    rng = np.random.default_rng(5)
    K, B = 256, 64
    x = rng.standard_normal((3, K)).astype(np.float16)
    u0 = orc.hadamard_rotate(x, B)
    x2 = x.copy()
    x2[1, 70] += np.float16(1.0)                     # block 1 of row 1
    u1 = orc.hadamard_rotate(x2, B)
    diff = u0 != u1
    assert diff[1, 64:128].all()
    diff[1, 64:128] = False
    assert not diff.any()
    assert (orc.hadamard_rotate(x, 1) == x.astype(np.float32)).all()
    # blocks are transformed independently and identically
    assert (orc.hadamard_rotate(x[:, 64:128], B) == u0[:, 64:128]).all()
    with pytest.raises(ValueError):
        orc.hadamard_rotate(x, 96)


# ------------------------------------------------------------------ quantizer

def _read_quant_cases(golden_dir):
    xs, codes = [], []
    with open(os.path.join(golden_dir, "quant_exact_multiples.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            a, b = line.split()
            xs.append(float(a))
            codes.append(int(b))
    return np.array(xs, dtype=np.float16), np.array(codes, dtype=np.int64)


def test_quantizer_hand_computed_codes(golden_dir):
    x, codes = _read_quant_cases(golden_dir)
    s = 0.125
    u = orc.hadamard_rotate(x.reshape(1, -1), 1)
    got_t = orc.msq_quantize(u, 0, 999.0, s, 1)       # all rows text
    got_v = orc.msq_quantize(u, 1, s, 999.0, 1)       # all rows visual
    assert got_t.dtype == np.int8
    assert (got_t[0] == codes).all()
    assert (got_v[0] == codes).all()


def test_quantizer_folds_sqrtB_and_uses_per_span_scale():
    """With B = 4, s = 2^-k the multiplier 1/(s sqrt(B)) is a power of two, so
    codes are hand-computable: u = x H_4, code = u / (2 s)."""
    B = 4
    x = np.array([[1.0, 0.0, 0.0, 0.0],      # u = (1, 1, 1, 1)
                  [1.0, 1.0, 1.0, 1.0],      # u = (4, 0, 0, 0)
                  [3.0, 1.0, -1.0, 0.5],     # u = (3.5, 0.5, 4.5, 3.5)
                  [3.0, 1.0, -1.0, 0.5]], dtype=np.float16)
    u = orc.hadamard_rotate(x, B)
    assert (u[2] == np.array([3.5, 0.5, 4.5, 3.5], dtype=np.float32)).all()
    s_vis, s_txt = 0.25, 0.0625                       # multipliers 2 and 8
    xq = orc.msq_quantize(u, 3, s_vis, s_txt, B)
    assert xq[0].tolist() == [2, 2, 2, 2]
    assert xq[1].tolist() == [8, 0, 0, 0]
    assert xq[2].tolist() == [7, 1, 9, 7]
    assert xq[3].tolist() == [28, 4, 36, 28]          # row 3 is text: other scale
    assert float(orc.quant_multiplier(s_vis, B)) == 2.0
    assert float(orc.quant_multiplier(s_txt, B)) == 8.0


def test_quantizer_ties_to_even_not_away():
    u = np.array([[0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 127.5, -127.5, -128.5]], dtype=np.float32)
    xq = orc.msq_quantize(u, 0, 1.0, 1.0, 1)
    assert xq[0].tolist() == [0, 2, 2, 0, -2, -2, 126, 127, -128, -128]


def test_msq_special_cases():
    rng = np.random.default_rng(9)
    u = (rng.standard_normal((10, 32)) * 30).astype(np.float32)
    s1, s2 = 0.3, 0.011
    all_txt = orc.msq_quantize(u, 0, s1, s2, 1)
    all_vis = orc.msq_quantize(u, 10, s2, s1, 1)
    assert (all_txt == all_vis).all()                 # V=0 / V=T: plain per-tensor static
    same = orc.msq_quantize(u, 4, s2, s2, 1)
    assert (same == all_txt).all()                    # equal scales: V irrelevant
    mixed = orc.msq_quantize(u, 4, s1, s2, 1)
    assert (mixed[4:] == all_txt[4:]).all()
    assert (mixed[:4] == orc.msq_quantize(u, 10, s1, s2, 1)[:4]).all()
    assert (mixed[3] != all_txt[3]).any()             # rows V-1 and V use different scales


def test_calibrated_absmax_maps_to_127():
    rng = np.random.default_rng(13)
    for B in (1, 16, 128, 512):
        x = (rng.standard_normal((32, 1024)) * 5).astype(np.float16)
        s = orc.calibrate_static_scale(x, B)
        assert s.dtype == np.float32
        u = orc.hadamard_rotate(x, B)
        want = np.abs(u.astype(np.float64)).max() / math.sqrt(B) / 127.0
        assert abs(float(s) / want - 1.0) < 1e-6
        xq = orc.msq_quantize(u, 0, s, s, B)
        assert np.abs(xq.astype(np.int32)).max() == 127
        assert (np.abs(xq.astype(np.int32)) == 127).sum() >= 1
        # a value 1.5x beyond the calibrated range saturates
        xq2 = orc.msq_quantize(u * np.float32(1.5), 0, s, s, B)
        assert xq2.max() == 127 and xq2.min() >= -128


def test_quantized_rotation_reconstructs_input():
    """Dequantised codes, rotated back with H/sqrt(B), recover x to within the
    quantisation step: pins sign, normalisation and scale direction together."""
    rng = np.random.default_rng(17)
    B = 128
    x = rng.standard_normal((8, 256)).astype(np.float16)
    s = orc.calibrate_static_scale(x, B)
    xq = orc.msq_quantize(orc.hadamard_rotate(x, B), 0, s, s, B)
    H = orc.hadamard_matrix(B).astype(np.float64) / math.sqrt(B)
    for b in range(2):
        rec = (xq[:, b * B:(b + 1) * B].astype(np.float64) * float(s)) @ H.T
        err = rec - x[:, b * B:(b + 1) * B].astype(np.float64)
        assert np.abs(err).max() < float(s) * 0.5 * math.sqrt(B) * 0.5
        assert np.sqrt((err ** 2).mean()) < float(s) / math.sqrt(12) * 1.2


# ------------------------------------------------- other activation bit-widths

def test_a4_quantizer_hand_computed_codes(golden_dir):
    xs, codes = [], []
    with open(os.path.join(golden_dir, "quant_a4_exact_multiples.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                a, b = line.split()
                xs.append(float(a))
                codes.append(int(b))
    u = orc.hadamard_rotate(np.array(xs, dtype=np.float16).reshape(1, -1), 1)
    got = orc.msq_quantize_bits(u, 0, 999.0, 0.5, 1, 4)
    assert (got[0] == np.array(codes)).all()
    assert got.min() == -8 and got.max() == 7


def test_bits_8_is_the_int8_quantizer_and_narrower_is_its_clamp():
    rng = np.random.default_rng(21)
    u = (rng.standard_normal((7, 128)) * 40).astype(np.float32)
    a = orc.msq_quantize(u, 3, 0.9, 0.11, 64)
    assert (orc.msq_quantize_bits(u, 3, 0.9, 0.11, 64, 8) == a).all()
    for bits in (2, 4, 6):
        lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
        assert (orc.msq_quantize_bits(u, 3, 0.9, 0.11, 64, bits) == np.clip(a, lo, hi)).all()
    # scale of Eq. (2) for b = 4: the largest rotated magnitude lands on 7
    s4 = orc.static_scale_from_absmax_bits(np.abs(u).max(), 64, 4)
    q4 = orc.msq_quantize_bits(u, 0, s4, s4, 64, 4)
    assert np.abs(q4.astype(np.int64)).max() == 7
