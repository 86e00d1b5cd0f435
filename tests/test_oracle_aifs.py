"""Pins for the AIFS part of the oracle (Sec. 3.1, Eq. (5), Eq. (6), appendix on
rotary position embedding): the printed index formula, permutation properties,
the closed-form unified mask against the perm rule, attention invariance."""
import itertools
import os

import numpy as np
import pytest

from oracle import mquant_oracle as orc


def _read_index_cases(golden_dir):
    cases = []
    with open(os.path.join(golden_dir, "aifs_index_formula.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            left, right = line.split("|")
            L, m, n = (int(t) for t in left.split())
            cases.append((L, m, n, [int(t) for t in right.split()]))
    return cases


def test_perm_matches_printed_index_formula(golden_dir):
    cases = _read_index_cases(golden_dir)
    assert len(cases) >= 5
    for L, m, n, order_1based in cases:
        perm, inv, V = orc.aifs_build_perm(L, [(m - 1, n - m + 1)])
        assert V == n - m + 1
        assert (perm + 1).tolist() == order_1based


def test_perm_formula_all_single_spans():
    for L in range(1, 14):
        for m in range(1, L + 1):
            for n in range(m, L + 1):
                perm, inv, V = orc.aifs_build_perm(L, [(m - 1, n - m + 1)])
                expect = list(range(m, n + 1)) + list(range(1, m)) + list(range(n + 1, L + 1))
                assert (perm + 1).tolist() == expect
                assert sorted(perm.tolist()) == list(range(L))
                assert (perm[inv] == np.arange(L)).all()
                assert (inv[perm] == np.arange(L)).all()


def test_perm_no_span_is_identity_and_full_span_is_identity():
    perm, inv, V = orc.aifs_build_perm(9, [])
    assert V == 0 and perm.tolist() == list(range(9)) and inv.tolist() == list(range(9))
    perm, inv, V = orc.aifs_build_perm(9, [(0, 9)])
    assert V == 9 and perm.tolist() == list(range(9))
    perm, inv, V = orc.aifs_build_perm(0, [])
    assert V == 0 and perm.shape == (0,)


def test_perm_multi_span_is_stable_partition():
    T = 23
    spans = [(2, 3), (9, 4), (20, 2)]
    perm, inv, V = orc.aifs_build_perm(T, spans)
    assert V == 9
    vis = [2, 3, 4, 9, 10, 11, 12, 20, 21]
    txt = [i for i in range(T) if i not in vis]
    assert perm.tolist() == vis + txt
    # stable: strictly increasing inside each modality
    assert (np.diff(perm[:V]) > 0).all() and (np.diff(perm[V:]) > 0).all()


def test_perm_rejects_bad_spans():
    with pytest.raises(ValueError):
        orc.aifs_build_perm(8, [(6, 4)])
    with pytest.raises(ValueError):
        orc.aifs_build_perm(8, [(1, 3), (3, 2)])


def test_permute_rows_is_a_gather():
    x = np.arange(7 * 3, dtype=np.float16).reshape(7, 3)
    perm, _, _ = orc.aifs_build_perm(7, [(2, 3)])
    xu = orc.aifs_permute_rows(x, perm)
    assert xu[:, 0].tolist() == [6, 9, 12, 0, 3, 15, 18]
    assert xu.dtype == np.float16


def test_causal_mask_is_lower_triangular():
    M = orc.causal_mask(5)
    assert M.dtype == bool
    assert (M == np.tril(np.ones((5, 5), dtype=bool))).all()


def test_eq6_closed_form_equals_perm_rule_bruteforce():
    """Eq. (6) (with V = n-m+1 where the paper prints n-m) must be the causal
    mask carried through the reorder, for every single segment up to L = 12."""
    for L in range(1, 13):
        M = orc.causal_mask(L)
        for m in range(1, L + 1):
            for n in range(m, L + 1):
                perm, _, V = orc.aifs_build_perm(L, [(m - 1, n - m + 1)])
                Mu = orc.aifs_remap_mask(M, perm)
                assert (Mu == orc.unified_mask_eq6(L, m, n)).all(), (L, m, n)
                # explicit definition: allowed iff original position of j <= that of i
                expect = perm.reshape(1, L) <= perm.reshape(L, 1)
                assert (Mu == expect).all()


def test_eq6_as_printed_is_off_by_one():
    """Documents the reading: with the printed (n-m) the formula is NOT the
    remapped causal mask (it differs for the last visual token)."""
    L, m, n = 7, 3, 5
    perm, _, _ = orc.aifs_build_perm(L, [(m - 1, n - m + 1)])
    Mu = orc.aifs_remap_mask(orc.causal_mask(L), perm)
    printed = np.zeros((L, L), dtype=bool)
    for i in range(1, L + 1):
        for j in range(1, L + 1):
            if i <= n - m:
                ok = (j <= i) or (n - m < j <= n)
            elif i <= n:
                ok = n - m < j <= i
            else:
                ok = j <= i
            printed[i - 1, j - 1] = ok
    assert not (printed == Mu).all()


def test_remapped_mask_row_counts():
    T = 40
    perm, _, _ = orc.aifs_build_perm(T, [(5, 11), (22, 9)])
    Mu = orc.aifs_remap_mask(orc.causal_mask(T), perm)
    assert (Mu.sum(axis=1) == perm + 1).all()
    assert Mu.diagonal().all()


def test_remap_mask_on_arbitrary_mask():
    rng = np.random.default_rng(3)
    M = rng.integers(0, 2, size=(9, 9)).astype(bool)
    perm, _, _ = orc.aifs_build_perm(9, [(3, 4)])
    Mu = orc.aifs_remap_mask(M, perm)
    for i, j in itertools.product(range(9), range(9)):
        assert Mu[i, j] == M[perm[i], perm[j]]


@pytest.mark.parametrize("T,spans,D", [
    (12, [(3, 5)], 8),
    (33, [(4, 7), (15, 9), (30, 3)], 16),
    (64, [(8, 48)], 32),
])
def test_attention_invariance(T, spans, D):
    """Sec. 3.1: attention on the reordered tokens with M^u equals the original
    attention, row i of the new result being row perm[i] of the old one."""
    rng = np.random.default_rng(T)
    Q, K, Vv = (rng.standard_normal((T, D)) for _ in range(3))
    perm, inv, V = orc.aifs_build_perm(T, spans)
    M = orc.causal_mask(T)
    Mu = orc.aifs_remap_mask(M, perm)
    ref = orc.causal_attention_f64(Q, K, Vv, M)
    got = orc.causal_attention_f64(orc.aifs_permute_rows(Q, perm), orc.aifs_permute_rows(K, perm),
                                   orc.aifs_permute_rows(Vv, perm), Mu)
    np.testing.assert_allclose(got, ref[perm], rtol=0, atol=1e-12)
    # and a wrong mask (plain causal on the reordered tokens) must break it
    bad = orc.causal_attention_f64(orc.aifs_permute_rows(Q, perm), orc.aifs_permute_rows(K, perm),
                                   orc.aifs_permute_rows(Vv, perm), M)
    assert np.abs(bad - ref[perm]).max() > 1e-3


def test_attention_invariance_config2_layout_sampled_rows():
    """Config-2 layout (T = 4096, 3584 visual tokens at offset 256): checked on a
    sample of rows so the fp64 attention stays cheap."""
    T, D = 4096, 16
    rng = np.random.default_rng(2)
    Q, K, Vv = (rng.standard_normal((T, D)) for _ in range(3))
    perm, inv, V = orc.aifs_build_perm(T, [(256, 3584)])
    assert V == 3584
    rows = np.array([0, 1, 255, 256, 257, 2000, 3583, 3584, 3585, 3839, 3840, 4095])
    Mu_rows = perm.reshape(1, T) <= perm[rows].reshape(-1, 1)
    got = orc.causal_attention_f64(Q[perm][rows], K[perm], Vv[perm], Mu_rows)
    M_rows = np.arange(T).reshape(1, T) <= perm[rows].reshape(-1, 1)
    ref = orc.causal_attention_f64(Q[perm[rows]], K, Vv, M_rows)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
