"""Pins for the multi-head AIFS attention and the rotary embedding with reordered
position ids (Sec. 3.1, Eq. (5)-(6); appendix "Rotary Position Embedding for AIFS")."""
import math

import numpy as np
import pytest

from oracle import mquant_oracle as orc


def _rand(rng, T, H, D):
    return rng.standard_normal((T, H * D))


def test_position_rule_equals_eq6_regions_for_every_single_span():
    """pos[j] <= pos[i] is the three-region rule of Eq. (6) (with V = n-m+1)."""
    for L in range(1, 11):
        for m in range(1, L + 1):
            for n in range(m, L + 1):
                perm, _, V = orc.aifs_build_perm(L, [(m - 1, n - m + 1)])
                allowed = perm[None, :] <= perm[:, None]
                assert (allowed == orc.unified_mask_eq6(L, m, n)).all(), (L, m, n)


def test_multi_head_attention_is_per_head_masked_softmax():
    rng = np.random.default_rng(0)
    T, Hq, Hkv, D = 13, 4, 2, 8
    q, k, v = _rand(rng, T, Hq, D), _rand(rng, T, Hkv, D), _rand(rng, T, Hkv, D)
    perm, _, _ = orc.aifs_build_perm(T, [(3, 5)])
    out = orc.aifs_attention_f64(q, k, v, perm, Hq, Hkv)
    # brute force, element by element
    for h in range(Hq):
        g = h // 2
        for i in range(T):
            w = np.array([math.exp(q[i, h * D:(h + 1) * D] @ k[j, g * D:(g + 1) * D] / math.sqrt(D))
                          if perm[j] <= perm[i] else 0.0 for j in range(T)])
            want = (w[:, None] * v[:, g * D:(g + 1) * D]).sum(axis=0) / w.sum()
            assert np.allclose(out[i, h * D:(h + 1) * D], want, rtol=1e-12, atol=1e-12)


def test_attention_is_invariant_under_the_aifs_reorder():
    """Reordering tokens and switching to the unified mask leaves every token's output
    unchanged (the invariance AIFS is named for), several visual spans included."""
    rng = np.random.default_rng(1)
    T, Hq, Hkv, D = 40, 6, 2, 16
    q, k, v = _rand(rng, T, Hq, D), _rand(rng, T, Hkv, D), _rand(rng, T, Hkv, D)
    ref = orc.aifs_attention_f64(q, k, v, np.arange(T), Hq, Hkv)          # original order, causal
    perm, _, _ = orc.aifs_build_perm(T, [(2, 9), (20, 7), (33, 4)])
    got = orc.aifs_attention_f64(q[perm], k[perm], v[perm], perm, Hq, Hkv)
    assert np.allclose(got, ref[perm], rtol=1e-12, atol=1e-12)
    # and a plain lower-triangular mask on the reordered tokens is wrong
    bad = orc.aifs_attention_f64(q[perm], k[perm], v[perm], np.arange(T), Hq, Hkv)
    assert not np.allclose(bad, ref[perm], rtol=1e-3, atol=1e-3)


def test_closed_forms():
    rng = np.random.default_rng(2)
    T, H, D = 9, 2, 4
    k, v = _rand(rng, T, H, D), _rand(rng, T, H, D)
    perm, _, _ = orc.aifs_build_perm(T, [(4, 3)])
    # zero queries: uniform weights over the allowed set -> mean of allowed values
    out = orc.aifs_attention_f64(np.zeros((T, H * D)), k, v, perm, H, H)
    for i in range(T):
        allowed = perm <= perm[i]
        assert np.allclose(out[i], v[allowed].mean(axis=0), rtol=1e-13, atol=1e-13)
    # the token that came first in the original sequence sees only itself
    first = int(np.where(perm == 0)[0][0])
    out2 = orc.aifs_attention_f64(_rand(rng, T, H, D), k, v, perm, H, H)
    assert np.allclose(out2[first], v[first], rtol=1e-13, atol=1e-13)
    # rows subset
    sub = orc.aifs_attention_f64(_rand(np.random.default_rng(3), T, H, D), k, v, perm, H, H, rows=[1, 7])
    full = orc.aifs_attention_f64(_rand(np.random.default_rng(3), T, H, D), k, v, perm, H, H)
    assert np.allclose(sub, full[[1, 7]])


# ---------------------------------------------------------------------- RoPE

def test_rope_frequencies_and_small_case_by_hand():
    f = orc.rope_inv_freq(4)
    assert np.allclose(f, [1.0, 10000.0 ** -0.5])                      # theta_1 = 1, theta_2 = 1/100
    x = np.array([[1.0, 0.0, 0.0, 2.0]])
    out = orc.rope_apply_f64(x, [3], 1)
    want = [math.cos(3.0), math.sin(3.0), -2.0 * math.sin(0.03), 2.0 * math.cos(0.03)]
    assert np.allclose(out[0], want, rtol=1e-14, atol=1e-14)


def test_rope_position_zero_is_identity_and_norms_are_kept():
    rng = np.random.default_rng(4)
    x = _rand(rng, 6, 3, 8)
    assert np.allclose(orc.rope_apply_f64(x, np.zeros(6), 3), x)
    y = orc.rope_apply_f64(x, [5, 0, 17, 2, 9, 1000], 3)
    assert np.allclose((y.reshape(6, 3, 4, 2) ** 2).sum(-1), (x.reshape(6, 3, 4, 2) ** 2).sum(-1))


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(5)
    D = 16
    qv, kv = rng.standard_normal((1, D)), rng.standard_normal((1, D))
    def score(pq, pk):
        return (orc.rope_apply_f64(qv, [pq], 1) @ orc.rope_apply_f64(kv, [pk], 1).T).item()
    assert math.isclose(score(10, 3), score(107, 100), rel_tol=1e-10, abs_tol=1e-12)
    assert math.isclose(score(5, 5), (qv @ kv.T).item(), rel_tol=1e-12)
    assert not math.isclose(score(10, 3), score(10, 4), rel_tol=1e-6)


def test_rope_with_reordered_ids_commutes_with_the_reorder():
    """Applying RoPE with position ids = the AIFS index vector to reordered tokens equals
    reordering the RoPE'd original tokens (what keeps attention equivalent, appendix)."""
    rng = np.random.default_rng(6)
    T, H, D = 12, 2, 8
    x = _rand(rng, T, H, D)
    perm, _, _ = orc.aifs_build_perm(T, [(3, 4)])
    a = orc.rope_apply_f64(x[perm], perm, H)
    b = orc.rope_apply_f64(x, np.arange(T), H)[perm]
    assert np.allclose(a, b, rtol=1e-14, atol=1e-14)
