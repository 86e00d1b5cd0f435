"""Property-based pins of the oracle (hypothesis): statements that hold for every input, checked on
drawn inputs against brute-force definitions written out here."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import mquant_oracle as orc

FAST = settings(max_examples=60, deadline=None)


@st.composite
def spans_in(draw, max_T=40):
    """T and a sorted list of disjoint half-open visual spans inside [0, T)."""
    T = draw(st.integers(1, max_T))
    cuts = sorted(draw(st.lists(st.integers(0, T), min_size=0, max_size=8, unique=True)))
    if len(cuts) % 2:
        cuts = cuts[:-1]
    spans = [(cuts[i], cuts[i + 1] - cuts[i]) for i in range(0, len(cuts), 2)]
    return T, spans


@FAST
@given(spans_in())
def test_aifs_order_is_the_stable_partition(ts):
    """E^u lists the visual tokens in their original order, then the text tokens in theirs
    (Sec. 3.1): written out as two list comprehensions."""
    T, spans = ts
    perm, inv, V = orc.aifs_build_perm(T, spans)
    is_vis = np.zeros(T, dtype=bool)
    for s, l in spans:
        is_vis[s:s + l] = True
    want = [i for i in range(T) if is_vis[i]] + [i for i in range(T) if not is_vis[i]]
    assert perm.tolist() == want and V == int(is_vis.sum())
    assert (inv[perm] == np.arange(T)).all()


@FAST
@given(spans_in(max_T=24))
def test_unified_mask_is_causality_in_original_positions(ts):
    """M^u[i, j] = 1 exactly when token j of E^u was not after token i in E (Eq. (5) carried
    through the reorder): element by element."""
    T, spans = ts
    perm, _, _ = orc.aifs_build_perm(T, spans)
    mu = orc.aifs_remap_mask(orc.causal_mask(T), perm)
    for i in range(T):
        for j in range(T):
            assert mu[i, j] == (1 if perm[j] <= perm[i] else 0)
    assert (mu.sum(axis=1) == perm + 1).all()            # token i sees itself and everything before it


@FAST
@given(st.integers(0, 2 ** 32 - 1), st.floats(0.01, 3.0), st.floats(0.01, 3.0), st.integers(0, 7))
def test_quantizer_matches_eq2_element_by_element(seed, s_vis, s_txt, V):
    """Eq. (2) with z = 0 and Eq. (3): clamp(round_half_even(x / s_row), -128, 127), the division
    realised as the fp32 multiplier of the oracle's header; B = 1 so that u = x."""
    rng = np.random.default_rng(seed)
    u = (rng.standard_normal((7, 16)) * 60).astype(np.float32)
    got = orc.msq_quantize(u, V, s_vis, s_txt, 1)
    for i in range(7):
        c = orc.quant_multiplier(s_vis if i < V else s_txt, 1)
        for k in range(16):
            t = np.float32(u[i, k]) * np.float32(c)
            want = int(np.clip(np.rint(np.float64(t)), -128, 127))
            assert got[i, k] == want


@FAST
@given(st.integers(0, 2 ** 32 - 1))
def test_int4_pack_unpack_and_integer_gemm(seed):
    rng = np.random.default_rng(seed)
    N, K, T = int(rng.integers(1, 6)), 2 * int(rng.integers(1, 9)), int(rng.integers(1, 5))
    w = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    u = (w.astype(np.int16) & 0xF).astype(np.uint8)
    packed = (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)
    assert (orc.unpack_w4(packed) == w).all()
    xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
    acc = orc.gemm_i8_i4_i32(xq, w)
    want = [[sum(int(xq[t, k]) * int(w[n, k]) for k in range(K)) for n in range(N)] for t in range(T)]
    assert acc.tolist() == want


@FAST
@given(st.integers(0, 2 ** 32 - 1), st.sampled_from([2, 4, 8, 16, 32]))
def test_block_hadamard_is_the_dense_product_on_integers(seed, B):
    """On small integers every butterfly is exact, so the fixed stage order must reproduce the
    dense product with the Sylvester matrix of every block."""
    rng = np.random.default_rng(seed)
    x = rng.integers(-50, 51, size=(3, 2 * B)).astype(np.float16)
    got = orc.hadamard_rotate(x, B)
    H = orc.hadamard_matrix(B).astype(np.float64)
    for b in range(2):
        want = x[:, b * B:(b + 1) * B].astype(np.float64) @ H
        assert (got[:, b * B:(b + 1) * B].astype(np.float64) == want).all()
