"""GPU parity of the AIFS attention kernel and the rotary embedding with reordered
position ids against the fp64 oracle.

Tolerance of the attention output (derived from the arithmetic), per query i and
channel d: probabilities are rounded to fp16 before the P V product (relative 2^-11
each -> at most 2^-11 sum_j p_ij |v_jd| in the output), the output is rounded to fp16
(2^-11 |o_id|), logits and the softmax statistics are fp32 (1e-6 relative,
negligible).  Bound used: 1.5 * 2^-11 * (sum_j p_ij |v_jd| + |o_id|) + 1e-6, where the
first sum is the oracle's attention applied to |v|.  It scales with what a query really
attends to, so at T = 4096, where a late row averages thousands of values, a key tile
that is wrongly skipped or wrongly admitted still stands out (a bound in max|v| would
hide it).  The tile-indicator cases make that explicit: V is one-hot on channel
(key tile index mod 128), so output channel c is the probability mass of tile c.
RoPE: sines and cosines in double on both sides, products in fp32, fp16 result:
2^-11 relative to the pair's magnitude, bound 1e-3 * |pair|."""
import sys

import numpy as np
import pytest

from oracle import mquant_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mq():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2502_00425_amd import binding
    return binding


def say(msg):
    print(f"[parity-attn] {msg}", flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make_qkv(rng, T, Hq, Hkv, D=128, q_gain=1.0):
    q = (rng.standard_normal((T, Hq * D)) * q_gain).astype(np.float16)
    k = rng.standard_normal((T, Hkv * D)).astype(np.float16)
    v = (rng.standard_normal((T, Hkv * D)) * 2.0).astype(np.float16)
    return q, k, v


def attention_tolerance(q, k, v, pos, Hq, Hkv, ref, rows=None):
    mass = ref if (v >= 0).all() else orc.aifs_attention_f64(q, k, np.abs(v), pos, Hq, Hkv, rows=rows)
    return 1.5 * 2.0 ** -11 * (mass + np.abs(ref)) + 1e-6


def check_attention(mq, q, k, v, pos, Hq, Hkv, rows=None, what=""):
    got = mq.aifs_attention(dev(q), dev(k), dev(v), dev(pos.astype(np.int32)), Hq, Hkv).cpu().numpy()
    ref = orc.aifs_attention_f64(q, k, v, pos, Hq, Hkv, rows=rows)
    if rows is not None:
        got = got[np.asarray(rows)]
    tol = attention_tolerance(q, k, v, pos, Hq, Hkv, ref, rows)
    err = np.abs(got.astype(np.float64) - ref)
    assert np.isfinite(got).all(), what
    worst = np.unravel_index((err - tol).argmax(), err.shape)
    assert (err <= tol).all(), f"{what}: error {err[worst]:.3e} > {tol[worst]:.3e} at {worst}"
    return ref


def tile_indicator_values(T, Hkv, D=128):
    """v[j] = one-hot on channel (j // 64) % D for every key/value head: the attention output
    channel c of a query is then the probability mass it puts on key tile c (tiles of 64 keys,
    the kernel's tile)."""
    v = np.zeros((T, Hkv * D), dtype=np.float16)
    tile = (np.arange(T) // 64) % D
    for h in range(Hkv):
        v[np.arange(T), h * D + tile] = 1.0
    return v


@pytest.mark.parametrize("T,spans,Hq,Hkv", [
    (64, [(8, 48)], 2, 1),                       # one key tile, configs[0] layout
    (1, [], 1, 1),
    (37, [(0, 5)], 2, 2),                        # ragged, visual first already
    (200, [(16, 100)], 4, 2),                    # several tiles, ragged tail
    (301, [(5, 100), (150, 7), (290, 11)], 3, 1),  # several visual spans, visual at the very end
    (256, [], 2, 1),                             # text only: plain causal
    (256, [(0, 256)], 2, 1),                     # visual only
    # work-group -> (head, query block) mappings: key/value heads that do not divide the 8 XCDs
    # (heads dealt in order), one XCD per key/value head, and a grid with idle work-groups
    (200, [(16, 100)], 6, 3),
    (300, [(40, 120), (200, 30)], 16, 8),
    (130, [(3, 60)], 5, 1),
    (700, [(100, 400)], 12, 6),
])
def test_attention_small_full(mq, T, spans, Hq, Hkv):
    say(f"attention T={T} spans={spans}")
    rng = np.random.default_rng(T + Hq)
    q, k, v = make_qkv(rng, T, Hq, Hkv, q_gain=0.5)
    perm, _, _ = orc.aifs_build_perm(T, spans)
    check_attention(mq, q[perm], k[perm], v[perm], perm, Hq, Hkv, what=f"T={T}")


def test_attention_seeded_layout_sweep(mq):
    """Sixteen seeded layouts: random length (1 .. 700), up to three random visual spans, head
    counts that exercise every work-group mapping; every output against the oracle."""
    rng = np.random.default_rng(2024)
    heads = [(1, 1), (2, 1), (4, 2), (6, 3), (8, 8), (7, 1), (5, 5), (12, 4)]
    for case in range(16):
        T = int(rng.integers(1, 701))
        spans, start = [], 0
        for _ in range(int(rng.integers(0, 4))):
            if start >= T:
                break
            s0 = int(rng.integers(start, T))
            ln = int(rng.integers(1, T - s0 + 1))
            spans.append((s0, ln))
            start = s0 + ln + int(rng.integers(0, 20))
        Hq, Hkv = heads[case % len(heads)]
        say(f"attention sweep {case}: T={T} spans={spans} heads={Hq}/{Hkv}")
        q, k, v = make_qkv(rng, T, Hq, Hkv, q_gain=float(rng.choice([0.3, 1.0, 3.0])))
        perm, _, _ = orc.aifs_build_perm(T, spans)
        check_attention(mq, q[perm], k[perm], v[perm], perm, Hq, Hkv, what=f"sweep {case} T={T} {spans} {Hq}/{Hkv}")


def test_attention_peaked_softmax_and_ties(mq):
    """Large logits (one key dominates) and repeated positions (ties attend each other)."""
    say("attention peaked / ties")
    rng = np.random.default_rng(3)
    T, Hq, Hkv = 130, 2, 1
    q, k, v = make_qkv(rng, T, Hq, Hkv, q_gain=4.0)
    pos = rng.integers(0, 20, size=T)
    check_attention(mq, q, k, v, pos, Hq, Hkv, what="ties")


def test_attention_is_invariant_under_the_reorder_on_the_gpu(mq):
    """The claim AIFS is named for, end to end on the device: reordered tokens with the
    position rule give the outputs of the original order, row for row."""
    say("attention invariance")
    rng = np.random.default_rng(4)
    T, Hq, Hkv = 192, 2, 1
    q, k, v = make_qkv(rng, T, Hq, Hkv, q_gain=0.5)
    perm, _, _ = orc.aifs_build_perm(T, [(10, 90), (130, 20)])
    a = mq.aifs_attention(dev(q), dev(k), dev(v), dev(np.arange(T, dtype=np.int32)), Hq, Hkv).cpu().numpy()
    b = mq.aifs_attention(dev(q[perm]), dev(k[perm]), dev(v[perm]), dev(perm.astype(np.int32)), Hq, Hkv).cpu().numpy()
    ref = orc.aifs_attention_f64(q, k, v, np.arange(T), Hq, Hkv)
    tol = 2 * attention_tolerance(q, k, v, np.arange(T), Hq, Hkv, ref)
    assert (np.abs(a[perm].astype(np.float64) - b.astype(np.float64)) <= tol[perm]).all()


def test_attention_strided_views_of_a_qkv_buffer(mq):
    """q, k, v as column slices of one [T, (Hq + 2 Hkv) D] projection output."""
    say("attention strided")
    rng = np.random.default_rng(5)
    T, Hq, Hkv, D = 100, 4, 1, 128
    q, k, v = make_qkv(rng, T, Hq, Hkv, q_gain=0.5)
    perm, _, _ = orc.aifs_build_perm(T, [(20, 50)])
    buf = dev(np.concatenate([q[perm], k[perm], v[perm]], axis=1))
    got = mq.aifs_attention(buf[:, :Hq * D], buf[:, Hq * D:(Hq + Hkv) * D], buf[:, (Hq + Hkv) * D:],
                            dev(perm.astype(np.int32)), Hq, Hkv).cpu().numpy()
    ref = orc.aifs_attention_f64(q[perm], k[perm], v[perm], perm, Hq, Hkv)
    tol = attention_tolerance(q[perm], k[perm], v[perm], perm, Hq, Hkv, ref)
    assert (np.abs(got.astype(np.float64) - ref) <= tol).all()


def test_attention_config2_layout_sampled(mq):
    """configs[2]: T = 4096 (visual 256..3839), 28 query heads on 4 key/value heads; sampled rows."""
    say("attention c2 sampled")
    rng = np.random.default_rng(6)
    T, Hq, Hkv = 4096, 28, 4
    q, k, v = make_qkv(rng, T, Hq, Hkv, q_gain=0.3)
    perm, _, V = orc.aifs_build_perm(T, [(256, 3584)])
    rows = np.unique(np.r_[0, 1, 127, 128, V - 1, V, V + 1, V + 255, V + 256, T - 1, rng.choice(T, 20, replace=False)])
    check_attention(mq, q[perm], k[perm], v[perm], perm, Hq, Hkv, rows=rows, what="c2")


def test_attention_config1_layout_sampled(mq):
    """configs[1]: T = 1280 (visual 16..1039), 28 query heads on 4 key/value heads, the launch
    bench.py times; sampled rows."""
    say("attention c1 sampled")
    rng = np.random.default_rng(7)
    T, Hq, Hkv = 1280, 28, 4
    q, k, v = make_qkv(rng, T, Hq, Hkv, q_gain=0.3)
    perm, _, V = orc.aifs_build_perm(T, [(16, 1024)])
    rows = np.unique(np.r_[0, 1, 127, 128, V - 1, V, V + 15, V + 16, T - 1, rng.choice(T, 24, replace=False)])
    check_attention(mq, q[perm], k[perm], v[perm], perm, Hq, Hkv, rows=rows, what="c1")


def test_attention_config4_layout_sampled(mq):
    """configs[4]: T = 16384, four visual spans of 3072 between five text spans, 28 query heads
    on 4 key/value heads (256 key tiles, 128 query blocks, seven rounds of work-groups): sampled
    rows around every modality and span edge of the reordered sequence."""
    say("attention c4 sampled")
    rng = np.random.default_rng(11)
    T, Hq, Hkv = 16384, 28, 4
    spans = [(800, 3072), (4704, 3072), (8592, 3072), (12488, 3072)]
    q, k, v = make_qkv(rng, T, Hq, Hkv, q_gain=0.3)
    perm, _, V = orc.aifs_build_perm(T, spans)
    inv = np.argsort(perm)
    edges = [0, 1, 63, 64, 127, 128, V - 1, V, V + 1, T - 2, T - 1]
    for s0, l in spans:
        edges += [int(inv[p]) for p in (s0 - 1, s0, s0 + l - 1, s0 + l) if 0 <= p < T]
    rows = np.unique(np.r_[np.array(edges), rng.choice(T, 16, replace=False)])
    check_attention(mq, q[perm], k[perm], v[perm], perm, Hq, Hkv, rows=rows, what="c4")


@pytest.mark.parametrize("name,T,spans,q_gain", [
    ("configs[1]", 1280, [(16, 1024)], 0.3),
    ("configs[2]", 4096, [(256, 3584)], 0.3),
    ("configs[2] peaked", 4096, [(256, 3584)], 4.0),
    ("four spans", 4096, [(200, 768), (1176, 768), (2148, 768), (3122, 768)], 0.3),
    ("configs[4]", 16384, [(800, 3072), (4704, 3072), (8592, 3072), (12488, 3072)], 0.3),
])
def test_attention_every_key_tile_is_visible_on_the_config_layouts(mq, name, T, spans, q_gain):
    """One-hot values per key tile: output channel c of a sampled query is the probability mass
    on key tile c (64 tiles at T = 4096, each with its own channel).  A tile skipped by the
    kernel's tile-level tests (smallest position of the tile against the largest of the query
    group, tiles hidden from or visible to a whole wave) reads 0 where the oracle has its mass,
    a wrongly admitted one reads mass where the oracle has exactly 0; either is orders of
    magnitude beyond the bound, which is relative to that mass."""
    say(f"attention tile indicator {name}")
    rng = np.random.default_rng(T + len(spans))
    Hq, Hkv = 28, 4
    q, k, _ = make_qkv(rng, T, Hq, Hkv, q_gain=q_gain)
    perm, _, V = orc.aifs_build_perm(T, spans)
    v = tile_indicator_values(T, Hkv)                     # indexed by AIFS row: tiles of the kernel's key order
    edges = [0, 1, 63, 64, 127, 128, V - 1, V, V + 1, T - 2, T - 1]
    for s0, l in spans:                                   # AIFS rows of the tokens around every span edge
        inv = np.argsort(perm)
        edges += [int(inv[p]) for p in (s0 - 1, s0, s0 + l - 1, s0 + l) if 0 <= p < T]
    rows = np.unique(np.r_[np.array(edges), rng.choice(T, 24, replace=False)])
    ref = check_attention(mq, q[perm], k[perm], v, perm, Hq, Hkv, rows=rows, what=name)
    # the case is not degenerate: masked tiles exist (exact zeros) next to visible ones
    assert (ref == 0).any() and (ref > 1e-3).any()


def test_attention_argument_errors(mq):
    x = torch.zeros((4, 128), dtype=torch.float16, device="cuda")
    pos = torch.zeros(4, dtype=torch.int32, device="cuda")
    ws = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    call = lambda hq, hkv, d, wsp, wsb: mq.lib.mquant_aifs_attention(
        x.data_ptr(), 128, x.data_ptr(), 128, x.data_ptr(), 128, x.data_ptr(), 128, pos.data_ptr(), 4,
        hq, hkv, d, wsp, wsb, None)
    assert call(1, 1, 64, ws.data_ptr(), 1 << 16) == mq.ERR_UNSUPPORTED
    assert call(3, 2, 128, ws.data_ptr(), 1 << 16) == mq.ERR_BAD_SHAPE
    assert call(1, 1, 128, None, 0) == mq.ERR_WORKSPACE
    assert call(2, 1, 128, ws.data_ptr(), 1 << 16) == mq.ERR_BAD_SHAPE      # ldq < 2 * 128
    assert call(1, 1, 128, ws.data_ptr(), 1 << 16) == mq.OK
    torch.cuda.synchronize()


# ---------------------------------------------------------------------- RoPE

@pytest.mark.parametrize("T,H", [(1, 1), (77, 4), (1280, 32)])
def test_rope_matches_oracle(mq, T, H):
    say(f"rope T={T} H={H}")
    rng = np.random.default_rng(T + H)
    D = 128
    x = rng.standard_normal((T, H * D)).astype(np.float16)
    perm, _, _ = orc.aifs_build_perm(T, [(T // 5, T // 2)]) if T > 4 else (np.arange(T), None, 0)
    pos = perm.astype(np.int64) * (16000 // max(T, 1) if T > 1 else 1)      # positions up to ~16000
    xd = dev(x[perm])
    mq.rope_apply(xd, dev(pos.astype(np.int32)), H)
    got = xd.cpu().numpy().astype(np.float64)
    ref = orc.rope_apply_f64(x[perm], pos, H)
    mag = np.sqrt((ref.reshape(T, H, D // 2, 2) ** 2).sum(-1))
    err = np.abs(got - ref).reshape(T, H, D // 2, 2).max(-1)
    assert (err <= 1e-3 * np.maximum(mag, 2.0 ** -14)).all()


def test_rope_leaves_the_rest_of_the_row_alone(mq):
    rng = np.random.default_rng(9)
    x = rng.standard_normal((10, 3 * 128)).astype(np.float16)
    xd = dev(x)
    mq.rope_apply(xd, dev(np.arange(10, dtype=np.int32)), 2)        # rotate the first two heads only
    got = xd.cpu().numpy()
    assert (got[:, 256:] == x[:, 256:]).all()
    assert (got[0] == x[0]).all()                                   # position 0: identity
    assert not (got[1:, :256] == x[1:, :256]).all()
