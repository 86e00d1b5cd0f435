"""GPU parity of the weight-only group-128 W4 linear (mquant_w4g128_gemm) against
the oracle.  The dequantised fp16 weight is checked bit for bit through one-hot
activations; the linear within
    1e-3 * |ref| + 1e-5 * sum_k |x_k W~_nk|
of the oracle's double-precision sum: the first term covers the fp16 rounding of
the result (2^-11), the second the fp32 accumulation of the matrix core (K/16
additions of relative error <= 2^-23 on partial sums of size ~ sqrt(K) terms:
below 2e-6 of the absolute sum at K = 18944)."""
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
    print(f"[parity-w4g128] {msg}", flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def pack_int4(wq):
    u = (wq.astype(np.int16) & 0xF).astype(np.uint8)
    return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)


def make_weight(rng, N, K):
    """Gaussian weight with a few large entries, quantised by the oracle's group quantiser."""
    W = rng.standard_normal((N, K)) * 0.02
    W[rng.integers(0, N, 8), rng.integers(0, K, 8)] *= 12.0
    return orc.quantize_weight_groups_int4(W)


def check(y_gpu, ref, mag, what):
    y = y_gpu.astype(np.float64)
    tol = 1e-3 * np.abs(ref) + 1e-5 * mag + 2.0 ** -24
    bad = np.abs(y - ref) > tol
    assert not bad.any(), f"{what}: {int(bad.sum())} outputs out of tolerance (first {np.argwhere(bad)[:3].tolist()})"


def test_dequantised_weight_bit_exact_through_one_hot_rows(mq):
    """x = identity: y[k, n] is the dequantised weight itself, so nibble order, the +8 storage,
    the group of every channel and the single rounding are all fixed bit for bit."""
    rng = np.random.default_rng(31)
    N, K = 72, 384
    wq = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    sc = rng.uniform(0.001, 0.08, size=(N, K // 128)).astype(np.float16)
    sc[0, 0] = np.float16(1e-5)                          # a subnormal scale: subnormal products
    want = orc.dequant_weight_groups_f16(wq, sc)
    wp = mq.w4g128_prepack(dev(pack_int4(wq)), dev(sc))
    x = np.eye(K, dtype=np.float16)
    say(f"one-hot T={K} N={N} K={K}")
    y = mq.w4g128_gemm(dev(x), wp, N).cpu().numpy()
    assert (np.ascontiguousarray(y.T).view(np.uint16) == want.view(np.uint16)).all()
    assert (want[0, :128] != 0).any() and (np.abs(want[0, :128]) < 6.1e-5).any()


@pytest.mark.parametrize("T,N,K", [
    (1, 32, 128), (5, 200, 256), (9, 72, 1152), (16, 200, 640), (31, 40, 2176), (32, 136, 384),   # GEMV
    (33, 64, 128), (64, 136, 384),                          # two GEMV launches
    (50, 16400, 128),                                       # 64x128 GEMM tiles (many channels)
    (65, 264, 512), (130, 300, 256),                        # 128x256 tiles; N % 8 != 0 -> 2-byte stores
    (257, 1000, 640), (300, 520, 1024),
    (1100, 6200, 256),                                      # many tiles, ragged both ways
])
def test_linear_matches_oracle(mq, T, N, K):
    rng = np.random.default_rng(T * 7 + N)
    wq, sc = make_weight(rng, N, K)
    x = (rng.standard_normal((T, K)) * 1.5).astype(np.float16)
    ref, mag = orc.w4g128_linear(x, wq, sc)
    wp = mq.w4g128_prepack(dev(pack_int4(wq)), dev(sc))
    say(f"T={T} N={N} K={K}")
    y = mq.w4g128_gemm(dev(x), wp, N).cpu().numpy()
    check(y, ref, mag, f"w4g128 {(T, N, K)}")


def test_strided_rows_and_untouched_padding(mq):
    rng = np.random.default_rng(41)
    T, N, K = 150, 264, 256
    wq, sc = make_weight(rng, N, K)
    xb = (rng.standard_normal((T, K + 24)) * 1.5).astype(np.float16)
    ref, mag = orc.w4g128_linear(np.ascontiguousarray(xb[:, :K]), wq, sc)
    wp = mq.w4g128_prepack(dev(pack_int4(wq)), dev(sc))
    for pad in (8, 3):                                      # wide stores, then 2-byte stores
        yb = torch.full((T, N + pad), 7.0, dtype=torch.float16, device="cuda")
        say(f"strided ldx={K + 24} ldy={N + pad}")
        mq.w4g128_gemm(dev(xb)[:, :K], wp, N, out=yb[:, :N])
        got = yb.cpu().numpy()
        check(got[:, :N], ref, mag, f"strided pad={pad}")
        assert (got[:, N:] == 7.0).all()


@pytest.mark.parametrize("T,N,K,name", [
    (1280, 37888, 3584, "gate_up 7B"), (1280, 3584, 18944, "down 7B"), (1, 4608, 3584, "qkv decode")])
def test_full_size_sampled(mq, T, N, K, name):
    """The shapes of the 7B model's projections in the launch configuration the benchmark times;
    the oracle computes sampled rows and columns."""
    rng = np.random.default_rng(len(name) + T)
    wq = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    sc = rng.uniform(0.002, 0.01, size=(N, K // 128)).astype(np.float16)
    x = (rng.standard_normal((T, K)) * 1.5).astype(np.float16)
    wp = mq.w4g128_prepack(dev(pack_int4(wq)), dev(sc))
    say(f"full size {name}: T={T} N={N} K={K}")
    y = mq.w4g128_gemm(dev(x), wp, N).cpu().numpy()
    rows = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, 24)]))
    cols = np.unique(np.concatenate([[0, N - 1, N - 33], rng.integers(0, N, 160)]))
    ref, mag = orc.w4g128_linear(x[rows], wq[cols], sc[cols])
    check(y[np.ix_(rows, cols)], ref, mag, f"full size {name}")
    assert np.isfinite(y.astype(np.float32)).all()


def test_argument_errors_and_empty_inputs(mq):
    b = mq
    wq = np.zeros((32, 256), dtype=np.int8)
    sc = np.ones((32, 2), dtype=np.float16)
    wp = b.w4g128_prepack(dev(pack_int4(wq)), dev(sc))
    x = torch.zeros((4, 256), dtype=torch.float16, device="cuda")
    assert b.w4g128_gemm(x[:0], wp, 32).shape == (0, 32)
    assert (b.w4g128_gemm(x, wp, 32).cpu().numpy() == 0).all()
    assert b.lib.mquant_w4g128_prepacked_bytes(32, 192) == b.ERR_UNSUPPORTED
    assert b.lib.mquant_w4g128_prepacked_bytes(-1, 128) == b.ERR_BAD_SHAPE
    assert b.w4g128_prepacked_bytes(33, 256) == 2 * 4 * 1024 + 2 * 64 * 2
    y = torch.zeros((4, 32), dtype=torch.float16, device="cuda")
    lib = b.lib
    assert lib.mquant_w4g128_gemm(x.data_ptr(), 192, wp.data_ptr(), y.data_ptr(), 32, 4, 32, 256, None) == b.ERR_BAD_SHAPE
    assert lib.mquant_w4g128_gemm(x.data_ptr(), 256, wp.data_ptr(), y.data_ptr(), 16, 4, 32, 256, None) == b.ERR_BAD_SHAPE
    assert lib.mquant_w4g128_gemm(x.data_ptr(), 260, wp.data_ptr(), y.data_ptr(), 32, 4, 32, 256, None) == b.ERR_ALIGNMENT
    assert lib.mquant_w4g128_gemm(x.data_ptr() + 2, 256, wp.data_ptr(), y.data_ptr(), 32, 3, 32, 256, None) == b.ERR_ALIGNMENT
    assert lib.mquant_w4g128_gemm(x.data_ptr(), 256, wp.data_ptr(), y.data_ptr(), 32, 4, 32, 64, None) == b.ERR_UNSUPPORTED
    assert lib.mquant_w4g128_gemm(None, 256, wp.data_ptr(), y.data_ptr(), 32, 4, 32, 256, None) == b.ERR_NULL
    torch.cuda.synchronize()


@pytest.mark.parametrize("tile", [0, 1])
def test_both_gemm_tiles_on_ragged_shapes(mq, tile):
    """The dispatcher picks 128x256 or 96x256 from a cost model; force each (the tuning hook of
    the library) so that both see ragged shapes whatever the model prefers."""
    mq.tune_set(mq.TUNE_G128_TILE, tile)
    try:
        rng = np.random.default_rng(70 + tile)
        for T, N, K in [(65, 264, 128), (200, 300, 384), (410, 1000, 640)]:
            wq, sc = make_weight(rng, N, K)
            x = (rng.standard_normal((T, K)) * 1.5).astype(np.float16)
            ref, mag = orc.w4g128_linear(x, wq, sc)
            wp = mq.w4g128_prepack(dev(pack_int4(wq)), dev(sc))
            say(f"tile {tile} T={T} N={N} K={K}")
            y = mq.w4g128_gemm(dev(x), wp, N).cpu().numpy()
            check(y, ref, mag, f"w4g128 tile {tile} {(T, N, K)}")
    finally:
        mq.tune_set(mq.TUNE_G128_TILE, -1)


def test_output_beyond_2_31_elements(mq):
    """T x N > 2^31 outputs: 64-bit addressing of y, on sampled rows (K = one group)."""
    T, N, K = 70000, 37888, 128
    rng = np.random.default_rng(77)
    say(f"w4g128 T={T} N={N} K={K}")
    wq = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    sc = rng.uniform(0.002, 0.01, size=(N, 1)).astype(np.float16)
    x = torch.randn((T, K), device="cuda", generator=torch.Generator(device="cuda").manual_seed(3)).half()
    wp = mq.w4g128_prepack(dev(pack_int4(wq)), dev(sc))
    y = torch.full((T, N), 9.0, dtype=torch.float16, device="cuda")
    mq.w4g128_gemm(x, wp, N, out=y)
    torch.cuda.synchronize()
    mark = 2 ** 31 // N
    rows = torch.tensor([0, 127, 128, mark - 1, mark, mark + 1, T - 129, T - 1], device="cuda")
    ref, mag = orc.w4g128_linear(x[rows].cpu().numpy(), wq, sc)
    check(y[rows].cpu().numpy(), ref, mag, "w4g128 beyond 2^31")
    assert not bool((y == 9.0).all(dim=1).any().item())
    del y
    torch.cuda.empty_cache()
