"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the
same seeded inputs.  Bit-exact on the permutation, the int8 codes and the
int32 accumulators; |y - ref| <= 1e-3 * max(|ref|, 2^-14) on the fp16 output
(ref = the oracle's fp32 dequantised value) -- and, on the configurations, the
oracle's fp16 bits exactly, since both sides round the same fp32 product."""
import math
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import mquant_oracle as orc                      # noqa: E402
from paper_2502_00425_amd import workloads as wl             # noqa: E402


@pytest.fixture(scope="module")
def mq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2502_00425_amd import binding
    return binding


@pytest.fixture
def forced_tile(mq):
    """Sets a tuning override of the library and puts the cost model back afterwards."""
    keys = []

    def force(key, value):
        mq.tune_set(key, value)
        keys.append(key)
    yield force
    for key in keys:
        mq.tune_set(key, 0 if key == mq.TUNE_GEMM_NOSPLIT else -1)


def say(msg):
    print(f"[parity] {msg}", flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_y(y_gpu, ref, what):
    y = y_gpu.astype(np.float32)
    tol = 1e-3 * np.maximum(np.abs(ref), 2.0 ** -14)
    bad = np.abs(y - ref) > tol
    assert not bad.any(), f"{what}: {int(bad.sum())} outputs beyond 1e-3 (first {np.argwhere(bad)[:3].tolist()})"
    assert (y[ref == 0] == 0).all(), f"{what}: zero reference but non-zero output"


def scales_from_calib(inp):
    B = inp["had_block"]
    s_vis = float(orc.calibrate_static_scale(inp["calib_vis"], B))
    s_txt = float(orc.calibrate_static_scale(inp["calib_txt"], B))
    return s_vis, s_txt


# ------------------------------------------------------------------ AIFS

@pytest.mark.parametrize("T,K,spans", [
    (64, 512, [(8, 48)]),
    (301, 264, [(5, 100), (150, 7), (290, 11)]),
    (1, 8, []),
    (1280, 3584, [(16, 1024)]),
])
def test_aifs_permute(mq, T, K, spans):
    say(f"permute T={T} K={K}")
    rng = np.random.default_rng(T + K)
    x = rng.standard_normal((T, K)).astype(np.float16)
    perm, inv, V = mq.aifs_build_perm(T, spans)
    operm, _, oV = orc.aifs_build_perm(T, spans)
    assert V == oV and (perm == operm).all()
    got = mq.aifs_permute(dev(x), dev(perm)).cpu().numpy()
    want = orc.aifs_permute_rows(x, operm)
    assert (got.view(np.uint16) == want.view(np.uint16)).all()


def test_aifs_permute_strided(mq):
    say("permute strided")
    rng = np.random.default_rng(5)
    T, K = 37, 72
    big = rng.standard_normal((T, 96)).astype(np.float16)
    perm, _, _ = orc.aifs_build_perm(T, [(3, 20)])
    xd = dev(big)[:, :K]
    out = torch.zeros((T, 80), dtype=torch.float16, device="cuda")
    mq.aifs_permute(xd, dev(perm), out=out[:, :K])
    got = out.cpu().numpy()
    assert (got[:, :K] == big[perm][:, :K]).all()
    assert (got[:, K:] == 0).all()


@pytest.mark.parametrize("T,spans", [(64, [(8, 48)]), (203, [(9, 50), (100, 31)]), (7, [])])
def test_aifs_remap_mask_small(mq, T, spans):
    say(f"mask T={T}")
    rng = np.random.default_rng(T)
    perm, _, _ = orc.aifs_build_perm(T, spans)
    for M in (orc.causal_mask(T), rng.integers(0, 2, size=(T, T)).astype(bool)):
        got = mq.aifs_remap_mask(dev(M.astype(np.uint8)), dev(perm)).cpu().numpy()
        assert (got == orc.aifs_remap_mask(M, perm).astype(np.uint8)).all()


@pytest.mark.parametrize("T,spans", [(1024, [(10, 300), (500, 24), (900, 124)]), (16, [(4, 8)]), (2064, [(0, 2064)]),
                                     (18448, [(100, 9000)])])
def test_aifs_remap_mask_staged_rows(mq, T, spans):
    """T % 16 == 0 takes the kernel that stages source rows in LDS (8, 4 or 1 rows per group
    depending on T); any non-zero input byte means "may attend" and comes out as 1."""
    say(f"mask staged rows T={T}")
    rng = np.random.default_rng(T)
    perm, _, _ = orc.aifs_build_perm(T, spans)
    M = rng.choice(np.array([0, 0, 1, 2, 255], dtype=np.uint8), size=(T, T))
    got = mq.aifs_remap_mask(dev(M), dev(perm)).cpu().numpy()
    want = orc.aifs_remap_mask(M != 0, perm).astype(np.uint8)
    assert (got == want).all()


def test_aifs_remap_mask_config2(mq):
    """4096 x 4096 causal mask of config 2: equal to the oracle's remap (which
    the CPU tests tie to Eq. (6) and to attention invariance)."""
    say("mask config2 4096")
    w = wl.workload(2)
    T = w.T
    perm, _, V = orc.aifs_build_perm(T, w.vis_spans)
    M = orc.causal_mask(T)
    got = mq.aifs_remap_mask(dev(M.astype(np.uint8)), dev(perm)).cpu().numpy().astype(bool)
    assert (got == orc.aifs_remap_mask(M, perm)).all()
    assert (got.sum(axis=1) == perm + 1).all()


# --------------------------------------------------- rotation + quantizer

@pytest.mark.parametrize("T,K,B,V,use_perm", [
    (64, 512, 512, 48, True),
    (33, 1024, 1024, 10, False),
    (70, 640, 128, 0, True),
    (70, 640, 128, 70, False),
    (19, 1536, 256, 7, True),
    (5, 64, 16, 2, False),
    (9, 72, 8, 4, True),
    (9, 40, 4, 4, False),
    (9, 40, 2, 4, False),
    (6, 24, 1, 3, True),
    (300, 3584, 512, 111, True),
])
def test_hadamard_quant_bit_exact(mq, T, K, B, V, use_perm):
    say(f"hadamard_quant T={T} K={K} B={B} V={V} perm={use_perm}")
    rng = np.random.default_rng(1000 * B + T)
    x = rng.standard_normal((T, K)).astype(np.float32)
    x[: T // 2] *= 20.0
    x[:, 3 % K] *= 50.0
    x = x.astype(np.float16)
    s_vis, s_txt = 0.37 * math.sqrt(1.0), 0.021
    if use_perm:
        spans = [(min(T // 3, T - V), V)] if V else []
        perm, _, V2 = orc.aifs_build_perm(T, spans)
        assert V2 == V
        permd = dev(perm)
        x_u = orc.aifs_permute_rows(x, perm)
    else:
        permd = None
        x_u = x
    want = orc.msq_quantize(orc.hadamard_rotate(x_u, B), V, s_vis, s_txt, B)
    got = mq.hadamard_quant_act(dev(x), V, s_vis, s_txt, B, perm_dev=permd).cpu().numpy()
    assert got.dtype == np.int8
    assert (got == want).all(), f"{int((got != want).sum())} codes differ"
    assert np.abs(want.astype(np.int32)).max() > 20          # the case is not degenerate


def test_hadamard_quant_strided_input_and_saturation(mq):
    say("hadamard_quant strided + saturation")
    rng = np.random.default_rng(77)
    T, K, B = 21, 512, 512
    big = (rng.standard_normal((T, 1024)) * 300).astype(np.float16)
    x = big[:, :K]
    s = 0.05                                                # far too small: most codes clamp
    want = orc.msq_quantize(orc.hadamard_rotate(np.ascontiguousarray(x), B), 9, s, s * 3, B)
    got = mq.hadamard_quant_act(dev(big)[:, :K], 9, s, s * 3, B).cpu().numpy()
    assert (got == want).all()
    assert (want == 127).sum() > 100 and (want == -128).sum() > 100


@pytest.mark.parametrize("B", [1, 16, 128, 512, 1024])
def test_hadamard_absmax(mq, B):
    say(f"absmax B={B}")
    rng = np.random.default_rng(B)
    x = (rng.standard_normal((50, 2048)) * 7).astype(np.float16)
    want = orc.rotated_absmax(x, B)
    out = torch.zeros(1, dtype=torch.float32, device="cuda")
    mq.hadamard_absmax(dev(x), B, out)
    assert np.float32(out.item()) == want


# -------------------------------------------------------- prepack + GEMM

def run_linear_gpu(mq, inp, s_vis, s_txt, want_acc=True, fused=False):
    T, K, N, B = inp["T"], inp["K"], inp["N"], inp["had_block"]
    perm, inv, V = mq.aifs_build_perm(T, inp["vis_spans"])
    xd = dev(inp["x"])
    permd = dev(perm)
    wp = mq.w4_prepack(dev(inp["w_packed"]))
    wsd = dev(inp["w_scale"])
    out = {"perm": perm, "V": V}
    if fused:
        ws = torch.empty(mq.w4a8_linear_prefill_workspace_bytes(T, N, K), dtype=torch.uint8, device="cuda")
        y = mq.w4a8_linear_prefill(xd, permd, wp, wsd, N, V, s_vis, s_txt, B, ws)
        out["xq"] = ws[: T * K].view(torch.int8).reshape(T, K)
    else:
        xq = mq.hadamard_quant_act(xd, V, s_vis, s_txt, B, perm_dev=permd)
        out["xq"] = xq
        nws = mq.w4a8_workspace_bytes(T, N, K)
        ws = torch.empty(max(nws, 1), dtype=torch.uint8, device="cuda") if nws else None
        acc = torch.empty((T, N), dtype=torch.int32, device="cuda") if want_acc else None
        y = mq.w4a8_gemm(xq, wp, wsd, N, V, s_vis, s_txt, acc_out=acc, workspace=ws)
        out["acc"] = acc
    out["y"] = y
    torch.cuda.synchronize()
    return out


def test_config0_full(mq):
    say("config 0 full")
    w = wl.workload(0)
    inp = wl.make_linear_inputs(w, "lin")
    s_vis, s_txt = scales_from_calib(inp)
    o = orc.w4a8_linear(inp["x"], inp["vis_spans"], inp["w_packed"], inp["w_scale"], s_vis, s_txt, w.had_block)
    for fused in (False, True):
        g = run_linear_gpu(mq, inp, s_vis, s_txt, fused=fused)
        assert (g["perm"] == o["perm"]).all() and g["V"] == o["V"] == 48
        assert (g["xq"].cpu().numpy() == o["xq"]).all()
        if not fused:
            assert (g["acc"].cpu().numpy() == o["acc"]).all()
        check_y(g["y"].cpu().numpy(), o["ref"], f"config0 fused={fused}")
        assert (g["y"].cpu().numpy().view(np.uint16) == o["y"].view(np.uint16)).all()     # same two fp32 multiplies


@pytest.mark.parametrize("T,N,K,V", [
    (300, 544, 384, 120),       # two M tiles, three N tiles, ragged both ways
    (257, 100, 128, 257),       # N below one tile, T one row past a tile
    (512, 256, 1024, 0),
    (40, 72, 256, 13),          # above the GEMV limit, far below one tile
    (130, 300, 192, 64),        # K % 128 != 0
])
def test_gemm_small_shapes_full(mq, T, N, K, V):
    say(f"gemm T={T} N={N} K={K} V={V}")
    rng = np.random.default_rng(T * 7 + N)
    xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    s_vis, s_txt = 0.41, 0.013
    acc_want = orc.gemm_i8_i4_i32(xq, orc.unpack_w4(packed))
    ref, _ = orc.dequant(acc_want, V, s_vis, s_txt, w_scale)
    wp = mq.w4_prepack(dev(packed))
    acc = torch.full((T, N), -7, dtype=torch.int32, device="cuda")
    ldy = N + 8
    ybuf = torch.full((T, ldy), 9.0, dtype=torch.float16, device="cuda")
    mq.w4a8_gemm(dev(xq), wp, dev(w_scale), N, V, s_vis, s_txt, out=ybuf[:, :N], acc_out=acc)
    assert (acc.cpu().numpy() == acc_want).all()
    yb = ybuf.cpu().numpy()
    check_y(yb[:, :N], ref, "gemm small")
    assert (yb[:, N:] == 9.0).all()                           # nothing written past N
    # without acc_out the output is the same
    y2 = mq.w4a8_gemm(dev(xq), wp, dev(w_scale), N, V, s_vis, s_txt).cpu().numpy()
    assert (y2.view(np.uint16) == yb[:, :N].view(np.uint16)).all()


@pytest.mark.parametrize("T,N,K,V,ldy_pad", [
    (300, 520, 8192, 77, 0),     # split-K (few tiles, long K), ragged T and N, wide stores
    (300, 516, 8192, 300, 4),    # split-K with N % 8 != 0: plain stores in the reduce kernel
    (70, 250, 16384, 0, 0),      # N % 4 != 0: split-K is not taken
    (513, 264, 4096, 512, 0),    # one row past two 256-row tiles, K too short to split
])
def test_gemm_split_k_and_store_paths(mq, T, N, K, V, ldy_pad):
    say(f"gemm split/store paths T={T} N={N} K={K}")
    rng = np.random.default_rng(T + N + K)
    xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    s_vis, s_txt = 0.11, 0.004
    acc_want = orc.gemm_i8_i4_i32(xq, orc.unpack_w4(packed))
    ref, _ = orc.dequant(acc_want, V, s_vis, s_txt, w_scale)
    wp = mq.w4_prepack(dev(packed))
    ws_bytes = mq.w4a8_workspace_bytes(T, N, K)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device="cuda")
    ldy = N + ldy_pad
    for want_acc in (False, True):
        ybuf = torch.full((T, ldy), 7.0, dtype=torch.float16, device="cuda")
        acc = torch.full((T, N), -3, dtype=torch.int32, device="cuda") if want_acc else None
        mq.w4a8_gemm(dev(xq), wp, dev(w_scale), N, V, s_vis, s_txt, out=ybuf[:, :N], acc_out=acc,
                     workspace=ws if ws_bytes else None)
        yb = ybuf.cpu().numpy()
        check_y(yb[:, :N], ref, f"split/store want_acc={want_acc}")
        assert (yb[:, N:] == 7.0).all()
        if want_acc:
            assert (acc.cpu().numpy() == acc_want).all()


def test_gemm_workspace_is_required_when_split(mq):
    T, N, K = 300, 520, 8192
    assert mq.w4a8_workspace_bytes(T, N, K) > 0
    xq = torch.zeros((T, K), dtype=torch.int8, device="cuda")
    wp = torch.zeros(mq.w4_prepacked_bytes(N, K), dtype=torch.uint8, device="cuda")
    y = torch.empty((T, N), dtype=torch.float16, device="cuda")
    st = mq.lib.mquant_w4a8_gemm(xq.data_ptr(), wp.data_ptr(), torch.ones(N, dtype=torch.float16, device="cuda").data_ptr(),
                                 y.data_ptr(), N, None, T, N, K, 0, 1.0, 1.0, None, 0, None)
    assert st == mq.ERR_WORKSPACE


def test_gemm_extreme_values_no_overflow(mq):
    say("gemm extremes K=29568")
    K, T, N = 29568, 64, 64
    xq = np.full((T, K), -128, dtype=np.int8)
    xq[1::2] = 127
    packed = np.full((N, K // 2), 0x88, dtype=np.uint8)          # every weight -8
    packed[1::2] = 0x77                                          # every weight +7
    acc_want = orc.gemm_i8_i4_i32(xq, orc.unpack_w4(packed))
    assert acc_want.max() == K * 1024
    acc = torch.empty((T, N), dtype=torch.int32, device="cuda")
    mq.w4a8_gemm(dev(xq), mq.w4_prepack(dev(packed)), dev(np.ones(N, dtype=np.float16)), N, 0,
                 2.0 ** -20, 2.0 ** -20, acc_out=acc)
    assert (acc.cpu().numpy() == acc_want).all()
    # and the decode kernel on the same extremes
    acc1 = torch.empty((2, N), dtype=torch.int32, device="cuda")
    mq.w4a8_gemm(dev(xq[:2]), mq.w4_prepack(dev(packed)), dev(np.ones(N, dtype=np.float16)), N, 0,
                 2.0 ** -20, 2.0 ** -20, acc_out=acc1)
    assert (acc1.cpu().numpy() == acc_want[:2]).all()


def test_gemm_at_the_maximum_k(mq):
    """K = 65536 is the documented limit: the accumulator holds 16 x the sum, and with every
    activation at -128 and every weight at -8 that is 2^30, the largest value it can take.
    Closed form (every product equal) for the accumulators, the oracle for the mixed rows;
    the GEMV, the direct GEMM, split-K with its workspace, and the wide and the 2-byte stores."""
    K, N = 65536, 72
    say(f"gemm at K={K}")
    packed = np.full((N, K // 2), 0x88, dtype=np.uint8)          # every weight -8
    packed[1::2] = 0x77                                          # every weight +7
    wq = orc.unpack_w4(packed)
    wp = mq.w4_prepack(dev(packed))
    ones = dev(np.ones(N, dtype=np.float16))
    for T in (3, 40, 300):
        xq = np.full((T, K), -128, dtype=np.int8)
        xq[1::3] = 127
        xq[2::3, ::2] = 55                                       # a row with mixed values
        acc_want = orc.gemm_i8_i4_i32(xq, wq)
        assert acc_want[0, 0] == K * 1024 == 2 ** 26 and acc_want[0, 1] == -K * 128 * 7
        nws = mq.w4a8_workspace_bytes(T, N, K)
        ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
        acc = torch.empty((T, N), dtype=torch.int32, device="cuda")
        y = mq.w4a8_gemm(dev(xq), wp, ones, N, 0, 2.0 ** -20, 2.0 ** -20, acc_out=acc, workspace=ws)
        assert (acc.cpu().numpy() == acc_want).all(), T
        ref, _ = orc.dequant(acc_want, 0, 2.0 ** -20, 2.0 ** -20, np.ones(N, dtype=np.float16))
        check_y(y.cpu().numpy(), ref, f"max K, T={T}")
        y2 = mq.w4a8_gemm(dev(xq), wp, ones, N, 0, 2.0 ** -20, 2.0 ** -20, workspace=ws)
        check_y(y2.cpu().numpy(), ref, f"max K, no acc_out, T={T}")
    assert mq.lib.mquant_w4_prepacked_bytes(N, K + 64) == mq.ERR_UNSUPPORTED


@pytest.mark.parametrize("T", [1, 2, 4, 16, 31, 32])
def test_gemv_small_shapes_full(mq, T):
    say(f"gemv T={T}")
    rng = np.random.default_rng(T)
    N, K, V = 200, 832, min(T, 3)
    xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    s_vis, s_txt = 0.2, 0.03
    acc_want = orc.gemm_i8_i4_i32(xq, orc.unpack_w4(packed))
    ref, _ = orc.dequant(acc_want, V, s_vis, s_txt, w_scale)
    acc = torch.empty((T, N), dtype=torch.int32, device="cuda")
    y = mq.w4a8_gemm(dev(xq), mq.w4_prepack(dev(packed)), dev(w_scale), N, V, s_vis, s_txt, acc_out=acc)
    assert (acc.cpu().numpy() == acc_want).all()
    check_y(y.cpu().numpy(), ref, f"gemv T={T}")


@pytest.mark.parametrize("T", [1, 3, 4, 7, 16, 21, 32])
@pytest.mark.parametrize("K,Ns", [(3584, (3584, 512, 512)), (1024, (18944, 18944)), (18944, (3584,)),
                                  (384, (40, 0, 200, 72)), (192, (100, 36))])
def test_gemv_grouped_equals_the_oracle_per_linear(mq, T, K, Ns):
    """Several linears sharing one input in one launch (q/k/v; gate/up): every output of every
    linear against the oracle, bit for bit on the fp16 value (accumulators are checked through
    the single-linear entry on the same kernel); untouched padding columns stay untouched.
    Up to 4 rows the streaming kernel takes the group, 5 to 16 rows it takes few-tile groups,
    everything else (and K % 128 != 0) is one launch of the tile kernel."""
    say(f"grouped gemv T={T} K={K} Ns={Ns}")
    rng = np.random.default_rng(T * 1000 + K + len(Ns))
    xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
    V, s_vis, s_txt = min(T, 2), 0.21, 0.034
    lin, want = [], []
    for N in Ns:
        packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
        w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
        out = torch.full((T, N + 8), 3.0, dtype=torch.float16, device="cuda")
        wp = mq.w4_prepack(dev(packed)) if N else torch.empty(0, dtype=torch.uint8, device="cuda")
        lin.append((wp, dev(w_scale), N, out[:, :N]))
        acc = orc.gemm_i8_i4_i32(xq, orc.unpack_w4(packed)) if N else np.zeros((T, 0), dtype=np.int32)
        want.append(orc.dequant(acc, V, s_vis, s_txt, w_scale)[1] if N else np.zeros((T, 0), dtype=np.float16))
    xqd = dev(xq)
    mq.w4a8_gemv_grouped(xqd, lin, V, s_vis, s_txt)
    torch.cuda.synchronize()
    for (wp, ws, N, out), w in zip(lin, want):
        got = out.cpu().numpy()
        assert (got.view(np.uint16) == w.view(np.uint16)).all(), f"N={N}"
        if N:
            assert torch.equal(mq.w4a8_gemm(xqd, wp, ws, N, V, s_vis, s_txt), out)
    # the padding columns of every output buffer still hold the fill value
    for (wp, ws, N, out) in lin:
        buf = out._base if out._base is not None else out
        assert bool((buf[:, N:] == 3.0).all())


@pytest.mark.parametrize("T,N,K", [(5, 200, 1024), (8, 72, 128), (11, 3584, 3584), (16, 520, 18944), (13, 16416, 256),
                                   (16, 18944, 384), (4, 264, 29568), (9, 40, 640)])
def test_gemv_streamed_rows_full(mq, T, N, K):
    """5..16 rows (and few rows of a very long K): the GEMV that streams xq next to the weights,
    16-channel units (few output tiles) and 32-channel units (N >= 16384); accumulators and fp16
    outputs of every element against the oracle."""
    say(f"gemv streamed rows T={T} N={N} K={K}")
    rng = np.random.default_rng(T * 31 + N + K)
    xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    V, s_vis, s_txt = T // 2, 0.2, 0.03
    acc_want = orc.gemm_i8_i4_i32(xq, orc.unpack_w4(packed))
    ref, y_want = orc.dequant(acc_want, V, s_vis, s_txt, w_scale)
    wp = mq.w4_prepack(dev(packed))
    acc = torch.full((T, N), -7, dtype=torch.int32, device="cuda")
    ybuf = torch.full((T, N + 8), 9.0, dtype=torch.float16, device="cuda")
    mq.w4a8_gemm(dev(xq), wp, dev(w_scale), N, V, s_vis, s_txt, out=ybuf[:, :N], acc_out=acc)
    assert (acc.cpu().numpy() == acc_want).all()
    yb = ybuf.cpu().numpy()
    assert (yb[:, :N].view(np.uint16) == y_want.view(np.uint16)).all()
    check_y(yb[:, :N], ref, "gemv streamed rows")
    assert (yb[:, N:] == 9.0).all()


@pytest.mark.parametrize("T,N,K", [(33, 3584, 3584), (64, 520, 1024), (65, 200, 640), (96, 4608, 3584),
                                   (50, 8192, 8192), (40, 72, 18944), (128, 264, 1024), (127, 40, 256),
                                   (129, 264, 1024), (70, 9000, 128), (60, 12320, 256), (64, 12288, 128),
                                   (50, 18944, 384), (64, 37888, 256), (33, 33000, 128), (100, 18944, 256),
                                   (128, 10240, 384), (128, 37888, 128)])
def test_short_prompts_on_small_matrices(mq, T, N, K):
    """33 to 64 rows against a matrix with few output channels (up to 128 rows against a small
    one) run as 64-row passes of the tile GEMV, two row blocks per weight tile, the last pass
    ragged or a plain 32-row one; one row or one tile column more runs as the prefill GEMM,
    which takes 64-row tiles (64x128 or 64x256 by the number of work-groups) up to 128 rows.
    Accumulators and fp16 bits of every output on both sides of each switch, the visual / text
    boundary inside a pass."""
    say(f"short prompt T={T} N={N} K={K}")
    rng = np.random.default_rng(T * 7 + N + K)
    xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    V, s_vis, s_txt = T // 2 + 3, 0.2, 0.03
    acc_want = orc.gemm_i8_i4_i32(xq, orc.unpack_w4(packed))
    ref, y_want = orc.dequant(acc_want, V, s_vis, s_txt, w_scale)
    wp = mq.w4_prepack(dev(packed))
    ws_bytes = mq.w4a8_workspace_bytes(T, N, K)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    acc = torch.full((T, N), -7, dtype=torch.int32, device="cuda")
    ybuf = torch.full((T, N + 8), 9.0, dtype=torch.float16, device="cuda")
    mq.w4a8_gemm(dev(xq), wp, dev(w_scale), N, V, s_vis, s_txt, out=ybuf[:, :N], acc_out=acc, workspace=ws)
    assert (acc.cpu().numpy() == acc_want).all()
    yb = ybuf.cpu().numpy()
    assert (yb[:, :N].view(np.uint16) == y_want.view(np.uint16)).all()
    assert (yb[:, N:] == 9.0).all()
    y2 = mq.w4a8_gemm(dev(xq), wp, dev(w_scale), N, V, s_vis, s_txt, workspace=ws)     # the path as timed
    assert (y2.cpu().numpy().view(np.uint16) == y_want.view(np.uint16)).all()


def test_gemv_grouped_argument_errors(mq):
    P = 0x1000
    L = mq.lib
    lin = (mq.Linear * 5)()
    for i in range(5):
        lin[i].w_prepacked_dev, lin[i].w_scale_dev, lin[i].y_dev, lin[i].ldy, lin[i].N = P, P, P, 64, 64
    lp = __import__("ctypes").cast(lin, __import__("ctypes").c_void_p)
    f = L.mquant_w4a8_gemv_grouped
    assert f(P, 1, 128, 0, 1.0, 1.0, lp, 5, None) == mq.ERR_UNSUPPORTED          # more than four linears
    assert f(P, 33, 128, 0, 1.0, 1.0, lp, 2, None) == mq.ERR_UNSUPPORTED         # not a decode shape
    assert f(P, 1, 100, 0, 1.0, 1.0, lp, 2, None) == mq.ERR_UNSUPPORTED          # K % 64
    assert f(None, 1, 128, 0, 1.0, 1.0, lp, 2, None) == mq.ERR_NULL
    assert f(P, 1, 128, 0, 1.0, 1.0, None, 2, None) == mq.ERR_NULL
    assert f(P, 1, 128, 2, 1.0, 1.0, lp, 2, None) == mq.ERR_BAD_SHAPE            # n_vis > T
    assert f(P, 1, 128, 0, 0.0, 1.0, lp, 2, None) == mq.ERR_BAD_SHAPE
    lin[1].ldy = 32
    assert f(P, 1, 128, 0, 1.0, 1.0, lp, 2, None) == mq.ERR_BAD_SHAPE            # ldy < N
    lin[1].ldy, lin[1].y_dev = 64, None
    assert f(P, 1, 128, 0, 1.0, 1.0, lp, 2, None) == mq.ERR_NULL
    assert f(P, 0, 128, 0, 1.0, 1.0, lp, 2, None) == mq.OK                       # T == 0
    assert f(P, 1, 128, 0, 1.0, 1.0, lp, 0, None) == mq.OK


def test_empty_inputs_are_noops(mq):
    say("empty inputs")
    e16 = torch.empty((0, 512), dtype=torch.float16, device="cuda")
    assert mq.hadamard_quant_act(e16, 0, 1.0, 1.0, 512).shape == (0, 512)
    assert mq.aifs_permute(e16, torch.empty(0, dtype=torch.int32, device="cuda")).shape == (0, 512)
    wp = mq.w4_prepack(dev(np.zeros((32, 256), dtype=np.uint8)))
    y = mq.w4a8_gemm(torch.empty((0, 512), dtype=torch.int8, device="cuda"), wp,
                     dev(np.ones(32, dtype=np.float16)), 32, 0, 1.0, 1.0)
    assert y.shape == (0, 32)
    torch.cuda.synchronize()


# ------------------------------------------- full-size configurations
#
# configs[1] and configs[2]: the oracle computes EVERY output of all four projections (about
# 8 s and 26 s of host time) and three GPU paths are held against it:
#   - separate entries with acc_out: int8 codes and int32 accumulators bit for bit;
#   - separate entries as timed (acc_out = NULL: the wide LDS-transposed stores, split-K reduce);
#   - the fused prefill entry.
# Both sides evaluate fp16((float(acc) * s_row) * w_scale[n]) with the same two fp32 multiplies,
# so beyond the stated bar (1e-3 of the fp32 reference) the fp16 outputs must be the oracle's
# bit for bit.  Outputs are pre-filled with NaN: an unwritten element cannot pass.

NAN16 = float("nan")


def bands(n, width, rng, extra=()):
    """One seeded index inside every band [b*width, (b+1)*width) of 0..n-1, plus `extra`."""
    picks = set(int(e) for e in extra if 0 <= e < n)
    for b0 in range(0, n, width):
        picks.add(int(rng.integers(b0, min(b0 + width, n))))
    return np.array(sorted(picks), dtype=np.int64)


def assert_y_bits(y_gpu, y_want, what):
    a = y_gpu.view(torch.int16) if isinstance(y_gpu, torch.Tensor) else torch.from_numpy(y_gpu.view(np.int16))
    b = y_want.view(torch.int16) if isinstance(y_want, torch.Tensor) else torch.from_numpy(y_want.view(np.int16))
    if a.is_cuda != b.is_cuda:
        a, b = a.cuda(), b.cuda()
    bad = a != b
    n_bad = int(bad.sum().item())
    assert n_bad == 0, f"{what}: {n_bad} fp16 outputs differ in bits (first {bad.nonzero()[:3].tolist()})"


def gpu_paths(mq, inp, s_vis, s_txt, want_acc):
    """(perm, V, xq, acc or None, y_acc_path or None, y_timed_path, xq_fused, y_fused) on the GPU."""
    T, K, N, B = inp["T"], inp["K"], inp["N"], inp["had_block"]
    perm, inv, V = mq.aifs_build_perm(T, inp["vis_spans"])
    xd, permd = dev(inp["x"]), dev(perm)
    wp = mq.w4_prepack(dev(inp["w_packed"]))
    wsd = dev(inp["w_scale"])
    xq = mq.hadamard_quant_act(xd, V, s_vis, s_txt, B, perm_dev=permd)
    nws = mq.w4a8_workspace_bytes(T, N, K)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
    acc = y_acc = None
    if want_acc:
        acc = torch.full((T, N), -(2 ** 31), dtype=torch.int32, device="cuda")
        y_acc = torch.full((T, N), NAN16, dtype=torch.float16, device="cuda")
        mq.w4a8_gemm(xq, wp, wsd, N, V, s_vis, s_txt, out=y_acc, acc_out=acc, workspace=ws)
    y_timed = torch.full((T, N), NAN16, dtype=torch.float16, device="cuda")
    mq.w4a8_gemm(xq, wp, wsd, N, V, s_vis, s_txt, out=y_timed, workspace=ws)
    wsf = torch.empty(mq.w4a8_linear_prefill_workspace_bytes(T, N, K), dtype=torch.uint8, device="cuda")
    y_fused = torch.full((T, N), NAN16, dtype=torch.float16, device="cuda")
    mq.w4a8_linear_prefill(xd, permd, wp, wsd, N, V, s_vis, s_txt, B, wsf, out=y_fused)
    torch.cuda.synchronize()
    xq_fused = wsf[: T * K].view(torch.int8).reshape(T, K)
    return perm, V, xq, acc, y_acc, y_timed, xq_fused, y_fused


def every_output_case(mq, cfg, proj):
    w = wl.workload(cfg)
    inp = wl.make_linear_inputs(w, proj)
    s_vis, s_txt = scales_from_calib(inp)
    say(f"cfg {cfg} {proj} T={inp['T']} K={inp['K']} N={inp['N']}: oracle on every output")
    o = orc.w4a8_linear(inp["x"], inp["vis_spans"], inp["w_packed"], inp["w_scale"], s_vis, s_txt, w.had_block)
    say(f"cfg {cfg} {proj}: GPU paths")
    perm, V, xq, acc, y_acc, y_timed, xq_fused, y_fused = gpu_paths(mq, inp, s_vis, s_txt, want_acc=True)
    assert (perm == o["perm"]).all() and V == o["V"]
    xq_want = dev(o["xq"])
    assert torch.equal(xq, xq_want), "int8 codes differ (separate entry)"
    assert torch.equal(xq_fused, xq_want), "int8 codes differ (fused entry)"
    del xq_want
    assert torch.equal(acc, dev(o["acc"])), "int32 accumulators differ"
    del acc
    y_want = dev(o["y"])
    for name, y in (("acc_out path", y_acc), ("timed path", y_timed), ("fused entry", y_fused)):
        assert not bool(torch.isnan(y).any().item()), f"{name}: unwritten outputs"
        assert_y_bits(y, y_want, f"cfg{cfg} {proj} {name}")
    # the stated bar, against the fp32 reference (implied by the bit comparison; kept as the contract)
    check_y(y_timed.cpu().numpy(), o["ref"], f"cfg{cfg} {proj} timed path")
    torch.cuda.empty_cache()


@pytest.mark.parametrize("proj", ["qkv", "o", "gate_up", "down"])
def test_config1_prefill_T1280_every_output(mq, proj):
    every_output_case(mq, 1, proj)


@pytest.mark.parametrize("proj", ["qkv", "o", "gate_up", "down"])
def test_config2_prefill_T4096_every_output(mq, proj):
    every_output_case(mq, 2, proj)


@pytest.mark.parametrize("proj", ["qkv", "o", "gate_up", "down"])
def test_config4_72b_T16384_every_32x32_block(mq, proj):
    """configs[4] is 28.8 TOP: the oracle computes one seeded row in every band of 32 rows and
    one seeded column in every band of 32 columns (plus the modality boundary, the span edges and
    the ends), so every 32 x 32 block of the output -- hence every tile of every compiled tile
    shape and every wave's MFMA block -- holds a checked element; the int8 codes are compared on
    every element.  All outputs start as NaN and none may remain."""
    w = wl.workload(4)
    inp = wl.make_linear_inputs(w, proj)
    s_vis, s_txt = scales_from_calib(inp)
    T, N = inp["T"], inp["N"]
    rng = np.random.default_rng(4000 + N)
    _, _, V = orc.aifs_build_perm(T, inp["vis_spans"])
    edges = [0, 1, T - 2, T - 1, V - 2, V - 1, V, V + 1]
    for k in range(1, 4):
        edges += [k * 3072 - 1, k * 3072]                        # where one visual span meets the next
    rows = bands(T, 32, rng, edges)
    cols = bands(N, 32, rng, [0, 1, N - 2, N - 1])
    say(f"cfg 4 {proj} T={T} K={inp['K']} N={N}: oracle on {len(rows)} rows x {len(cols)} columns")
    o = orc.w4a8_linear(inp["x"], inp["vis_spans"], inp["w_packed"], inp["w_scale"], s_vis, s_txt,
                        w.had_block, rows=rows, cols=cols)
    perm, V2, xq, acc, y_acc, y_timed, xq_fused, y_fused = gpu_paths(mq, inp, s_vis, s_txt, want_acc=True)
    assert (perm == o["perm"]).all() and V2 == o["V"] == V
    xq_want = dev(o["xq"])
    assert torch.equal(xq, xq_want) and torch.equal(xq_fused, xq_want), "int8 codes differ"
    del xq_want, xq, xq_fused
    rd, cd = torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()
    assert torch.equal(acc[rd][:, cd], dev(o["acc"])), "int32 accumulators differ"
    del acc
    y_want = dev(o["y"])
    for name, y in (("acc_out path", y_acc), ("timed path", y_timed), ("fused entry", y_fused)):
        assert not bool(torch.isnan(y).any().item()), f"{name}: unwritten outputs"
        assert_y_bits(y[rd][:, cd].contiguous(), y_want, f"cfg4 {proj} {name}")
    check_y(y_timed[rd][:, cd].cpu().numpy(), o["ref"], f"cfg4 {proj} timed path")
    # the three paths agree on every one of the T x N outputs
    assert torch.equal(y_timed.view(torch.int16), y_fused.view(torch.int16))
    assert torch.equal(y_timed.view(torch.int16), y_acc.view(torch.int16))
    torch.cuda.empty_cache()


@pytest.mark.parametrize("cfg,proj", [(1, "qkv"), (1, "o"), (1, "gate_up"), (1, "down"),
                                      (2, "qkv"), (2, "o"), (2, "gate_up"), (2, "down"),
                                      (4, "qkv"), (4, "o"), (4, "gate_up"), (4, "down")])
def test_accumulators_seen_through_the_timed_store_path(mq, cfg, proj):
    """acc_out switches the GEMM to its 2-byte stores, so the path that is timed (wide stores,
    split-K reduce) never shows its int32 sums directly.  Here it shows them through y: with
    s_vis = s_txt = 1 and w_scale = 1 the output is fp16(acc), exact for |acc| <= 2048.  Row i
    carries ONE non-zero code v_i at channel k_i, so acc[i, n] = v_i * wq[n, k_i] (|.| <= 1024)
    for every one of the T x N outputs at the full size of the configuration: a misplaced row,
    column, k-block, tile or split shows as a wrong integer.  k_i steps by 129 channels per row, so
    every 256-row tile meets every 128-channel k-block.  The expected values are the oracle's
    unpacked weights, gathered."""
    w = wl.workload(cfg)
    K, N = w.projections[proj]
    T = w.T
    say(f"one-hot accumulators cfg {cfg} {proj} T={T} K={K} N={N}")
    rng = np.random.default_rng(cfg * 100 + N % 97)
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    wq = orc.unpack_w4(packed)                                   # [N, K] in [-8, 7]
    k_idx = (np.arange(T, dtype=np.int64) * 129 + 7) % K
    v = rng.integers(1, 128, size=T).astype(np.int8) * rng.choice(np.array([-1, 1], dtype=np.int8), size=T)
    v[::5] = -128
    xq = torch.zeros((T, K), dtype=torch.int8, device="cuda")
    xq[torch.arange(T, device="cuda"), torch.from_numpy(k_idx).cuda()] = torch.from_numpy(v).cuda()
    wp = mq.w4_prepack(dev(packed))
    ones = torch.ones(N, dtype=torch.float16, device="cuda")
    nws = mq.w4a8_workspace_bytes(T, N, K)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
    y = torch.full((T, N), NAN16, dtype=torch.float16, device="cuda")
    n_vis = T // 3
    mq.w4a8_gemm(xq, wp, ones, N, n_vis, 1.0, 1.0, out=y, workspace=ws)
    torch.cuda.synchronize()
    # expected: v_i * wq[n, k_i], gathered from the oracle's weights on the device (indexing only)
    wq_d = dev(wq)
    want = (wq_d[:, torch.from_numpy(k_idx).cuda()].t().to(torch.int32)
            * torch.from_numpy(v.astype(np.int32)).cuda()[:, None])
    assert int(want.abs().max().item()) <= 1024
    got = y.to(torch.float32)
    assert not bool(torch.isnan(got).any().item()), "unwritten outputs"
    bad = got != want.to(torch.float32)
    assert int(bad.sum().item()) == 0, f"{int(bad.sum().item())} accumulators wrong, first {bad.nonzero()[:3].tolist()}"
    del y, got, want, wq_d, xq
    torch.cuda.empty_cache()


@pytest.mark.parametrize("T", [1, 4, 16])
def test_config3_decode_full(mq, T):
    """Decode shapes are small enough for the oracle to compute every output."""
    w = wl.workload(3, T)
    for proj in w.projections:
        inp = wl.make_linear_inputs(w, proj)
        s_txt = float(orc.calibrate_static_scale(inp["calib_txt"], w.had_block))
        say(f"cfg 3 {proj} T={T} K={inp['K']} N={inp['N']}")
        o = orc.w4a8_linear(inp["x"], (), inp["w_packed"], inp["w_scale"], s_txt, s_txt, w.had_block)
        g = run_linear_gpu(mq, inp, s_txt, s_txt)
        assert g["V"] == 0
        assert (g["xq"].cpu().numpy() == o["xq"]).all()
        assert (g["acc"].cpu().numpy() == o["acc"]).all()
        check_y(g["y"].cpu().numpy(), o["ref"], f"cfg3 {proj} T={T}")
        assert (g["y"].cpu().numpy().view(np.uint16) == o["y"].view(np.uint16)).all()
        # the path as timed (no acc_out) gives the same bits
        y2 = mq.w4a8_gemm(g["xq"], mq.w4_prepack(dev(inp["w_packed"])), dev(inp["w_scale"]), inp["N"], 0, s_txt, s_txt)
        assert torch.equal(y2, g["y"])


def test_measurement_probes_run(mq):
    """The attainable-peak probes of the benchmark (their own library): launch, finish,
    report their work."""
    from paper_2502_00425_amd import probes
    data = torch.randint(0, 256, (1 << 16,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    assert probes.mfma_i8(10, data, sink) == 10 * 8 * 65536 * 4 * 1024
    assert probes.hbm_read(data, sink) == 1 << 16
    probes.empty(256, 256)
    torch.cuda.synchronize()


@pytest.mark.parametrize("T,N,K,B", [(1, 200, 896, 128), (1, 3584, 3584, 512), (4, 512, 3584, 512),
                                     (3, 3584, 18944, 512), (2, 18944, 3584, 512), (1, 8192, 8192, 128),
                                     (4, 264, 1024, 1)])
def test_fused_decode_linear_equals_separate_entries_and_oracle(mq, T, N, K, B):
    """Rotate + quantize + GEMV + dequant in one launch: same bits as the two-launch path,
    and within 1e-3 of the oracle."""
    say(f"fused decode T={T} N={N} K={K} B={B}")
    rng = np.random.default_rng(T + N + K)
    x = (rng.standard_normal((T, K)) * rng.uniform(0.5, 3.0, size=(T, 1))).astype(np.float16)
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    V = min(T, 1)
    u = orc.hadamard_rotate(x, B)
    s_vis = float(orc.static_scale_from_absmax(np.abs(u).max(), B))
    s_txt = s_vis * 0.8
    o = orc.w4a8_linear(x, [(0, V)], packed, w_scale, s_vis, s_txt, B)
    wp = mq.w4_prepack(dev(packed))
    y = mq.w4a8_linear_decode(dev(x), wp, dev(w_scale), N, V, s_vis, s_txt, B)
    xq = mq.hadamard_quant_act(dev(x), V, s_vis, s_txt, B)
    y2 = mq.w4a8_gemm(xq, wp, dev(w_scale), N, V, s_vis, s_txt)
    assert torch.equal(y, y2)
    check_y(y.cpu().numpy(), o["ref"], "fused decode")


def test_fused_decode_linear_argument_errors(mq):
    x = torch.zeros((5, 512), dtype=torch.float16, device="cuda")
    wp = torch.zeros(mq.w4_prepacked_bytes(32, 512), dtype=torch.uint8, device="cuda")
    ws = torch.ones(32, dtype=torch.float16, device="cuda")
    y = torch.empty((5, 32), dtype=torch.float16, device="cuda")
    call = lambda T, B: mq.lib.mquant_w4a8_linear_decode(x.data_ptr(), 512, wp.data_ptr(), ws.data_ptr(),
                                                          y.data_ptr(), 32, T, 32, 512, 0, 1.0, 1.0, B, None)
    assert call(5, 512) == mq.ERR_UNSUPPORTED
    assert call(1, 256) == mq.ERR_UNSUPPORTED
    assert call(0, 512) == mq.OK
    assert call(1, 512) == mq.OK
    torch.cuda.synchronize()


@pytest.mark.parametrize("T,K,B,Ns", [(1, 3584, 512, (3584, 512, 512)), (4, 3584, 512, (18944, 18944)),
                                      (3, 1024, 128, (40, 0, 200, 72)), (2, 8192, 128, (8192, 1024, 1024)),
                                      (1, 18944, 512, (3584,)), (4, 29568, 128, (264, 96)), (2, 640, 1, (520, 24))])
def test_fused_decode_grouped_equals_the_oracle_per_linear(mq, T, K, B, Ns):
    """Rotate + quantize once, then several linears that share the input, all in one launch
    (q/k/v; gate/up): the fp16 bits of every output of every linear against the oracle's whole
    path, and against the single-linear entry; padding columns untouched.  (4, 29568) is past
    the one-launch kernel's range and runs as one launch per linear."""
    say(f"fused grouped decode T={T} K={K} B={B} Ns={Ns}")
    rng = np.random.default_rng(T * 977 + K + B + len(Ns))
    x = (rng.standard_normal((T, K)) * rng.uniform(0.5, 3.0, size=(T, 1))).astype(np.float16)
    V = min(T, 1)
    u = orc.hadamard_rotate(x, B)
    s_vis = float(orc.static_scale_from_absmax(np.abs(u).max(), B))
    s_txt = s_vis * 0.8
    lin, want = [], []
    for N in Ns:
        packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
        w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
        out = torch.full((T, N + 8), 3.0, dtype=torch.float16, device="cuda")
        wp = mq.w4_prepack(dev(packed)) if N else torch.empty(0, dtype=torch.uint8, device="cuda")
        lin.append((wp, dev(w_scale), N, out[:, :N]))
        want.append(orc.w4a8_linear(x, [(0, V)], packed, w_scale, s_vis, s_txt, B)["y"] if N
                    else np.zeros((T, 0), dtype=np.float16))
    xd = dev(x)
    mq.w4a8_linear_decode_grouped(xd, lin, V, s_vis, s_txt, B)
    torch.cuda.synchronize()
    for (wp, ws, N, out), w in zip(lin, want):
        assert (out.cpu().numpy().view(np.uint16) == w.view(np.uint16)).all(), f"N={N}"
        if N:
            assert torch.equal(mq.w4a8_linear_decode(xd, wp, ws, N, V, s_vis, s_txt, B), out)
        buf = out._base if out._base is not None else out
        assert bool((buf[:, N:] == 3.0).all())


def test_fused_decode_grouped_argument_errors(mq):
    import ctypes
    P = 0x1000
    lin = (mq.Linear * 5)()
    for i in range(5):
        lin[i].w_prepacked_dev, lin[i].w_scale_dev, lin[i].y_dev, lin[i].ldy, lin[i].N = P, P, P, 64, 64
    lp = ctypes.cast(lin, ctypes.c_void_p)
    f = mq.lib.mquant_w4a8_linear_decode_grouped
    assert f(P, 512, 1, 512, 0, 1.0, 1.0, 512, lp, 5, None) == mq.ERR_UNSUPPORTED     # more than four linears
    assert f(P, 512, 5, 512, 0, 1.0, 1.0, 512, lp, 2, None) == mq.ERR_UNSUPPORTED     # more than four rows
    assert f(P, 512, 1, 512, 0, 1.0, 1.0, 256, lp, 2, None) == mq.ERR_UNSUPPORTED     # Hadamard block
    assert f(P, 512, 1, 640, 0, 1.0, 1.0, 512, lp, 2, None) == mq.ERR_UNSUPPORTED     # K % block
    assert f(None, 512, 1, 512, 0, 1.0, 1.0, 512, lp, 2, None) == mq.ERR_NULL
    assert f(P, 512, 1, 512, 0, 1.0, 1.0, 512, None, 2, None) == mq.ERR_NULL
    assert f(P, 512, 1, 512, 2, 1.0, 1.0, 512, lp, 2, None) == mq.ERR_BAD_SHAPE       # n_vis > T
    assert f(P, 512, 1, 512, 0, 1.0, -1.0, 512, lp, 2, None) == mq.ERR_BAD_SHAPE
    assert f(P, 256, 1, 512, 0, 1.0, 1.0, 512, lp, 2, None) == mq.ERR_BAD_SHAPE       # ldx < K
    assert f(P, 516, 1, 512, 0, 1.0, 1.0, 512, lp, 2, None) == mq.ERR_ALIGNMENT       # ldx % 8
    lin[1].ldy = 32
    assert f(P, 512, 1, 512, 0, 1.0, 1.0, 512, lp, 2, None) == mq.ERR_BAD_SHAPE       # ldy < N
    lin[1].ldy, lin[1].y_dev = 64, None
    assert f(P, 512, 1, 512, 0, 1.0, 1.0, 512, lp, 2, None) == mq.ERR_NULL
    assert f(P, 512, 0, 512, 0, 1.0, 1.0, 512, lp, 2, None) == mq.OK                  # T == 0
    assert f(P, 512, 1, 512, 0, 1.0, 1.0, 512, lp, 0, None) == mq.OK


def test_gemm_seeded_shape_sweep(mq):
    """Thirty seeded shapes across the dispatch boundaries (GEMV / both GEMM tiles / row slabs for
    K % 128 != 0, one k-block, single channels, N not a multiple of 8): accumulators bit for bit."""
    rng = np.random.default_rng(2024)
    shapes = [(33, 40, 128), (64, 1, 64), (257, 9, 192), (129, 257, 128), (40, 600, 2048), (300, 31, 1024)]
    while len(shapes) < 30:
        shapes.append((int(rng.integers(1, 301)), int(rng.integers(1, 601)), 64 * int(rng.integers(1, 33))))
    for T, N, K in shapes:
        say(f"sweep T={T} N={N} K={K}")
        xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
        packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
        w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
        V = int(rng.integers(0, T + 1))
        acc_want = orc.gemm_i8_i4_i32(xq, orc.unpack_w4(packed))
        ref, _ = orc.dequant(acc_want, V, 0.07, 0.009, w_scale)
        acc = torch.full((T, N), -7, dtype=torch.int32, device="cuda")
        y = mq.w4a8_gemm(dev(xq), mq.w4_prepack(dev(packed)), dev(w_scale), N, V, 0.07, 0.009, acc_out=acc)
        assert (acc.cpu().numpy() == acc_want).all(), (T, N, K)
        check_y(y.cpu().numpy(), ref, f"sweep {(T, N, K)}")
        y2 = mq.w4a8_gemm(dev(xq), mq.w4_prepack(dev(packed)), dev(w_scale), N, V, 0.07, 0.009)
        check_y(y2.cpu().numpy(), ref, f"sweep, no acc_out {(T, N, K)}")


def test_prefill_step_as_hip_graph_replays_match_plain_launches(mq):
    """The benchmark replays a step (mask remap, row permute, rotate+quant and GEMM per linear)
    from one captured HIP graph.  Every replay must reproduce the plain launches bit for bit,
    with other work and synchronisations between the replays; shapes cover the GEMV, both GEMM
    tiles and the split-K path with its workspace."""
    rng = np.random.default_rng(88)
    T, B = 300, 64
    spans = [(10, 120), (200, 60)]
    perm, _, V = mq.aifs_build_perm(T, spans)
    permd = dev(perm)
    mask = torch.tril(torch.ones((T, T), dtype=torch.uint8, device="cuda"))
    mask_u = torch.empty_like(mask)
    lins = []
    for K, N in [(512, 264), (8192, 264), (1024, 2048)]:
        x = dev((rng.standard_normal((T, K)) * 2).astype(np.float16))
        wp = mq.w4_prepack(dev(rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)))
        w_scale = dev(rng.uniform(0.005, 0.02, size=N).astype(np.float16))
        nws = mq.w4a8_workspace_bytes(T, N, K)
        lins.append({"x": x, "wp": wp, "w_scale": w_scale, "N": N, "K": K,
                     "xq": torch.empty((T, K), dtype=torch.int8, device="cuda"),
                     "y": torch.empty((T, N), dtype=torch.float16, device="cuda"),
                     "ws": torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None})
    assert any(l["ws"] is not None for l in lins), "one shape must take the split-K path"
    x_u = torch.empty_like(lins[0]["x"])

    def step():
        mq.aifs_remap_mask(mask, permd, out=mask_u)
        mq.aifs_permute(lins[0]["x"], permd, out=x_u)
        for l in lins:
            mq.hadamard_quant_act(l["x"], V, 0.05, 0.02, B, perm_dev=permd, out=l["xq"])
            mq.w4a8_gemm(l["xq"], l["wp"], l["w_scale"], l["N"], V, 0.05, 0.02, out=l["y"], workspace=l["ws"])

    outputs = lambda: [mask_u.clone(), x_u.clone()] + [l["y"].clone() for l in lins] + [l["xq"].clone() for l in lins]
    say("graph: plain launches")
    step()
    torch.cuda.synchronize()
    want = outputs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                                           # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        say(f"graph: replay {rep}")
        for t in [mask_u, x_u] + [l["y"] for l in lins] + [l["xq"] for l in lins]:
            t.fill_(3)                                   # eager work of the program between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(outputs(), want):
            assert torch.equal(a, b), f"replay {rep} differs from the plain launches"


@pytest.mark.parametrize("tile,name", [(0, "256x256"), (1, "128x256"), (2, "192x128"), (3, "64x128"), (4, "64x256")])
def test_every_gemm_tile_on_ragged_shapes(mq, tile, name, forced_tile):
    """The dispatcher picks a tile from a cost model; this forces each compiled tile in turn
    (the tuning hook of the library) so that all of them see ragged T and N, one k-block and
    many, whatever the model prefers."""
    forced_tile(mq.TUNE_GEMM_TILE, tile)
    rng = np.random.default_rng(900 + tile)
    for T, N, K in [(33, 40, 128), (200, 136, 384), (450, 520, 1024), (577, 300, 2048)]:
        say(f"tile {name} T={T} N={N} K={K}")
        xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
        packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
        w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
        V = T // 3
        acc_want = orc.gemm_i8_i4_i32(xq, orc.unpack_w4(packed))
        ref, _ = orc.dequant(acc_want, V, 0.07, 0.009, w_scale)
        acc = torch.full((T, N), -7, dtype=torch.int32, device="cuda")
        y = mq.w4a8_gemm(dev(xq), mq.w4_prepack(dev(packed)), dev(w_scale), N, V, 0.07, 0.009, acc_out=acc)
        assert (acc.cpu().numpy() == acc_want).all(), (name, T, N, K)
        check_y(y.cpu().numpy(), ref, f"tile {name} {(T, N, K)}")
        y2 = mq.w4a8_gemm(dev(xq), mq.w4_prepack(dev(packed)), dev(w_scale), N, V, 0.07, 0.009)
        check_y(y2.cpu().numpy(), ref, f"tile {name}, wide stores {(T, N, K)}")


def test_gemm_output_beyond_2_31_elements(mq):
    """T x N > 2^31 outputs (5.3 GB of fp16): every index that addresses y must be 64-bit.
    Rows from both ends and from either side of the 2^31-element mark are compared with the
    oracle; K is one k-block so that the run is short."""
    T, N, K = 70000, 37888, 128
    assert T * N > 2 ** 31
    say(f"gemm T={T} N={N} K={K} (y has {T * N / 2 ** 31:.2f} x 2^31 elements)")
    rng = np.random.default_rng(231)
    V = 40000
    xq = torch.randint(-128, 128, (T, K), dtype=torch.int8, device="cuda",
                       generator=torch.Generator(device="cuda").manual_seed(5))
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    y = torch.full((T, N), 9.0, dtype=torch.float16, device="cuda")
    mq.w4a8_gemm(xq, mq.w4_prepack(dev(packed)), dev(w_scale), N, V, 0.07, 0.009, out=y)
    torch.cuda.synchronize()
    mark = 2 ** 31 // N                                          # the row that holds element 2^31
    rows = np.array([0, 1, 255, 256, V - 1, V, mark - 1, mark, mark + 1, T - 257, T - 2, T - 1])
    got = y[torch.from_numpy(rows).cuda()].cpu().numpy()
    acc_want = orc.gemm_i8_i4_i32(xq[torch.from_numpy(rows).cuda()].cpu().numpy(), orc.unpack_w4(packed))
    for i, r in enumerate(rows):
        ref, _ = orc.dequant(acc_want[i:i + 1], 1 if r < V else 0, 0.07, 0.009, w_scale)
        check_y(got[i:i + 1], ref, f"row {r}")
    # every row was written (9.0 survives nowhere): a device-side reduction over all 2.65e9 outputs
    assert not bool((y == 9.0).all(dim=1).any().item())
    del y
    torch.cuda.empty_cache()


def test_front_end_and_mask_beyond_2_31_elements(mq):
    """The same 64-bit index check for the row permute, the rotate+quant front end (T x K >
    2^31) and the mask remap (T^2 > 2^31), on sampled rows."""
    T, K, B = 70000, 32768, 512
    assert T * K > 2 ** 31
    say(f"front end T={T} K={K}")
    g = torch.Generator(device="cuda").manual_seed(9)
    x = torch.empty((T, K), dtype=torch.float16, device="cuda")
    for r0 in range(0, T, 10000):                            # filled in slabs: no fp32 temporary of 9 GB
        x[r0:r0 + 10000] = torch.randn((min(10000, T - r0), K), device="cuda", generator=g).half()
    spans = [(5, 30000), (40000, 20000)]
    perm, _, V = mq.aifs_build_perm(T, spans)
    permd = dev(perm)
    rows = np.array([0, 1, V - 1, V, 2 ** 31 // K - 1, 2 ** 31 // K, 2 ** 31 // K + 1, T - 2, T - 1])
    rd = torch.from_numpy(rows).cuda()
    src = x[torch.from_numpy(perm[rows].astype(np.int64)).cuda()].cpu().numpy()     # rows of E^u
    xq = mq.hadamard_quant_act(x, V, 0.11, 0.07, B, perm_dev=permd)
    got = xq[rd].cpu().numpy()
    for i, r in enumerate(rows):
        want = orc.msq_quantize(orc.hadamard_rotate(src[i:i + 1], B), 1 if r < V else 0, 0.11, 0.07, B)
        assert (got[i:i + 1] == want).all(), f"codes of row {r}"
    del xq
    xu = mq.aifs_permute(x, permd)
    assert (xu[rd].cpu().numpy().view(np.uint16) == src.view(np.uint16)).all()
    del xu, x
    torch.cuda.empty_cache()

    Tm = 47000
    assert Tm * Tm > 2 ** 31
    say(f"mask remap T={Tm}")
    perm2, _, _ = mq.aifs_build_perm(Tm, [(100, 20000), (30000, 9000)])
    mask = torch.tril(torch.ones((Tm, Tm), dtype=torch.uint8, device="cuda"))
    mu = mq.aifs_remap_mask(mask, dev(perm2))
    del mask
    rows2 = np.array([0, 1, 19999, 20000, 2 ** 31 // Tm, 2 ** 31 // Tm + 1, Tm - 1])
    got2 = mu[torch.from_numpy(rows2).cuda()].cpu().numpy()
    for i, r in enumerate(rows2):
        want = (perm2 <= perm2[r]).astype(np.uint8)          # M^u[i, j] = M[perm[i], perm[j]], M causal
        assert (got2[i] == want).all(), f"mask row {r}"
    del mu
    torch.cuda.empty_cache()
