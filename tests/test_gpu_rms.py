"""GPU parity of the Rotation Magnitude Suppression run-time path
(mquant_w4a8_gemm_rms) against the oracle: main accumulators bit for bit, the
fp16 result within 1e-3 of the oracle's fp32 value (relative to the magnitude
of the terms that are added, since main and split parts may cancel)."""
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
    print(f"[parity-rms] {msg}", flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def pack_int4(wq):
    """[N, K] int8 in [-8,7] -> canonical [N, K/2] bytes, even k in the low nibble."""
    u = (wq.astype(np.int16) & 0xF).astype(np.uint8)
    return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)


def make_case(rng, T, N, K, B, n_split):
    xq = rng.integers(-128, 128, size=(T, K), dtype=np.int8)
    wq = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    blocks = rng.choice(K // B, size=n_split, replace=False)
    idx = np.sort(blocks).astype(np.int32) * B                  # first row of some Hadamard blocks
    wq[:, idx] = 0                                              # zeroed in the main weight
    wsplit = rng.integers(-8, 8, size=(n_split, N), dtype=np.int8)
    ssplit = rng.uniform(0.05, 0.4, size=n_split).astype(np.float32)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    return xq, wq, idx, wsplit, ssplit, w_scale


def check(y_gpu, ref, mag, what):
    y = y_gpu.astype(np.float32)
    tol = 1e-3 * np.maximum(mag, 2.0 ** -14)
    bad = np.abs(y - ref) > tol
    assert not bad.any(), f"{what}: {int(bad.sum())} outputs beyond 1e-3 (first {np.argwhere(bad)[:3].tolist()})"


@pytest.mark.parametrize("T,N,K,B,n_split", [
    (1, 200, 832, 64, 1), (16, 200, 832, 64, 3),            # GEMV
    (75, 300, 1024, 512, 2),                                 # short prompt: GEMV pass of 64 rows + one of 11
    (140, 300, 1024, 512, 2),                                # GEMM, narrow stores
    (260, 264, 3584, 512, 1), (260, 520, 3584, 512, 7),      # GEMM, wide stores
    (300, 520, 8192, 128, 5),                                # split-K + reduce kernel
    (40, 64, 18944, 512, 37),                                # every block flagged
    (33, 96, 8192, 128, 64),                                 # the most the entry point takes
])
def test_rms_gemm_matches_oracle(mq, T, N, K, B, n_split):
    say(f"rms T={T} N={N} K={K} splits={n_split}")
    rng = np.random.default_rng(T + N + K + n_split)
    xq, wq, idx, wsplit, ssplit, w_scale = make_case(rng, T, N, K, B, n_split)
    V, s_vis, s_txt = T // 3, 0.11, 0.004
    acc_want = orc.gemm_i8_i4_i32(xq, wq)
    ref, _ = orc.dequant_rms(acc_want, xq, V, s_vis, s_txt, w_scale, idx, wsplit, ssplit)
    main, _ = orc.dequant(acc_want, V, s_vis, s_txt, w_scale)
    mag = np.abs(main) + np.abs(ref - main)
    wp = mq.w4_prepack(dev(pack_int4(wq)))
    args = (dev(xq), wp, dev(w_scale), N, V, s_vis, s_txt, idx, dev(wsplit), ssplit)
    acc = torch.empty((T, N), dtype=torch.int32, device="cuda")
    y = mq.w4a8_gemm_rms(*args, acc_out=acc)
    assert (acc.cpu().numpy() == acc_want).all()
    check(y.cpu().numpy(), ref, mag, "rms with acc_out")
    y2 = mq.w4a8_gemm_rms(*args)
    check(y2.cpu().numpy(), ref, mag, "rms")


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
def test_rms_on_every_gemm_tile(mq, tile):
    """The split epilogue on each compiled GEMM tile (forced through the tuning hook; a forced
    tile also keeps short prompts on the GEMM): ragged rows and columns, narrow and wide stores."""
    rng = np.random.default_rng(70 + tile)
    mq.tune_set(mq.TUNE_GEMM_TILE, tile)
    try:
        for T, N, K, B, n_split in [(75, 300, 1024, 512, 2), (200, 264, 640, 128, 5)]:
            say(f"rms tile {tile} T={T} N={N} K={K}")
            xq, wq, idx, wsplit, ssplit, w_scale = make_case(rng, T, N, K, B, n_split)
            V, s_vis, s_txt = T // 3, 0.11, 0.004
            acc_want = orc.gemm_i8_i4_i32(xq, wq)
            ref, _ = orc.dequant_rms(acc_want, xq, V, s_vis, s_txt, w_scale, idx, wsplit, ssplit)
            main, _ = orc.dequant(acc_want, V, s_vis, s_txt, w_scale)
            mag = np.abs(main) + np.abs(ref - main)
            wp = mq.w4_prepack(dev(pack_int4(wq)))
            args = (dev(xq), wp, dev(w_scale), N, V, s_vis, s_txt, idx, dev(wsplit), ssplit)
            acc = torch.empty((T, N), dtype=torch.int32, device="cuda")
            y = mq.w4a8_gemm_rms(*args, acc_out=acc)
            assert (acc.cpu().numpy() == acc_want).all()
            check(y.cpu().numpy(), ref, mag, f"rms tile {tile} with acc_out")
            check(mq.w4a8_gemm_rms(*args).cpu().numpy(), ref, mag, f"rms tile {tile}")
    finally:
        mq.tune_set(mq.TUNE_GEMM_TILE, -1)


def test_rms_without_split_channels_equals_plain_gemm(mq):
    rng = np.random.default_rng(9)
    T, N, K = 70, 264, 1024
    xq, wq, idx, wsplit, ssplit, w_scale = make_case(rng, T, N, K, 128, 1)
    wp = mq.w4_prepack(dev(pack_int4(wq)))
    a = mq.w4a8_gemm(dev(xq), wp, dev(w_scale), N, 20, 0.1, 0.01)
    b = mq.w4a8_gemm_rms(dev(xq), wp, dev(w_scale), N, 20, 0.1, 0.01, None, None, None)
    assert torch.equal(a, b)


def test_rms_argument_errors(mq):
    xq = torch.zeros((4, 128), dtype=torch.int8, device="cuda")
    wp = torch.zeros(mq.w4_prepacked_bytes(32, 128), dtype=torch.uint8, device="cuda")
    ws = torch.ones(32, dtype=torch.float16, device="cuda")
    y = torch.empty((4, 32), dtype=torch.float16, device="cuda")
    call = lambda idx, w, s, n: mq.lib.mquant_w4a8_gemm_rms(
        xq.data_ptr(), wp.data_ptr(), ws.data_ptr(), y.data_ptr(), 32, None, 4, 32, 128, 0, 1.0, 1.0,
        idx, w, s, n, None, 0, None)
    import ctypes
    one_idx = (ctypes.c_int32 * 1)(500)
    one_sc = (ctypes.c_float * 1)(1.0)
    sw = torch.zeros((1, 32), dtype=torch.int8, device="cuda")
    assert call(ctypes.addressof(one_idx), sw.data_ptr(), ctypes.addressof(one_sc), 1) == mq.ERR_BAD_SHAPE
    assert call(None, None, None, 1) == mq.ERR_NULL
    assert call(None, None, None, -1) == mq.ERR_BAD_SHAPE
    assert call(None, None, None, 1000) == mq.ERR_BAD_SHAPE
    assert call(None, None, None, 0) == mq.OK
    torch.cuda.synchronize()


def test_rms_end_to_end_from_float_weights(mq):
    """Offline steps on the CPU (rotate the weight, flag by the mean condition, split, quantize),
    run-time path on the GPU: the result must equal the oracle's and must be closer to x W than
    the unsplit int4 linear is."""
    say("rms end to end")
    rng = np.random.default_rng(12)
    B, K, N, T = 128, 1024, 96, 48
    W = rng.standard_normal((K, N)) * 0.05 + rng.uniform(0.3, 0.6, size=(1, N))
    R = orc.rotate_weight(W, B)
    flagged = orc.rms_flag_channels(W, B)
    assert len(flagged) == K // B
    wq, w_scale, wsplit, ssplit = orc.rms_split_weight(R, flagged)
    x = rng.standard_normal((T, K)).astype(np.float16)
    u = orc.hadamard_rotate(x, B)
    s_act = float(orc.static_scale_from_absmax(np.abs(u).max(), B))
    xq_want = orc.msq_quantize(u, 0, s_act, s_act, B)
    xq = mq.hadamard_quant_act(dev(x), 0, s_act, s_act, B)
    assert (xq.cpu().numpy() == xq_want).all()
    y = mq.w4a8_gemm_rms(xq, mq.w4_prepack(dev(pack_int4(wq))), dev(w_scale), N, 0, s_act, s_act,
                         flagged, dev(wsplit), ssplit).cpu().numpy().astype(np.float64)
    ref, _ = orc.dequant_rms(orc.gemm_i8_i4_i32(xq_want, wq), xq_want, 0, s_act, s_act, w_scale,
                             flagged, wsplit, ssplit)
    assert np.allclose(y, ref, rtol=2e-3, atol=2e-3)
    wq0, s0 = orc.quantize_weight_rows_int4(R.T)
    y0 = mq.w4a8_gemm(xq, mq.w4_prepack(dev(pack_int4(wq0))), dev(s0), N, 0, s_act, s_act).cpu().numpy()
    want = x.astype(np.float64) @ W
    assert np.abs(y - want).mean() < 0.6 * np.abs(y0 - want).mean()


@pytest.mark.parametrize("n_split", [1, 37])
def test_rms_full_size_down_projection_sampled(mq, n_split):
    """configs[1] down projection (1280 x 18944 x 3584, the split-K launch bench.py times) with
    one flagged channel and with one per Hadamard block; sampled rows x channels."""
    say(f"rms full-size down splits={n_split}")
    rng = np.random.default_rng(100 + n_split)
    T, K, N, B = 1280, 18944, 3584, 512
    xq, wq, idx, wsplit, ssplit, w_scale = make_case(rng, T, N, K, B, n_split)
    V, s_vis, s_txt = 1024, 0.11, 0.004
    rows = np.unique(np.r_[0, 1, 255, 256, V - 1, V, T - 1, rng.choice(T, 24, replace=False)])
    cols = np.unique(np.r_[0, 1, 31, 32, 255, 256, N - 1, rng.choice(N, 96, replace=False)])
    acc_want = orc.gemm_i8_i4_i32(xq[rows], wq[cols])
    ref = np.empty(acc_want.shape, dtype=np.float32)
    main = np.empty_like(ref)
    for sel, v_count in ((rows < V, None), (rows >= V, 0)):
        if not sel.any():
            continue
        vv = int(sel.sum()) if v_count is None else 0
        ref[sel], _ = orc.dequant_rms(acc_want[sel], xq[rows][sel], vv, s_vis, s_txt, w_scale[cols], idx,
                                      wsplit[:, cols], ssplit)
        main[sel], _ = orc.dequant(acc_want[sel], vv, s_vis, s_txt, w_scale[cols])
    mag = np.abs(main) + np.abs(ref - main)
    y = mq.w4a8_gemm_rms(dev(xq), mq.w4_prepack(dev(pack_int4(wq))), dev(w_scale), N, V, s_vis, s_txt,
                         idx, dev(wsplit), ssplit)
    check(y.cpu().numpy()[np.ix_(rows, cols)], ref, mag, f"full-size down, {n_split} split channels")
