"""The fused prefill entry that allocates nothing (`mquant_w4a8_linear_prefill_static`): its
workspace is a device array inside the library.  Called through the C ABI and compared bit for
bit with the existing entry point on a caller workspace, on two calls in a row, the second one
smaller (stale contents of the shared array from the first call must not leak into it)."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def mq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2502_00425_amd import binding
    return binding


def say(msg):
    print(f"[no-alloc] {msg}", flush=True)
    sys.stdout.flush()


def make_case(mq, seed, T, N, K, spans):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((T, K)) * 3).astype(np.float16)
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    w_scale = rng.uniform(0.005, 0.02, size=N).astype(np.float16)
    perm, _, V = mq.aifs_build_perm(T, spans)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return {"x": d(x), "wp": mq.w4_prepack(d(packed)), "w_scale": d(w_scale), "perm": d(perm), "V": V,
            "T": T, "N": N, "K": K}


def test_static_scratch_entry_matches_the_workspace_entry_twice_in_a_row(mq):
    B = 64
    # (300, 520, 8192): split-K with partial sums in the scratch, ragged T and N.
    # (130, 264, 8192): a smaller problem right after it, same path.
    # (64, 96, 512): no split-K, only the int8 activations go through the scratch.
    cases = [make_case(mq, 1, 300, 520, 8192, [(10, 120), (200, 60)]),
             make_case(mq, 2, 130, 264, 8192, [(3, 40)]),
             make_case(mq, 3, 64, 96, 512, [(8, 48)])]
    assert mq.w4a8_workspace_bytes(300, 520, 8192) > 0 and mq.w4a8_workspace_bytes(130, 264, 8192) > 0
    want = []
    for c in cases:
        need = mq.w4a8_linear_prefill_workspace_bytes(c["T"], c["N"], c["K"])
        assert 0 < need <= mq.STATIC_SCRATCH_BYTES
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        want.append(mq.w4a8_linear_prefill(c["x"], c["perm"], c["wp"], c["w_scale"], c["N"], c["V"],
                                           0.21, 0.034, B, ws))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for rep in range(2):
        for c, w in zip(cases, want):
            say(f"rep {rep} T={c['T']} N={c['N']} K={c['K']}")
            y = torch.full((c["T"], c["N"] + 8), 5.0, dtype=torch.float16, device="cuda")
            st = mq.lib.mquant_w4a8_linear_prefill_static(
                c["x"].data_ptr(), c["K"], c["perm"].data_ptr(), c["wp"].data_ptr(), c["w_scale"].data_ptr(),
                y.data_ptr(), c["N"] + 8, c["T"], c["N"], c["K"], c["V"], 0.21, 0.034, B,
                torch.cuda.current_stream().cuda_stream or None)
            assert st == mq.OK
            torch.cuda.synchronize()
            assert torch.equal(y[:, :c["N"]], w), "differs from the entry point with a caller workspace"
            assert bool((y[:, c["N"]:] == 5.0).all())
            del y
    assert torch.cuda.memory_allocated() == before


def test_static_scratch_entry_rejects_what_does_not_fit(mq):
    P, Q = 0x1000, 0x2000
    f = mq.lib.mquant_w4a8_linear_prefill_static
    # the 72B-class down projection at T = 16384 needs 462 MiB of int8 activations alone
    assert mq.w4a8_linear_prefill_workspace_bytes(16384, 8192, 29568) > mq.STATIC_SCRATCH_BYTES
    assert f(P, 29568, None, P, P, Q, 8192, 16384, 8192, 29568, 12288, 1.0, 1.0, 128, None) == mq.ERR_WORKSPACE
    # argument errors of the existing entry point come through unchanged, nothing is launched
    assert f(None, 512, None, P, P, Q, 512, 64, 512, 512, 48, 1.0, 1.0, 512, None) == mq.ERR_NULL
    assert f(P, 512, None, P, P, Q, 512, 64, 512, 512, 65, 1.0, 1.0, 512, None) == mq.ERR_BAD_SHAPE
    assert f(P, 512, None, P, P, Q, 512, 64, 512, 512, 48, 1.0, 1.0, 96, None) == mq.ERR_UNSUPPORTED
    assert f(P, 512, None, P, P, Q, 512, 0, 512, 512, 0, 1.0, 1.0, 512, None) == mq.OK      # T == 0
    torch.cuda.synchronize()
