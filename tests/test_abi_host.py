"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, validates arguments before launching, and
the host-side AIFS index builder agrees with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import mquant_oracle as orc
from paper_2502_00425_amd import binding as mq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "mquant.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mquant_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) >= 12
    assert set(names) == set(mq.EXPORTS)
    raw = ctypes.CDLL(mq.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert mq.version() >= 200
    assert mq.status_string(0) == "ok"
    for code in range(-6, 0):
        assert mq.status_string(code) not in ("ok", "unknown status")
    assert mq.status_string(-99) == "unknown status"


def test_build_perm_matches_oracle():
    cases = [(0, []), (7, [(2, 3)]), (9, []), (9, [(0, 9)]), (64, [(8, 48)]), (23, [(2, 3), (9, 4), (20, 2)]),
             (16, [(0, 0), (3, 2), (5, 0), (5, 4)]), (16384, [(800, 3072), (4704, 3072), (8592, 3072), (12488, 3072)])]
    for T, spans in cases:
        perm, inv, V = mq.aifs_build_perm(T, spans)
        operm, oinv, oV = orc.aifs_build_perm(T, spans)
        assert V == oV
        assert (perm == operm).all() and (inv == oinv).all()


def test_build_perm_errors():
    nv = ctypes.c_int32(0)
    nvp = ctypes.cast(ctypes.byref(nv), ctypes.c_void_p)
    spans = (mq.Span * 2)()
    sp = ctypes.cast(spans, ctypes.c_void_p)
    f = mq.lib.mquant_aifs_build_perm
    assert f(4, None, 0, None, None, None) == mq.ERR_NULL
    assert f(4, None, 1, None, None, nvp) == mq.ERR_NULL
    assert f(-1, None, 0, None, None, nvp) == mq.ERR_BAD_SHAPE
    spans[0].start, spans[0].len = 2, 5
    assert f(4, sp, 1, None, None, nvp) == mq.ERR_BAD_SHAPE          # runs past T
    spans[0].start, spans[0].len = 2, 2
    spans[1].start, spans[1].len = 3, 1
    assert f(8, sp, 2, None, None, nvp) == mq.ERR_BAD_SHAPE          # overlap
    spans[1].start, spans[1].len = 1, 1
    assert f(8, sp, 2, None, None, nvp) == mq.ERR_BAD_SHAPE          # unsorted
    spans[1].start, spans[1].len = 5, -1
    assert f(8, sp, 2, None, None, nvp) == mq.ERR_BAD_SHAPE
    spans[1].start, spans[1].len = 5, 3
    assert f(8, sp, 2, None, None, nvp) == mq.OK and nv.value == 5   # count only


def test_device_entry_points_validate_before_launch():
    """Every call below must be rejected on the host (nothing is launched, so it
    is safe without a GPU).  Fake non-NULL pointers are never dereferenced."""
    P = 0x1000                 # 16-byte (and 256-byte) aligned fake address
    L = mq.lib
    # permute
    Q = 0x2000
    assert L.mquant_aifs_permute(None, 64, Q, 64, P, 4, 64, None) == mq.ERR_NULL
    assert L.mquant_aifs_permute(P, 32, Q, 64, P, 4, 64, None) == mq.ERR_BAD_SHAPE
    assert L.mquant_aifs_permute(P, 64, Q, 64, P, 4, 60, None) == mq.ERR_UNSUPPORTED
    assert L.mquant_aifs_permute(P + 2, 64, Q, 64, P, 4, 64, None) == mq.ERR_ALIGNMENT
    assert L.mquant_aifs_permute(P, 64, Q, 64, P, -1, 64, None) == mq.ERR_BAD_SHAPE
    assert L.mquant_aifs_permute(None, 0, None, 0, None, 0, 64, None) == mq.OK       # empty
    # mask
    assert L.mquant_aifs_remap_mask(None, P, P, 8, None) == mq.ERR_NULL
    assert L.mquant_aifs_remap_mask(None, None, None, 0, None) == mq.OK
    # hadamard + quant
    hq = L.mquant_hadamard_quant_act
    assert hq(None, 512, None, P, 4, 512, 2, 1.0, 1.0, 512, None) == mq.ERR_NULL
    assert hq(P, 512, None, None, 4, 512, 2, 1.0, 1.0, 512, None) == mq.ERR_NULL
    assert hq(P, 512, None, P, 4, 512, 5, 1.0, 1.0, 512, None) == mq.ERR_BAD_SHAPE    # n_vis > T
    assert hq(P, 512, None, P, 4, 512, -1, 1.0, 1.0, 512, None) == mq.ERR_BAD_SHAPE
    assert hq(P, 256, None, P, 4, 512, 2, 1.0, 1.0, 512, None) == mq.ERR_BAD_SHAPE    # ldx < K
    assert hq(P, 512, None, P, 4, 512, 2, 0.0, 1.0, 512, None) == mq.ERR_BAD_SHAPE    # scale <= 0
    assert hq(P, 512, None, P, 4, 512, 2, 1.0, float("inf"), 512, None) == mq.ERR_BAD_SHAPE
    assert hq(P, 512, None, P, 4, 512, 2, 1.0, 1.0, 96, None) == mq.ERR_UNSUPPORTED   # not a power of 2
    assert hq(P, 512, None, P, 4, 512, 2, 1.0, 1.0, 2048, None) == mq.ERR_UNSUPPORTED
    assert hq(P, 768, None, P, 4, 768, 2, 1.0, 1.0, 512, None) == mq.ERR_UNSUPPORTED  # B does not divide K
    assert hq(P, 516, None, P, 4, 516, 2, 1.0, 1.0, 4, None) == mq.ERR_UNSUPPORTED    # K % 8
    assert hq(P + 8, 512, None, P, 4, 512, 2, 1.0, 1.0, 512, None) == mq.ERR_ALIGNMENT
    assert hq(P, 512, None, P, 0, 512, 0, 1.0, 1.0, 512, None) == mq.OK               # T == 0
    assert L.mquant_hadamard_absmax(P, 512, 4, 512, 512, None, None) == mq.ERR_NULL
    # prepack / sizes
    assert L.mquant_w4_prepacked_bytes(512, 512) == 512 * 512 // 2
    assert L.mquant_w4_prepacked_bytes(33, 64) == 2 * 1024                            # N padded to 32
    assert L.mquant_w4_prepacked_bytes(512, 96) == mq.ERR_UNSUPPORTED
    assert L.mquant_w4_prepacked_bytes(-1, 64) == mq.ERR_BAD_SHAPE
    assert L.mquant_w4_prepacked_bytes(32, 131072) == mq.ERR_UNSUPPORTED
    assert L.mquant_w4_prepack(None, P, 32, 64, None) == mq.ERR_NULL
    assert L.mquant_w4_prepack(P, P, 32, 100, None) == mq.ERR_UNSUPPORTED
    assert L.mquant_w4a8_workspace_bytes(16, 512, 512) >= 0
    assert L.mquant_w4a8_workspace_bytes(16, 512, 100) == mq.ERR_UNSUPPORTED
    # gemm
    g = L.mquant_w4a8_gemm
    assert g(None, P, P, P, 512, None, 4, 512, 512, 0, 1.0, 1.0, None, 0, None) == mq.ERR_NULL
    assert g(P, P, P, P, 256, None, 4, 512, 512, 0, 1.0, 1.0, None, 0, None) == mq.ERR_BAD_SHAPE   # ldy < N
    assert g(P, P, P, P, 512, None, 4, 512, 512, 9, 1.0, 1.0, None, 0, None) == mq.ERR_BAD_SHAPE   # n_vis > T
    assert g(P, P, P, P, 512, None, 4, 512, 100, 0, 1.0, 1.0, None, 0, None) == mq.ERR_UNSUPPORTED
    assert g(P, P, P, P, 512, None, 4, 512, 512, 0, -1.0, 1.0, None, 0, None) == mq.ERR_BAD_SHAPE
    assert g(P + 1, P, P, P, 512, None, 4, 512, 512, 0, 1.0, 1.0, None, 0, None) == mq.ERR_ALIGNMENT
    assert g(None, None, None, None, 0, None, 0, 512, 512, 0, 1.0, 1.0, None, 0, None) == mq.OK    # T == 0
    # fused prefill
    f = L.mquant_w4a8_linear_prefill
    need = L.mquant_w4a8_linear_prefill_workspace_bytes(64, 512, 512)
    assert need >= 64 * 512
    assert f(P, 512, None, P, P, P, 512, 64, 512, 512, 48, 1.0, 1.0, 512, None, 0, None) == mq.ERR_WORKSPACE
    assert f(P, 512, None, P, P, P, 512, 64, 512, 512, 48, 1.0, 1.0, 512, P, need - 1, None) == mq.ERR_WORKSPACE
    assert f(None, 512, None, P, P, P, 512, 64, 512, 512, 48, 1.0, 1.0, 512, P, need, None) == mq.ERR_NULL
    assert f(P, 512, None, P, P, P, 512, 64, 512, 512, 48, 1.0, 1.0, 96, P, need, None) == mq.ERR_UNSUPPORTED
    assert f(P, 512, None, P, P, P, 512, 64, 512, 512, 65, 1.0, 1.0, 512, P, need, None) == mq.ERR_BAD_SHAPE
    # weight-only group-128 linear
    assert L.mquant_w4g128_prepacked_bytes(64, 256) == 2 * 4 * 1024 + 2 * 64 * 2
    assert L.mquant_w4g128_prepacked_bytes(33, 256) == 2 * 4 * 1024 + 2 * 64 * 2    # N padded to 32
    assert L.mquant_w4g128_prepacked_bytes(64, 192) == mq.ERR_UNSUPPORTED
    assert L.mquant_w4g128_prepacked_bytes(-1, 128) == mq.ERR_BAD_SHAPE
    assert L.mquant_w4g128_prepack(None, P, P, 32, 128, None) == mq.ERR_NULL
    assert L.mquant_w4g128_prepack(P, None, P, 32, 128, None) == mq.ERR_NULL
    assert L.mquant_w4g128_prepack(P, P, P + 8, 32, 128, None) == mq.ERR_ALIGNMENT
    assert L.mquant_w4g128_prepack(P, P, P, 32, 64, None) == mq.ERR_UNSUPPORTED
    assert L.mquant_w4g128_prepack(None, None, None, 0, 128, None) == mq.OK
    wo = L.mquant_w4g128_gemm
    assert wo(None, 256, P, P, 64, 4, 64, 256, None) == mq.ERR_NULL
    assert wo(P, 128, P, P, 64, 4, 64, 256, None) == mq.ERR_BAD_SHAPE               # ldx < K
    assert wo(P, 256, P, P, 32, 4, 64, 256, None) == mq.ERR_BAD_SHAPE               # ldy < N
    assert wo(P, 256, P, P, 64, 4, 64, 192, None) == mq.ERR_UNSUPPORTED             # K % 128
    assert wo(P, 260, P, P, 64, 4, 64, 256, None) == mq.ERR_ALIGNMENT               # ldx % 8
    assert wo(P + 2, 256, P, P, 64, 4, 64, 256, None) == mq.ERR_ALIGNMENT
    assert wo(None, 256, None, None, 64, 0, 64, 256, None) == mq.OK                 # T == 0


def test_widened_entry_points_validate_before_launch():
    """Same for the entry points beyond the W4A8 linear: rejected on the host, nothing launched."""
    P = 0x1000
    L = mq.lib
    qb = L.mquant_hadamard_quant_act_bits
    assert qb(P, 512, None, P, 4, 512, 2, 1.0, 1.0, 512, 9, None) == mq.ERR_UNSUPPORTED   # bits > 8
    assert qb(P, 512, None, P, 4, 512, 2, 1.0, 1.0, 512, 1, None) == mq.ERR_UNSUPPORTED   # bits < 2
    assert qb(None, 512, None, P, 4, 512, 2, 1.0, 1.0, 512, 4, None) == mq.ERR_NULL
    dq = L.mquant_hadamard_dynquant_act
    assert dq(P, 512, None, P, None, 4, 512, 512, None) == mq.ERR_NULL                    # no scale output
    assert dq(P, 256, None, P, P, 4, 512, 512, None) == mq.ERR_BAD_SHAPE
    assert dq(P, 512, None, P, P, 4, 512, 96, None) == mq.ERR_UNSUPPORTED
    assert dq(P, 65536, None, P, P, 4, 65536, 512, None) == mq.ERR_UNSUPPORTED            # row too long
    assert dq(None, 512, None, None, None, 0, 512, 512, None) == mq.OK
    rs = L.mquant_w4a8_gemm_rowscale
    assert rs(P, P, P, None, P, 512, None, 4, 512, 512, None, 0, None) == mq.ERR_NULL
    assert rs(P, P, P, P, P, 256, None, 4, 512, 512, None, 0, None) == mq.ERR_BAD_SHAPE
    assert rs(P, P, P, P + 2, P, 512, None, 4, 512, 512, None, 0, None) == mq.ERR_ALIGNMENT
    idx = (ctypes.c_int32 * 2)(0, 512)
    idx_out = (ctypes.c_int32 * 2)(0, 5120)
    sc = (ctypes.c_float * 2)(0.1, 0.2)
    sc_nan = (ctypes.c_float * 2)(0.1, float("nan"))
    rms = L.mquant_w4a8_gemm_rms
    assert rms(P, P, P, P, 512, None, 4, 512, 1024, 0, 1.0, 1.0, idx, None, sc, 2, None, 0, None) == mq.ERR_NULL
    assert rms(P, P, P, P, 512, None, 4, 512, 1024, 0, 1.0, 1.0, idx_out, P, sc, 2, None, 0, None) == mq.ERR_BAD_SHAPE
    assert rms(P, P, P, P, 512, None, 4, 512, 1024, 0, 1.0, 1.0, idx, P, sc_nan, 2, None, 0, None) == mq.ERR_BAD_SHAPE
    assert rms(P, P, P, P, 512, None, 4, 512, 1024, 0, 1.0, 1.0, idx, P, sc, 65, None, 0, None) == mq.ERR_BAD_SHAPE
    assert rms(P, P, P, P, 512, None, 4, 512, 1024, 0, 1.0, 1.0, idx, P, sc, -1, None, 0, None) == mq.ERR_BAD_SHAPE
    dec = L.mquant_w4a8_linear_decode
    assert dec(P, 512, P, P, P, 512, 5, 512, 512, 0, 1.0, 1.0, 512, None) == mq.ERR_UNSUPPORTED   # T > 4
    assert dec(P, 512, P, P, P, 512, 1, 512, 512, 0, 1.0, 1.0, 256, None) == mq.ERR_UNSUPPORTED   # block size
    assert dec(None, 512, P, P, P, 512, 1, 512, 512, 0, 1.0, 1.0, 512, None) == mq.ERR_NULL
    assert dec(P, 512, P, P, P, 512, 1, 512, 512, 2, 1.0, 1.0, 512, None) == mq.ERR_BAD_SHAPE     # n_vis > T
    assert dec(None, 512, None, None, None, 512, 0, 512, 512, 0, 1.0, 1.0, 512, None) == mq.OK
    rope = L.mquant_rope_apply
    assert rope(None, 1024, P, 4, 8, 128, 10000.0, None) == mq.ERR_NULL
    assert rope(P, 1024, P, 4, 8, 96, 10000.0, None) == mq.ERR_UNSUPPORTED                # head_dim
    assert rope(P, 512, P, 4, 8, 128, 10000.0, None) == mq.ERR_BAD_SHAPE                  # ldx < heads * dim
    assert rope(P, 1024, P, 4, 8, 128, 0.0, None) == mq.ERR_BAD_SHAPE
    assert rope(None, 1024, None, 0, 8, 128, 10000.0, None) == mq.OK
    att = L.mquant_aifs_attention
    need = L.mquant_aifs_attention_workspace_bytes(64, 4, 128)
    assert need >= 64 * 4 * 128 * 2
    assert att(P, 3584, P, 512, P, 512, P, 3584, P, 64, 28, 4, 128, P, need - 1, None) == mq.ERR_WORKSPACE
    assert att(P, 3584, P, 512, P, 512, P, 3584, P, 64, 28, 4, 64, P, need, None) == mq.ERR_UNSUPPORTED
    assert att(P, 3584, P, 512, P, 512, P, 3584, P, 64, 28, 5, 128, P, need, None) == mq.ERR_BAD_SHAPE   # 28 % 5
    assert att(None, 3584, P, 512, P, 512, P, 3584, P, 64, 28, 4, 128, P, need, None) == mq.ERR_NULL
    assert att(P, 3580, P, 512, P, 512, P, 3584, P, 64, 28, 4, 128, P, need, None) == mq.ERR_BAD_SHAPE   # ldq < heads * dim
    assert att(None, 3584, None, 512, None, 512, None, 3584, None, 0, 28, 4, 128, None, 0, None) == mq.OK


def test_static_scale_is_computed_by_the_library_and_matches_the_oracle():
    """Eq. (2)'s scale lives behind the C ABI (a host function), not in the Python package."""
    import paper_2502_00425_amd as pkg
    assert not hasattr(pkg, "static_scale_from_absmax")
    for absmax, B in [(1234.5, 512), (7.0, 128), (1e-3, 1), (65504.0 * 512, 512), (0.0, 16)]:
        assert np.float32(mq.static_scale_from_absmax(absmax, B)) == orc.static_scale_from_absmax(absmax, B)
        for bits in (2, 4, 8):
            assert (np.float32(mq.static_scale_from_absmax(absmax, B, bits))
                    == orc.static_scale_from_absmax_bits(absmax, B, bits))
    # a hand case: absmax of the unnormalised rotation 254 * sqrt(16) -> s = 254 / 127 = 2
    assert mq.static_scale_from_absmax(254.0 * 4.0, 16) == 2.0
    out = ctypes.c_float(0.0)
    po = ctypes.cast(ctypes.byref(out), ctypes.c_void_p)
    f = mq.lib.mquant_static_scale_from_absmax
    assert f(1.0, 512, 8, None) == mq.ERR_NULL
    assert f(1.0, 96, 8, po) == mq.ERR_UNSUPPORTED
    assert f(1.0, 2048, 8, po) == mq.ERR_UNSUPPORTED
    assert f(1.0, 512, 9, po) == mq.ERR_UNSUPPORTED
    assert f(1.0, 512, 1, po) == mq.ERR_UNSUPPORTED
    assert f(-1.0, 512, 8, po) == mq.ERR_BAD_SHAPE
    assert f(float("nan"), 512, 8, po) == mq.ERR_BAD_SHAPE
    assert f(float("inf"), 512, 8, po) == mq.ERR_BAD_SHAPE


def test_tune_hook_validates_and_resets():
    f = mq.lib.mquant_tune_set
    assert f(99, 0) == mq.ERR_BAD_SHAPE
    assert f(mq.TUNE_GEMM_TILE, 5) == mq.ERR_BAD_SHAPE
    assert f(mq.TUNE_GEMM_TILE, -2) == mq.ERR_BAD_SHAPE
    assert f(mq.TUNE_GEMM_NOSPLIT, 2) == mq.ERR_BAD_SHAPE
    assert f(mq.TUNE_G128_TILE, 2) == mq.ERR_BAD_SHAPE
    assert f(mq.TUNE_GEMV_VARIANT, 4) == mq.ERR_BAD_SHAPE
    # NOSPLIT changes the workspace a long-K, few-tile shape asks for; setting it back restores it
    base = mq.w4a8_workspace_bytes(300, 520, 8192)
    assert base > 0
    for key, val, back in ((mq.TUNE_GEMM_TILE, 2, -1), (mq.TUNE_GEMM_NOSPLIT, 1, 0), (mq.TUNE_G128_TILE, 1, -1)):
        assert f(key, val) == mq.OK
        assert f(key, back) == mq.OK
    assert mq.w4a8_workspace_bytes(300, 520, 8192) == base


def test_loaded_library_was_built_from_the_sources_in_the_tree():
    """A stale binary must not pass for the code under test: the hash compiled into the
    library equals the hash of the sources, headers and flags now in the tree."""
    from paper_2502_00425_amd import build as hip_build
    assert mq.build_id() == hip_build.source_hash()
    assert not hip_build.is_stale()


def test_probe_library_is_separate_from_the_product_abi():
    raw = ctypes.CDLL(mq.LIB_PATH)
    for n in ("mquant_probe_mfma_i8", "mquant_probe_hbm_read", "mqprobe_mfma_i8", "mqprobe_empty"):
        assert not hasattr(raw, n), n
    from paper_2502_00425_amd import probes
    for n in probes.EXPORTS:
        assert hasattr(probes.lib, n), n
    assert probes.lib.mqprobe_mfma_i8_ops(10) == 10 * 8 * 65536 * 4 * 1024
    assert probes.lib.mqprobe_mfma_i8_ops(-1) == mq.ERR_BAD_SHAPE
    assert probes.lib.mqprobe_mfma_i8(-1, 0x1000, 1 << 16, 0x1000, None) == mq.ERR_BAD_SHAPE
    assert probes.lib.mqprobe_hbm_read(None, 16, 0x1000, None) == mq.ERR_NULL
    assert probes.lib.mqprobe_empty(0, 256, None) == mq.ERR_BAD_SHAPE
    assert probes.lib.mqprobe_empty(1, 100, None) == mq.ERR_BAD_SHAPE


def test_binding_rejects_operands_the_abi_cannot_address():
    """The ABI has no leading dimension for xq, the weights, the index vector or the mask:
    the binding refuses non-contiguous tensors there instead of passing a wrong pointer."""
    torch = pytest.importorskip("torch")
    xq = torch.zeros((8, 256), dtype=torch.int8)[:, :128]
    wp = torch.zeros(mq.w4_prepacked_bytes(32, 128), dtype=torch.uint8)
    ws = torch.ones(32, dtype=torch.float16)
    with pytest.raises(mq.MQuantError):
        mq.w4a8_gemm(xq, wp, ws, 32, 0, 1.0, 1.0, out=torch.zeros((8, 32), dtype=torch.float16))
    x = torch.zeros((8, 64), dtype=torch.float16)
    with pytest.raises(mq.MQuantError):
        mq.aifs_permute(x.t(), torch.zeros(64, dtype=torch.int32))
    with pytest.raises(mq.MQuantError):
        mq.aifs_remap_mask(torch.zeros((8, 16), dtype=torch.uint8)[:, :8], torch.zeros(8, dtype=torch.int32))
    # in-place gather is rejected by the library itself
    P = 0x1000
    assert mq.lib.mquant_aifs_permute(P, 64, P, 64, P, 4, 64, None) == mq.ERR_BAD_SHAPE


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 (and as C++) on its own."""
    import shutil
    import subprocess
    hdr = os.path.join(ROOT, "include", "mquant.h")
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    for cmd in (["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr],
                ["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", hdr]):
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout
