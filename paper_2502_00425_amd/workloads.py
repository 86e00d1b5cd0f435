"""Seeded synthetic inputs for the W4A8 MSQ linear path.

This module only draws random numbers and lays out shapes; it contains none of
the method's arithmetic (no rotation, no quantization, no packing logic, no
scale calibration) and is the single source of inputs for both the CPU oracle
and the HIP path.  The recipe stands in for MLLM activations and GPTQ int4
weights: text rows are N(0,1); visual rows are N(0,20^2) with four outlier
channels fifty times larger (the paper's Fig. 1(b) observation that visual
activations are far wider than text ones); weights are uniform int4 drawn as
uniform random bytes (each nibble is then uniform in [-8,7] under 4-bit two's
complement); per-output-channel weight scales are fp16 U(0.005, 0.02).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

OUTLIER_CHANNELS = (3, 97, 200, 411)
OUTLIER_GAIN = 50.0
VIS_SIGMA = 20.0
CALIB_ROWS = 256


@dataclass(frozen=True)
class Workload:
    """One configuration: a token layout plus a set of (K, N) projections."""
    cfg: int
    name: str
    T: int
    vis_spans: Tuple[Tuple[int, int], ...]       # 0-based (start, length)
    had_block: int
    projections: Dict[str, Tuple[int, int]] = field(default_factory=dict)  # name -> (K, N)

    @property
    def n_vis(self) -> int:
        return sum(l for _, l in self.vis_spans)


_P7B_FUSED = {"qkv": (3584, 4608), "o": (3584, 3584),
              "gate_up": (3584, 37888), "down": (18944, 3584)}
_P7B_DECODE = {"q": (3584, 3584), "k": (3584, 512), "v": (3584, 512), "o": (3584, 3584),
               "gate": (3584, 18944), "up": (3584, 18944), "down": (18944, 3584)}
_P72B = {"qkv": (8192, 10240), "o": (8192, 8192),
         "gate_up": (8192, 59136), "down": (29568, 8192)}


def _c4_spans() -> Tuple[Tuple[int, int], ...]:
    text = (800, 832, 816, 824, 824)          # sums to 4096
    spans, pos = [], 0
    for i in range(4):
        pos += text[i]
        spans.append((pos, 3072))
        pos += 3072
    assert pos + text[4] == 16384
    return tuple(spans)


def workload(cfg: int, T: int | None = None) -> Workload:
    """The five configurations of the benchmark (cfg 3 takes T in {1,4,16})."""
    if cfg == 0:
        return Workload(0, "c0_single_512", 64, ((8, 48),), 512, {"lin": (512, 512)})
    if cfg == 1:
        return Workload(1, "c1_7b_prefill_T1280", 1280, ((16, 1024),), 512, dict(_P7B_FUSED))
    if cfg == 2:
        return Workload(2, "c2_7b_prefill_T4096", 4096, ((256, 3584),), 512, dict(_P7B_FUSED))
    if cfg == 3:
        t = 1 if T is None else T
        return Workload(3, f"c3_7b_decode_T{t}", t, (), 512, dict(_P7B_DECODE))
    if cfg == 4:
        return Workload(4, "c4_72b_prefill_T16384", 16384, _c4_spans(), 128, dict(_P72B))
    raise ValueError("cfg must be 0..4")


def seed_for(cfg: int, proj_index: int) -> int:
    return 1000 * cfg + proj_index


def _streams(seed: int):
    return [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(5)]


def _is_visual(T: int, spans) -> np.ndarray:
    m = np.zeros(T, dtype=bool)
    for s, l in spans:
        m[s:s + l] = True
    return m


def draw_activations(rng, T: int, K: int, is_vis: np.ndarray) -> np.ndarray:
    """fp16 [T, K]: text rows N(0,1); visual rows N(0,20^2), outlier channels x50."""
    x = rng.standard_normal((T, K), dtype=np.float32)
    gain = np.ones(K, dtype=np.float32) * VIS_SIGMA
    for c in OUTLIER_CHANNELS:
        if c < K:
            gain[c] *= OUTLIER_GAIN
    x[is_vis] *= gain
    return x.astype(np.float16)


def draw_weights(rng, N: int, K: int) -> np.ndarray:
    """Canonical packed int4 [N, K/2] (even k in the low nibble): uniform bytes."""
    return rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)


def draw_w_scale(rng, N: int) -> np.ndarray:
    return rng.uniform(0.005, 0.02, size=N).astype(np.float16)


def make_linear_inputs(wl: Workload, proj: str, *, want_calib: bool = True,
                       T_override: int | None = None) -> dict:
    """All inputs of one linear of one workload, in ORIGINAL token order."""
    names: List[str] = list(wl.projections)
    K, N = wl.projections[proj]
    T = wl.T if T_override is None else T_override
    r_x, r_w, r_s, r_cv, r_ct = _streams(seed_for(wl.cfg, names.index(proj)))
    is_vis = _is_visual(T, wl.vis_spans)
    out = {
        "T": T, "K": K, "N": N, "had_block": wl.had_block,
        "vis_spans": tuple(wl.vis_spans),
        "x": draw_activations(r_x, T, K, is_vis),
        "w_packed": draw_weights(r_w, N, K),
        "w_scale": draw_w_scale(r_s, N),
    }
    if want_calib:
        out["calib_vis"] = draw_activations(r_cv, CALIB_ROWS, K, np.ones(CALIB_ROWS, dtype=bool))
        out["calib_txt"] = draw_activations(r_ct, CALIB_ROWS, K, np.zeros(CALIB_ROWS, dtype=bool))
    return out


def device_linear_inputs(torch, wl: Workload, proj: str, *, want_x: bool = True) -> dict:
    """The same recipe drawn on the GPU with torch's seeded generator: benchmark inputs of the
    large configurations, where a host draw plus upload would dominate the run.  Distributions,
    shapes and token layout are those of make_linear_inputs; the values are another draw."""
    names: List[str] = list(wl.projections)
    K, N = wl.projections[proj]
    T = wl.T
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed_for(wl.cfg, names.index(proj)) + 7_000_000)
    gain = torch.full((K,), VIS_SIGMA, dtype=torch.float32, device="cuda")
    for c in OUTLIER_CHANNELS:
        if c < K:
            gain[c] *= OUTLIER_GAIN
    is_vis = torch.from_numpy(_is_visual(T, wl.vis_spans)).cuda()

    def draw(rows, vis_mask):
        out = torch.empty((rows, K), dtype=torch.float16, device="cuda")
        for r0 in range(0, rows, 2048):                       # slabs: no fp32 temporary of the whole matrix
            r1 = min(r0 + 2048, rows)
            blk = torch.randn((r1 - r0, K), dtype=torch.float32, device="cuda", generator=gen)
            m = vis_mask[r0:r1]
            blk[m] *= gain
            out[r0:r1] = blk.to(torch.float16)
        return out

    ones = torch.ones(CALIB_ROWS, dtype=torch.bool, device="cuda")
    res = {
        "T": T, "K": K, "N": N, "had_block": wl.had_block, "vis_spans": tuple(wl.vis_spans),
        "w_packed": torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda", generator=gen),
        "w_scale": (torch.rand(N, device="cuda", generator=gen) * 0.015 + 0.005).to(torch.float16),
        "calib_vis": draw(CALIB_ROWS, ones),
        "calib_txt": draw(CALIB_ROWS, ~ones),
    }
    if want_x:
        res["x"] = draw(T, is_vis)
    return res
