"""Information, not parity: how many int8 codes of the benchmark inputs depend on the two
rounding choices the oracle (and the kernel) make in the online rotation and the quantizer.

  (a) fp32 butterflies in stage order against the exact rotation: x H_B is exact in fp64 (every
      fp16 value is a multiple of 2^-24 below 2^16 and 512 of them fit 53 bits), so the exact
      rotated value is known; it is rounded once to fp32 and quantized by the same rule.
  (b) one fp32 multiply by c = fp32(1 / (s sqrt(B))) against a true fp32 division by s sqrt(B).
  (c) the oracle's codes against Eq. (2) evaluated in fp64 throughout.

Run: python -m oracle.rounding_report [cfg ...]      (CPU only; calls nothing but oracle/ and
the seeded input generator).  Test infrastructure, like the rest of oracle/.
"""
from __future__ import annotations

import math
import sys

import numpy as np

from oracle import mquant_oracle as orc
from paper_2502_00425_amd import workloads as wl


def report(cfg: int, chunk_rows: int = 1024):
    w = wl.workload(cfg)
    B = w.had_block
    H = orc.hadamard_matrix(B).astype(np.float64)
    out = []
    for proj in w.projections:
        inp = wl.make_linear_inputs(w, proj)
        s_vis = float(orc.calibrate_static_scale(inp["calib_vis"], B))
        s_txt = float(orc.calibrate_static_scale(inp["calib_txt"], B))
        perm, _, V = orc.aifs_build_perm(inp["T"], inp["vis_spans"])
        T, K = inp["T"], inp["K"]
        n = T * K
        d_rot = d_div = d_exact = 0
        c32 = {True: orc.quant_multiplier(s_vis, B), False: orc.quant_multiplier(s_txt, B)}
        for r0 in range(0, T, chunk_rows):
            rows = np.arange(r0, min(r0 + chunk_rows, T))
            x_u = inp["x"][perm[rows]]
            vis = (rows < V)[:, None]
            u32 = orc.hadamard_rotate(x_u, B)                                   # fp32 butterflies
            v_here = int((rows < V).sum())
            # the chunk keeps the AIFS order, so its first v_here rows are the visual ones
            codes = orc.msq_quantize(u32, v_here, s_vis, s_txt, B)
            u_exact = (x_u.astype(np.float64).reshape(len(rows), K // B, B) @ H).reshape(len(rows), K)
            codes_rot = orc.msq_quantize(u_exact.astype(np.float32), v_here, s_vis, s_txt, B)
            d_rot += int((codes != codes_rot).sum())
            denom32 = np.where(vis, np.float32(np.float32(s_vis) * np.float32(math.sqrt(B))),
                               np.float32(np.float32(s_txt) * np.float32(math.sqrt(B)))).astype(np.float32)
            t_div = (u32 / denom32).astype(np.float32)
            codes_div = np.clip(np.rint(t_div), -128, 127).astype(np.int8)
            d_div += int((codes != codes_div).sum())
            s64 = np.where(vis, float(np.float32(s_vis)), float(np.float32(s_txt)))
            codes_exact = np.clip(np.rint(u_exact / (math.sqrt(B) * s64)), -128, 127).astype(np.int8)
            d_exact += int((codes != codes_exact).sum())
        out.append((proj, n, d_rot, d_div, d_exact))
        print(f"configs[{cfg}] {proj:8s} T*K = {n:>11d}: fp32 butterflies vs exact rotation {d_rot} "
              f"({d_rot / n:.2e}), multiply vs divide {d_div} ({d_div / n:.2e}), oracle vs fp64 Eq. (2) "
              f"{d_exact} ({d_exact / n:.2e})", flush=True)
    return out


if __name__ == "__main__":
    for c in [int(a) for a in sys.argv[1:]] or [1]:
        report(c)
