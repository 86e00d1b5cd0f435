"""MI355X-native W4A8 linear layer with modality-specific static activation
scales (the hot path of MQuant, arXiv 2502.00425).

``paper_2502_00425_amd.binding`` is the ctypes binding of the HIP library
(importing it loads ``lib/libmquant.so`` and fails loudly if it is missing);
``paper_2502_00425_amd.workloads`` is the seeded synthetic input generator;
``paper_2502_00425_amd.build`` compiles the library with hipcc for gfx950.
"""
import math as _math

__all__ = ["static_scale_from_absmax"]


def static_scale_from_absmax(absmax_u: float, had_block: int) -> float:
    """Static per-tensor scale from the rotated absmax statistic returned by
    ``mquant_hadamard_absmax``: s = (max|u| / sqrt(B)) / 127, rounded to fp32
    (Eq. (2) of the paper with b = 8)."""
    import numpy as _np
    return float(_np.float32(float(absmax_u) / _math.sqrt(float(had_block)) / 127.0))
