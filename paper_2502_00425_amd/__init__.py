"""MI355X-native W4A8 linear layer with modality-specific static activation
scales (the hot path of MQuant, arXiv 2502.00425).

``paper_2502_00425_amd.binding`` is the ctypes binding of the HIP library
(importing it loads ``lib/libmquant.so`` and fails loudly if it is missing);
``paper_2502_00425_amd.workloads`` is the seeded synthetic input generator;
``paper_2502_00425_amd.build`` compiles the library with hipcc for gfx950.
The package itself holds no arithmetic of the method.
"""
