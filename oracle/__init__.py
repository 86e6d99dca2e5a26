"""CPU oracle for the VidKV hot path (KV-cache codec + decode attention).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its
Python binding) imports, calls or links anything in this package; only the
tests, the smoke check and the benchmark's cpu_baseline leg do.  The oracle in
turn imports nothing from the HIP path.

Modules
-------
vidkv_oracle : the method's arithmetic in float64, written from the paper's
               equations and algorithms (Eq. 3-7, Alg. 1-3).
layout       : an independent numpy reader/writer of the packed cache format,
               so the oracle can decode buffers that the GPU produced.
"""
