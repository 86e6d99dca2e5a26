"""MI355X-native VidKV hot path: sub-2-bit KV-cache codec + packed decode attention.

`paper_2503_16257_amd.binding` is the thin ctypes layer over the C-ABI library
built from `csrc/`; `paper_2503_16257_amd.synth` draws the synthetic inputs.
Importing the package loads nothing native; the library is loaded on first use
of the binding and its absence is an error, never a fallback.
"""
