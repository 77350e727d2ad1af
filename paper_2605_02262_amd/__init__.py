"""WindowQuant hot path on MI355X: a ctypes binding over a C-ABI HIP library.

``synth`` (seeded input generators) imports nothing but numpy; the GPU binding
lives in ``binding`` and is loaded on first use.
"""
