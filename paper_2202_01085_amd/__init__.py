"""MI355X-native F3M kernel matrix-vector product (arXiv 2202.01085).

`paper_2202_01085_amd.f3m` is the thin ctypes binding of the C-ABI library
built from csrc/ (it raises if the library is missing: there is no fallback);
`paper_2202_01085_amd.inputs` holds the seeded synthetic input generators.
"""
