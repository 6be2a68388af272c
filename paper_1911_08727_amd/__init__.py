"""MI355X-native per-layer error-compensated top-k sparsifier (LAGS-SGD hot path).

`paper_1911_08727_amd.lags` is the thin ctypes binding of the C-ABI library
(liblags.so, hand-written HIP for gfx950); `paper_1911_08727_amd.workloads`
holds the seeded synthetic layer tables and gradient generators.
"""
