"""MI355X-native batched IVF top-k retrieval (the retrieval stage of a
decoupled retrieve-then-generate RAG pipeline).

`ivf`        thin ctypes binding over the C-ABI library (HIP kernels, gfx950)
`workloads`  seeded synthetic inputs shared by tests, bench and the oracle's tests
"""
