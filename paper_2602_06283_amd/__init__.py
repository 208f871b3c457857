"""MI355X-native SOCKET decode path: soft-collision LSH scoring, top-k selection and
sparse flash-decode attention as hand-written gfx950 HIP kernels behind a C ABI.

`paper_2602_06283_amd.binding` is the thin ctypes layer over libsocket.so;
`paper_2602_06283_amd.workloads` draws the seeded synthetic inputs.
"""
__all__ = ["binding", "workloads", "build"]
