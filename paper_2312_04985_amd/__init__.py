"""SparQ Attention decode step for one MI355X: hand-written HIP kernels behind a C ABI.

`binding` is the thin ctypes layer over libsparq.so (argument marshalling only),
`workloads` draws the seeded synthetic inputs, `traffic` is the paper's transfer model.
Nothing here computes any part of the method on the host.
"""
__all__ = ["binding", "workloads", "traffic"]
