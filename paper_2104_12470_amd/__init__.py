"""MI355X-native decoder-layer hot path of the EET paper (arXiv 2104.12470).

`paper_2104_12470_amd.eet` is the thin ctypes binding over the C-ABI library built from
`csrc/`; `paper_2104_12470_amd.workloads` generates the seeded synthetic inputs.  Nothing
here falls back to a CPU path: using the binding without the built library raises.
"""
__all__ = ["workloads"]
