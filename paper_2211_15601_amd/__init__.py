"""MI355X-native Fast-SNARF articulation path (batched Broyden correspondence search).

`paper_2211_15601_amd.binding` is the thin ctypes layer over the C-ABI library built from
`csrc/`; `paper_2211_15601_amd.workloads` synthesises seeded inputs.  Nothing is loaded
on import; the binding raises if the HIP library has not been built.
"""
__all__ = ["binding", "workloads"]
