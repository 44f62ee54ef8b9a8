"""TABX batched battle-environment step for MI355X: HIP kernels behind a C ABI.

`binding` loads libtabx.so (built by `build`); `inputs` draws the seeded synthetic
workloads.  Nothing is imported eagerly so that the input generators stay usable
where the HIP library is not needed.
"""
__all__ = ["binding", "build", "inputs"]
