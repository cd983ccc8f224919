"""Crystal-KV decode hot path for MI355X (gfx950).

`paper_2601_16986_amd.ckv` is the thin Python binding of the C-ABI library
built from `csrc/`; `paper_2601_16986_amd.workloads` draws the seeded
synthetic inputs.  Importing the package loads nothing native; the binding
loads the shared library on first use and raises if it is not built.
"""
__all__ = ["ckv", "workloads"]
