"""MI355X-native hot path of LoopServe's online-sparsified prefill attention.

`paper_2507_13681_amd.binding` exposes the four C-ABI entry points of
libloopserve (ls_score, ls_select, ls_sparse_prefill, ls_kv_compress);
`paper_2507_13681_amd.inputs` draws the seeded synthetic workloads.
Importing the package loads nothing native; the binding loads the HIP library
on first use and raises if it is missing.
"""
__all__ = ["inputs", "binding"]
