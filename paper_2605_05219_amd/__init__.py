"""Resume-from-checkpoint GatedDeltaNet prefill with sparse checkpoint emission on MI355X.

`binding` wraps the C ABI of the HIP library (include/gdn_resume.h); `workloads` draws the
seeded synthetic inputs; `build` compiles the library in-tree.
"""
__all__ = ["binding", "workloads", "build"]
