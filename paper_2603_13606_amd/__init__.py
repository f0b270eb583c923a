"""One rank's share of MoE dispatch and combine on MI355X (gfx950).

`paper_2603_13606_amd.binding` wraps the C-ABI library (`libep_mi355x.so`, built from
`csrc/`); `paper_2603_13606_amd.buffer` is the framework-facing buffer on top of it;
`paper_2603_13606_amd.workloads` generates seeded synthetic inputs.  Importing
this package loads nothing: the shared library is opened on first use and its
absence is an error, never a fallback.
"""
__all__ = ["binding", "buffer", "workloads", "build"]
