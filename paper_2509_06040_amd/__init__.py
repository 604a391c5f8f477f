"""libbranchrollout: the BranchGRPO tree rollout (arXiv 2509.06040) on MI355X.

`paper_2509_06040_amd.binding` is the thin ctypes layer over the C-ABI library
built from `csrc/`; `paper_2509_06040_amd.synth` holds the seeded synthetic
input generators (no method arithmetic).  Nothing is imported eagerly so that
the generators can be used without the compiled library.
"""
__all__ = ["binding", "synth", "build"]
