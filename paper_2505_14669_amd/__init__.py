"""MI355X-native Quartet MXFP4 linear-layer path (arXiv 2505.14669, Algorithm 1).

`paper_2505_14669_amd.binding` loads the HIP library (C ABI declared in include/quartet.h) and
raises if it has not been built; `paper_2505_14669_amd.synth` makes the seeded synthetic inputs.
There is no CPU fallback.
"""
__all__ = ["binding", "synth"]
