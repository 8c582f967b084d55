"""MI355X-native Quartet MXFP4 linear-layer path (arXiv 2505.14669, Algorithm 1).

`paper_2505_14669_amd.binding` loads the HIP library (C ABI declared in include/quartet.h) and
raises if it has not been built; `paper_2505_14669_amd.synth` makes the seeded synthetic inputs;
`paper_2505_14669_amd.nn` wraps the two layer entry points as a torch autograd function and module.
There is no CPU fallback.
"""
__all__ = ["binding", "synth", "nn"]
