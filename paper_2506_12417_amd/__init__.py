"""MI355X-native MoE-layer forward (the hot path of HarMoEny, arXiv 2506.12417, on one GPU).

`paper_2506_12417_amd.binding` is the ctypes face of libmoe.so: same names as include/moe.h,
argument marshalling only.  `paper_2506_12417_amd.layer` chains the calls into one layer
forward.  Importing either raises if the built library is missing -- there is no fallback.
"""
__all__ = ["binding", "layer", "build"]
