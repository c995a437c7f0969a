"""MI355X-native hot path of the residual-vector-quantization KV-cache compressor
(arXiv 2410.15704): per-vector std scaling, channel grouping, greedy residual
encoding against shared codebooks, the matching decode and the moving-average
codebook update, as a C-ABI library of hand-written HIP kernels for gfx950.

``paper_2410_15704_amd.binding`` loads the library (and raises if it has not
been built); ``paper_2410_15704_amd.synth`` holds the seeded input generators.
Nothing is imported eagerly so that the generators can be used without a GPU.
"""

__all__ = ["binding", "synth", "build"]
