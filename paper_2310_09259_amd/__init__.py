"""MI355X-native QUIK hybrid-quantized linear layer (arXiv 2310.09259, Algorithm 1).

``paper_2310_09259_amd.api`` binds the C ABI declared in include/quik.h;
``paper_2310_09259_amd.synth`` draws the seeded synthetic inputs.  Importing the
package loads nothing; the shared library is loaded on first use and its absence
is an error (there is no fallback path).
"""
__all__ = ["api", "synth", "build"]
