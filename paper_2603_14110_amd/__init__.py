"""MI355X-native decode step of a ReGLU FFN gated by a low-rank SVD sparsity predictor.

``binding`` is the thin ctypes layer over the C-ABI library ``libsvdp.so``
(hand-written HIP kernels for gfx950); ``synth`` holds the seeded synthetic
input generators; ``cost`` the multiplication / byte accounting.  Importing the
package does not load the library; ``binding.lib()`` does and raises if it has
not been built.
"""

__all__ = ["binding", "synth", "cost"]
