"""MI355X-native hot path of Deep Gradient Compression (arXiv 1712.01887).

`synthetic` lists gradient-set shapes and draws seeded inputs; `binding`
wraps the C-ABI of libdgc (HIP kernels for gfx950); `build` compiles it.
Nothing is loaded at import time: `binding.load()` opens the shared library
and raises if it has not been built.
"""

__all__ = ["binding", "build", "synthetic"]
