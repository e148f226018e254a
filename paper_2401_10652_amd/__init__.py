"""MI355X-native executor of AutoChunk chunk plans (arXiv 2401.10652, section 2.2).

The compute path lives in ``csrc/`` (HIP kernels for gfx950 behind a C-ABI shared
library); ``binding`` marshals arguments to it and ``inputs`` draws the seeded
synthetic tensors.  Importing the package does not load the shared library;
``binding.lib()`` does and raises if it has not been built.
"""
