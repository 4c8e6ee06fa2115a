"""One GPU's share of a transformer layer's training step on MI355X (gfx950).

The compute lives in a C-ABI shared library of hand-written HIP kernels (csrc/); `binding`
marshals arguments for it and `inputs` draws seeded synthetic tensors.  Importing the package
does not load the library; `binding.lib()` does, and raises if it has not been built.
"""
