"""Co-sharded multi-head attention (forward + backward) for MI355X / gfx950.

The compute lives in a C-ABI shared library built from csrc/ (hand-written HIP
kernels); `binding` marshals arguments to it.  Importing this package does not
load the library; `binding.lib()` does, and raises if it has not been built.
"""
