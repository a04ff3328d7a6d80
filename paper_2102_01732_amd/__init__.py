"""MI355X-native hot path of truly sparse MLP training with SET (arXiv 2102.01732).

The compute lives in ``csrc/`` (hand-written HIP for gfx950) behind the C ABI declared in
``include/sparse_set.h``; ``binding`` marshals arguments to it.  Importing the package does not
load the native library; ``binding.lib()`` does, and fails loudly when it has not been built.
"""
