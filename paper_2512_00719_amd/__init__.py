"""MI355X-native sampling epilogue (logits -> token ids): HIP kernels behind a C boundary.

``binding`` loads the shared library; ``synth`` generates seeded synthetic inputs; ``build``
compiles the library in-tree.  Importing this package does not load the library.
"""
