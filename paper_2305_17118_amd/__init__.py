"""MI355X-native budgeted KV cache (Scissorhands, arxiv 2305.17118): decode hot path.

The compute lives in ``csrc/`` (HIP kernels for gfx950 behind a C ABI declared in
``include/sc.h``); ``binding`` marshals arguments to it and nothing else.  Importing the
package does not load the library; the first call does, and fails loudly if it is missing.
"""
