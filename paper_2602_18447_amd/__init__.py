"""MI355X-native batched verification pass for confidence-gated cascaded step verification.

The compute lives in libconfspec.so (hand-written HIP for gfx950 behind a C ABI, see
include/confspec.h).  `binding` mirrors the C entry points one to one; `runner.Verifier` owns the
device buffers around them.  Importing `binding` fails loudly if the library has not been built.
"""
