"""MI355X-native batched speculative verification (server-side hot path of SLED, arXiv 2506.09397).

`synth` draws seeded inputs and imports nothing heavy; `sled` is the ctypes binding of the
HIP library and fails loudly when the library has not been built.
"""
