"""MI355X-native DeepPoly back-substitution (hand-written HIP kernels behind a C ABI).

``workloads`` (seeded synthetic inputs) is pure numpy.  ``binding`` loads the
HIP shared library and fails loudly if it has not been built.
"""
