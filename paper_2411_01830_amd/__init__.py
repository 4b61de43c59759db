"""MI355X-native batched scatter-gather transfer engine (hot path of FaaSTube's
GPU-oriented data passing, arxiv 2411.01830) - Python side.

``binding`` marshals arguments into the C ABI of ``libfaastube.so`` (every step of
the path runs in the library's HIP kernels and host code); ``harness`` owns the
device and pinned memory the tests and the benchmark hand to it. There is no CPU
fallback: importing ``binding`` fails if the library has not been built.
"""
