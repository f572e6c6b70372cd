"""Straggler-aware distributed SGD (K-sync / K-batch-sync / K-async / AdaSync)
simulated as batched virtual workers on one MI355X.

``paper_2003_10579_amd.ssgd`` is the ctypes binding of the C-ABI library
(`include/ssgd.h`); ``paper_2003_10579_amd.synth`` makes the seeded inputs.
"""
