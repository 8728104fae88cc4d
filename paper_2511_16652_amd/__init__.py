"""MI355X-native EGGROLL hot path: population forward with low-rank perturbations + ES update.

The compute lives in hand-written HIP kernels behind a C ABI (``include/eggroll.h``,
``csrc/``); ``binding`` marshals arguments for it and ``inputs`` draws synthetic workloads.
"""
__all__ = ["binding", "inputs"]
