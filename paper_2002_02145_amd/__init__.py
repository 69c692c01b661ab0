"""MI355X-native forward convolution over blocked layouts (batch-reduce GEMM on MFMA).

``workloads`` (seeded synthetic layers) imports without the HIP library; ``binding`` loads
``libpsconv.so`` and raises ImportError if it has not been built.
"""
__all__ = ["workloads", "binding"]
