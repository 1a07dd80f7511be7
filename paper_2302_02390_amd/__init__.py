"""MI355X-native QSDP quantization codec and fused quantized SGD step.

The compute lives in hand-written HIP kernels behind a C ABI (``libqsdp.so``,
declared in ``include/qsdp.h``); :mod:`paper_2302_02390_amd.binding` marshals
torch tensors (device memory and streams only) into those calls.
"""
__all__ = ["binding", "workloads"]
