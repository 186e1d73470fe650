"""MI355X-native bit-packing and binary direct convolution (daBNN hot path, arXiv 1908.05858).

``paper_1908_05858_amd.binding`` loads the HIP library and exposes the C-ABI entry points under
the same names; ``paper_1908_05858_amd.workloads`` holds the seeded synthetic inputs.  Nothing is
loaded at package import time.
"""
__all__ = ["binding", "workloads"]
