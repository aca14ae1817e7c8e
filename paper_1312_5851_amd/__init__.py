"""FFT-based convolution passes (fprop / bprop / accGrad) for one conv layer on MI355X.

``paper_1312_5851_amd.fftconv`` is the binding to the HIP library (it raises at
import when the library has not been built); ``paper_1312_5851_amd.workloads``
names the synthetic layers and draws their seeded inputs.
"""
__all__ = ["fftconv", "workloads"]
