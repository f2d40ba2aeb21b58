"""MI355X-native 1D dilated convolution layer (forward, backward-data, backward-weight).

The compute lives in hand-written HIP kernels behind a C ABI (``include/conv1d.h``);
``paper_2104_08002_amd.binding`` marshals arguments to it.  ``inputs`` draws the
synthetic workloads.  Nothing here falls back to a CPU implementation.
"""
__all__ = ["binding", "inputs"]
