"""MI355X-native 2-bit lookup-table GEMM / convolution (DeepGEMM's LUT-16 method on gfx950).

``paper_2304_09049_amd.binding`` is the ctypes binding over the C-ABI library
(``libdeepgemm_hip.so``, declared in ``include/deepgemm_hip.h``);
``paper_2304_09049_amd.workloads`` draws the seeded synthetic inputs.
Importing this package loads neither torch nor the GPU library.
"""

__all__ = ["binding", "workloads"]
