"""MI355X-native CSR SPMM / SDDMM / FusedMM (FP32) behind a C-ABI library.

`paper_2311_00368_amd.binding` marshals torch device tensors into the C-ABI
calls declared in `include/csrk.h`; `paper_2311_00368_amd.inputs` is the seeded
synthetic-input generator used by tests and the benchmark.  Importing this
package loads nothing; the HIP library is loaded on first use of the binding
and its absence is an error (there is no CPU fallback).
"""

__all__ = ["binding", "inputs"]
