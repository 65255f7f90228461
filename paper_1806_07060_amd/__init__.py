"""Model-driven adaptive SGEMM for MI355X (gfx950).

fp32 GEMM served by a small family of hand-written HIP kernels behind a C-ABI
library (include/mdg_sgemm.h), with a decision tree, trained offline on
measured runtimes, compiled into the library's dispatch.

Sub-modules:
  binding    thin ctypes binding of the C-ABI (argument marshalling only)
  workloads  seeded synthetic cases and operands (no arithmetic of the method)
  tuning     offline phase: exhaustive timing, CART training, code generation, evaluation

Importing the package does not load the HIP library; `binding.lib()` does, and
raises if it has not been built.
"""
__all__ = ["binding", "workloads", "tuning"]
