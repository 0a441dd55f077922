"""fp64 CPU oracle of the truncated path-signature transform (test infrastructure only).

Nothing in the product imports this package: it exists so that tests, the smoke
check and the benchmark's cpu_baseline leg can compare the HIP path against the
paper's definition (Section 3.1, Eqs. 2-5 and Eq. 10), its level-by-level reformulation (Section 3.2,
Eqs. 6-10) and its gradient (Section 4.2, Eq. 11).
"""
from .sig_oracle import (build, signature, signature_backward, tensor_exp, tensor_mul, sig_size,
                         num_threads, level_slices)
from .sig_levelwise import signature_levelwise

__all__ = ["build", "signature", "signature_levelwise", "signature_backward", "tensor_exp", "tensor_mul", "sig_size",
           "num_threads", "level_slices"]
