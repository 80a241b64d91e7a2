"""PipeFusion patch-stage hot path for AMD MI355X (gfx950): HIP kernels behind a C boundary
(include/pfstage.h) and a thin ctypes binding.  Importing the package does not load the library;
the first call does, and raises if it has not been built."""
from .binding import (PF_BF16, PF_F32, PF_PATH_AUTO, PF_PATH_AUTO_PRESCALED_Q, PF_PATH_SIMT, PfError, Stage, load_library,  # noqa: F401
                      pf_op_attention, pf_op_attention_static, pf_op_axpby, pf_op_axpy, pf_op_gemm, pf_op_kv_scatter, pf_op_ln_modulate, pf_op_modulation, probe_mfma_tflops)
