// The 32 x 256 output tile of the int8 matrix-core kernel: the variants that walk a step list (Protocol 3 with per-token row sets)
// (see ring_gemm_kernel.h).
#include "ring_gemm_kernel.h"

template comet_gemm::GemmKernel comet_gemm::gemm_kernel_for<1, 4, 1, 2, true>(const GemmParams&);
