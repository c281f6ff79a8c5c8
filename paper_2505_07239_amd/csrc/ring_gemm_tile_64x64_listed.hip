// The 64 x 64 output tile of the int8 matrix-core kernel: the variants that walk a step list (Protocol 3 with per-token row sets)
// (see ring_gemm_kernel.h).
#include "ring_gemm_kernel.h"

template comet_gemm::GemmKernel comet_gemm::gemm_kernel_for<2, 2, 1, 1, true>(const GemmParams&);
