// The 32 x 128 output tile of the int8 matrix-core kernel: the variants whose weight-side operands
// arrive as digit planes (see PlaneLoader in ring_gemm_kernel.h).
#include "ring_gemm_kernel.h"

template comet_gemm::GemmKernel comet_gemm::gemm_planes_kernel_for<1, 4, 1, 1, false>(const GemmParams&);
