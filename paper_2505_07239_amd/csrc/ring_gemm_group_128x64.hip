// The grouped matrix-core kernel (several products of one shape in one launch), 128 x 64 output
// tile, weight planes: the variants that share output tiles between workgroups.
#include "ring_gemm_kernel.h"

template comet_gemm::GemmGroupKernel comet_gemm::gemm_group_kernel_for<2, 2, 2, 1, false>(const GemmParams&);
