// The 128 x 64 output tile of the int8 matrix-core kernel with weight planes: the variants for
// launches in which every workgroup owns whole output tiles (see owns_tiles()).
#include "ring_gemm_kernel.h"

template comet_gemm::GemmKernel comet_gemm::gemm_own_planes_kernel_for<2, 2, 2, 1>(const GemmParams&);
