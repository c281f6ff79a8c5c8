"""MI355X-native local computation of the sparse secret-shared FFN matmul over
Z_{2^64}: Python binding of the C-ABI library ``libcomet_ring.so``."""
from .binding import (AXIS_COLS, AXIS_ROWS, FULL_A, FULL_B, WEIGHTS_NEURON_MAJOR, WEIGHT_PLANES, WeightPlanes, OP_COMPACT, OP_SIMM, OP_SOMM,  # noqa: F401
                      TUNE_GEMM_CHUNK, TUNE_GEMM_GRID, TUNE_GEMM_TILE, TUNE_SKINNY, TUNE_SKINNY_SLICES, TUNE_COMPONENTS, TUNE_TIMING_STRIDE, TUNE_GROUP, CometError, Context, load_library, workspace_bytes)
