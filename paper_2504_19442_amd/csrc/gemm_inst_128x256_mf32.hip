// The signal-gated GEMM kernels (plain and grouped) of one tile configuration: 128 x 256 tiles, MFMA form 32x32x16.
#include "gemm_kernel.h"

AGG_GEMM_INSTANCE(128, 256, 32)
