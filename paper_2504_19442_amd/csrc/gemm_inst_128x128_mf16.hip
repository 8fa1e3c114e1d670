// The signal-gated GEMM kernels (plain and grouped) of one tile configuration: 128 x 128 tiles, MFMA form 16x16x32.
#include "gemm_kernel.h"

AGG_GEMM_INSTANCE(128, 128, 16)
