// The signal-gated GEMM kernels (plain and grouped) of one tile configuration: 256 x 256 tiles, MFMA form 16x16x32.
#include "gemm_kernel.h"

AGG_GEMM_INSTANCE(256, 256, 16)
