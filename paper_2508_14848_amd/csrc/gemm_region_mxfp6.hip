// gemm_mp_fp8_region_kernel<5>: one instance per file so that the instances compile in parallel.
#include "gemm_region_kernel.h"

GMP_REGION_INSTANCE(region_mxfp6, 5)
