// gemm_mp_owner_low_kernel: FP64 C tiles without an FP64 product; one instance per file so that the instances compile in parallel.
#include "gemm_owner_kernel.h"

GMP_OWNER_LOW_INSTANCE(owner_d_low)
