// gemm_mp_owner_kernel<double, true, false>: one instance per file so that the instances compile in parallel.
#include "gemm_owner_kernel.h"

GMP_OWNER_INSTANCE(owner_d_mixed, double, true, false)
