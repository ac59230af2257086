// Read half, matrix-core kernel (placeholder until the FP4 MFMA path lands).
#include "rkv_internal.h"

bool rkv_mfma_supported(const rkv_cache*) { return false; }

int rkv_launch_decode_mfma(rkv_cache*, const __half*, const int*, float*, float*, void*, hipStream_t) { return RKV_EINVAL; }
