// placeholder until the MFMA kernels land
#include "internal.h"
namespace sp {
bool gemm_mfma_supported(int, int64_t, int64_t, int64_t, const void*, const void*, const void*, const void*) { return false; }
void gemm_mfma(hipStream_t, int, int64_t, int64_t, int64_t, const void*, const void*, void*, const void*) {}
}
