// placeholder until the MFMA kernels land
#include "internal.h"
namespace sp {
bool attention_flash_supported(int, int, int, int, int) { return false; }
void attention_flash_fwd(hipStream_t, int, int, int, int, int, const void*, void*, float*) {}
void attention_flash_bwd(hipStream_t, int, int, int, int, int, const void*, const void*, const float*, const void*, void*, float*) {}
}
