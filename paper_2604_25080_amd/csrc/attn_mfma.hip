#include "kernels.h"
#include "cacheflow.h"
namespace cf {
bool attention_mfma_supported(int, int, int, int) { return false; }
void launch_attention_mfma(hipStream_t, const void*, void*, const void*, const AttnWork*, int, const int32_t*, int, KvGeom) {}
}
