#include "kernels.h"
#include "cacheflow.h"
namespace cf {
bool gemm_mfma_supported(int, int, int, int, int) { return false; }
void launch_gemm_mfma(hipStream_t, const void*, const void*, const void*, float*, void*, int, int, int, int) {}
}
