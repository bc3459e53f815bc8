// placeholder until the MFMA GEMM lands
#include "taw_internal.h"
namespace taw {
bool gemm_mfma_supported(int, int, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int, int64_t) { return false; }
int launch_gemm_mfma(int, int64_t, int64_t, int64_t, const void*, int64_t, const void*, int64_t, void*, int64_t, int, int, const void*, int64_t, hipStream_t) { return (int)hipErrorNotSupported; }
}
