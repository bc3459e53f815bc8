// placeholder until the MFMA attention lands
#include "taw_internal.h"
namespace taw {
bool attn_mfma_supported(int, int, int) { return false; }
int launch_attn_fwd_mfma(int, int, int, const void*, void*, float*, hipStream_t) { return (int)hipErrorNotSupported; }
int launch_attn_bwd_mfma(int, int, int, const void*, const void*, const float*, const float*, void*, hipStream_t) { return (int)hipErrorNotSupported; }
}
