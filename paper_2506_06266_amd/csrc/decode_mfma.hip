// placeholder until the MFMA decode kernels land
#include "cart_common.h"
namespace cart {
bool decode_mfma_supported(const cart_decode_desc&) { return false; }
size_t decode_mfma_workspace(const cart_decode_desc&) { return 0; }
int launch_decode_mfma(const cart_decode_desc&, float, const void*, const void*, const void*, const void*, const void*, const int32_t*, void*, float*, void*, hipStream_t) { return 1; }
}
