// placeholder until the MFMA backward and decode kernels land
#include "cart_common.h"
namespace cart {
bool attn_mfma_bwd_supported(const cart_attn_desc&) { return false; }
size_t attn_mfma_bwd_workspace(const cart_attn_desc&) { return 0; }
int launch_attn_bwd_mfma(const cart_attn_desc&, float, const void*, const void*, const void*, const void*, const void*, const void*, const float*, const void*, void*, void*, void*, float*, float*, void*, hipStream_t) { return 1; }
bool decode_mfma_supported(const cart_decode_desc&) { return false; }
size_t decode_mfma_workspace(const cart_decode_desc&) { return 0; }
int launch_decode_mfma(const cart_decode_desc&, float, const void*, const void*, const void*, const void*, const void*, const int32_t*, void*, float*, void*, hipStream_t) { return 1; }
}
