#include "launch.h"
extern "C" size_t fog_fp8_attn_workspace(int B, int H, int S, int D, int is_bwd) { (void)D; return is_bwd ? (size_t)B * H * S * 4 : 0; }
extern "C" fog_status fog_fp8_attn_fwd(int, int, int, int, float, int, const uint8_t*, const uint8_t*, const uint8_t*, const float*, const float*, const float*, const float*, void*, float*, float*, void*, size_t, void*) { return FOG_ERR_UNSUPPORTED; }
extern "C" fog_status fog_fp8_attn_bwd(int, int, int, int, float, int, const uint8_t*, const uint8_t*, const uint8_t*, const float*, const float*, const float*, const void*, const void*, const uint8_t*, const float*, const float*, const float*, const float*, void*, void*, void*, float*, void*, size_t, void*) { return FOG_ERR_UNSUPPORTED; }
