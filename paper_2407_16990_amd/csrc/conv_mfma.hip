#include "rh_internal.h"
rh_status rh_pack_weights_bf16(rh_ctx* ctx, const float*) { RH_FAIL(ctx, RH_E_UNIMPLEMENTED, "bf16 path not built yet"); }
rh_status rh_launch_enhance_bf16(rh_ctx* ctx, const uint8_t*, int, int, int, float*, const uint32_t*) { RH_FAIL(ctx, RH_E_UNIMPLEMENTED, "bf16 path not built yet"); }
