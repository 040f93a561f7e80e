// Placeholders until the MFMA denoisers land: the symbols exist and report "unsupported".
#include "sdden_internal.h"
extern "C" {
int sdden_lowrank_create(int32_t, int32_t, const float*, const float*, float, int32_t, const float*, sdden**) {
  return sdi::fail(sdi::g_den_create_error, SD_ERR_UNSUPPORTED, "sdden_lowrank_create: not built yet");
}
int sdden_mlp_create(int32_t, int32_t, int32_t, const uint16_t*, const float*, const uint16_t*, const float*,
                     const uint16_t*, const float*, int32_t, int32_t, sdden**) {
  return sdi::fail(sdi::g_den_create_error, SD_ERR_UNSUPPORTED, "sdden_mlp_create: not built yet");
}
}
