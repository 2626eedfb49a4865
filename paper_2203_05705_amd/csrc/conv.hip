// Convolution with dropped input feature maps (Sections 5, 6).
#include "engine.hpp"
#include "pattern.hpp"

using namespace ard;

extern "C" size_t ard_conv_workspace_bytes(int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t,
                                           int32_t, int32_t) {
  return 0;
}

extern "C" int32_t ard_fmap_drop_conv(int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t,
                                      int32_t, int32_t, double, int32_t, const void*, const void*, const void*, void*,
                                      uint8_t*, int32_t*, int32_t*, int64_t*, void*, size_t, void*) {
  return fail(ARD_EUNSUPPORTED, "ard_fmap_drop_conv is not built yet");
}
