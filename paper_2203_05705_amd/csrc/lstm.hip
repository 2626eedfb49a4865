// LSTM layer under a hidden-unit row pattern (Section 7.2.3).
#include "engine.hpp"
#include "pattern.hpp"

using namespace ard;

extern "C" size_t ard_lstm_workspace_bytes(int32_t, int32_t, int32_t, int32_t, int32_t, const ard_pattern*) { return 0; }

extern "C" int32_t ard_lstm_fwd(int32_t, int32_t, int32_t, int32_t, int32_t, const void*, const void*,
                                const ard_pattern*, void*, float*, float*, void*, size_t, void*) {
  return fail(ARD_EUNSUPPORTED, "ard_lstm_fwd is not built yet");
}

extern "C" int32_t ard_lstm_bwd(int32_t, int32_t, int32_t, int32_t, int32_t, const void*, const void*,
                                const ard_pattern*, const void*, const float*, const float*, const void*, void*, void*,
                                void*, size_t, void*) {
  return fail(ARD_EUNSUPPORTED, "ard_lstm_bwd is not built yet");
}
