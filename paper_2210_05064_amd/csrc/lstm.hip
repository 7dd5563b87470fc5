// placeholder until the LSTM kernels land
#include "common.h"
extern "C" size_t ver_lstm_workspace_bytes(const ver_lstm_cfg*, int32_t) { return 0; }
extern "C" int ver_lstm_fwd(const ver_lstm_cfg*, const void*, int32_t, const int32_t*, const int32_t*, const int32_t*,
                 const float*, const float*, int32_t, const float* const*, float*, float*, void*, size_t, void*) { return VER_EUNSUPPORTED; }
extern "C" int ver_lstm_bwd(const ver_lstm_cfg*, const void*, int32_t, const int32_t*, const int32_t*, const int32_t*,
                 const float*, const float*, int32_t, const float* const*, const float*, const float*,
                 float* const*, float*, void*, size_t, void*) { return VER_EUNSUPPORTED; }
