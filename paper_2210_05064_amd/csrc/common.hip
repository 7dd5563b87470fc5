#include "common.h"

namespace ver {

__global__ void fill_words_kernel(int32_t* p, size_t n, int32_t v) {
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

void fill_words(int32_t* p, size_t n, int32_t v, hipStream_t s) {
    if (n == 0) return;
    int blocks = (int)((n + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(fill_words_kernel, dim3(blocks), dim3(256), 0, s, p, n, v);
}

}  // namespace ver

extern "C" const char* ver_status_string(int status) {
    switch (status) {
        case VER_OK: return "ok";
        case VER_EINVAL: return "invalid argument";
        case VER_EWORKSPACE: return "workspace missing or too small";
        case VER_EUNSUPPORTED: return "unsupported shape";
        case VER_EHIP: return "HIP call or kernel launch failed";
        default: return "unknown status";
    }
}
