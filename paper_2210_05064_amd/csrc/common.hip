#include "common.h"

#include <vector>

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

uint32_t g_prof_mask = 0;
namespace {
struct ProfRec { int cls; hipEvent_t e0, e1; };
std::vector<ProfRec> g_prof_recs;
std::vector<hipEvent_t> g_prof_pool;
hipEvent_t prof_event() {
    if (!g_prof_pool.empty()) { hipEvent_t e = g_prof_pool.back(); g_prof_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}
}  // namespace

void prof_mark(int cls, bool begin, hipStream_t s) {
    if (begin) {
        ProfRec r{cls, prof_event(), prof_event()};
        (void)hipEventRecord(r.e0, s);
        g_prof_recs.push_back(r);
    } else {
        for (size_t i = g_prof_recs.size(); i-- > 0;)
            if (g_prof_recs[i].cls == cls) { (void)hipEventRecord(g_prof_recs[i].e1, s); break; }
    }
}

}  // namespace ver

extern "C" int ver_profile_enable(uint32_t mask) {
    ver::g_prof_mask = mask;
    return VER_OK;
}

extern "C" int ver_profile_read(double* total_ms, int64_t* launches) {
    if (!total_ms || !launches) return VER_EINVAL;
    for (int i = 0; i < VER_PROF_COUNT; ++i) { total_ms[i] = 0.0; launches[i] = 0; }
    int st = VER_OK;
    for (auto& r : ver::g_prof_recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) st = VER_EHIP;
        total_ms[r.cls] += ms;
        launches[r.cls] += 1;
        ver::g_prof_pool.push_back(r.e0);
        ver::g_prof_pool.push_back(r.e1);
    }
    ver::g_prof_recs.clear();
    return st;
}

extern "C" const char* ver_status_string(int status) {
    switch (status) {
        case VER_OK: return "ok";
        case VER_EINVAL: return "invalid argument";
        case VER_EWORKSPACE: return "workspace missing or too small";
        case VER_EUNSUPPORTED: return "unsupported shape";
        case VER_EHIP: return "HIP call or kernel launch failed";
        case VER_ETOOLARGE: return "input larger than the fixed scratch of this entry point (use the variant that takes a workspace)";
        default: return "unknown status";
    }
}
