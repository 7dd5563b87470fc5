// ver_adam_step: bias-corrected Adam over a list of tensors in ONE launch, with
// the cosine learning rate and optional clipping by the global gradient norm.
//
// Paper: section 4 "Training" and the appendix hyper-parameter table (Adam,
// 2.5e-4 decayed to zero with a cosine schedule); the step itself is Algorithm 1
// of the cited Adam paper.
//
// The step is bound by HBM: per parameter it reads p, g, m, v and writes p, m, v
// (28 bytes).  The tensors are cut into chunks of ADAM_CHUNK elements and every
// workgroup takes one chunk (table of chunk offsets per tensor in the kernel
// arguments), with 16-byte loads and stores; lr, the bias corrections and the
// clip threshold are scalars computed on the host in double precision.  The
// global norm is a two-stage sum of squares (per-chunk partials, then one
// workgroup adds them in index order: deterministic); the update kernel reads
// the resulting scale from the device, so the call never synchronises.
#include <cmath>

#include "common.h"

namespace ver {
namespace {

constexpr int ADAM_THREADS = 256;
constexpr int ADAM_CHUNK = 4096;   // elements per workgroup: 4 x 16 bytes per thread and array
constexpr int ADAM_MAX_CHUNKS = 1 << 20;

struct AdamTensors {
    float* p[VER_ADAM_MAX_TENSORS];
    const float* g[VER_ADAM_MAX_TENSORS];
    float* m[VER_ADAM_MAX_TENSORS];
    float* v[VER_ADAM_MAX_TENSORS];
    long long n[VER_ADAM_MAX_TENSORS];
    float lower[VER_ADAM_MAX_TENSORS], upper[VER_ADAM_MAX_TENSORS];   // box of tensor i (-inf / +inf = none)
    int first_chunk[VER_ADAM_MAX_TENSORS + 1];   // chunks of tensor i: [first_chunk[i], first_chunk[i+1])
    int count;
};

typedef float f4 __attribute__((ext_vector_type(4)));

// Which tensor a chunk belongs to (the table is short: linear search in scalar registers).
__device__ __forceinline__ int tensor_of_chunk(const AdamTensors& t, int chunk) {
    int i = 0;
    while (i + 1 < t.count && chunk >= t.first_chunk[i + 1]) ++i;
    return i;
}

__global__ __launch_bounds__(ADAM_THREADS) void adam_sumsq_kernel(AdamTensors t, float* __restrict__ partial) {
    __shared__ float red[ADAM_THREADS];
    const int chunk = blockIdx.x;
    const int i = tensor_of_chunk(t, chunk);
    const long long lo = (long long)(chunk - t.first_chunk[i]) * ADAM_CHUNK;
    const long long hi = lo + ADAM_CHUNK < t.n[i] ? lo + ADAM_CHUNK : t.n[i];
    const float* g = t.g[i];
    float s = 0.f;
    for (long long e = lo + threadIdx.x * 4; e < hi; e += ADAM_THREADS * 4) {
        if (e + 4 <= hi) {
            const f4 x = *reinterpret_cast<const f4*>(g + e);
            s += (x[0] * x[0] + x[1] * x[1]) + (x[2] * x[2] + x[3] * x[3]);
        } else {
            for (long long k = e; k < hi; ++k) s += g[k] * g[k];
        }
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = ADAM_THREADS / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[chunk] = red[0];
}

// out[0] = sqrt(sum of partials) (the norm), out[1] = min(1, max_norm / (norm + 1e-6)) or 1 without clipping.
__global__ __launch_bounds__(ADAM_THREADS) void adam_norm_kernel(const float* __restrict__ partial, int n, float max_norm,
                                                                  float* __restrict__ norm_out, float* __restrict__ scale) {
    __shared__ double red[ADAM_THREADS];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += ADAM_THREADS) s += (double)partial[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = ADAM_THREADS / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const float norm = (float)sqrt(red[0]);
        if (norm_out) norm_out[0] = norm;
        scale[0] = max_norm > 0.f ? fminf(1.f, max_norm / (norm + 1e-6f)) : 1.f;
    }
}

struct AdamScalars {
    float lr, beta1, beta2, eps;
    float omb1, omb2;       // 1 - beta, formed in double precision (in fp32 the subtraction loses 4 digits)
    float inv_c1, inv_c2;   // 1 / (1 - beta^t)
};

// One element's step, then the projection onto the tensor's box.
__device__ __forceinline__ void adam_elem(float& p, float g, float& m, float& v, const AdamScalars& a, float lower,
                                          float upper) {
    m = a.beta1 * m + a.omb1 * g;
    v = a.beta2 * v + a.omb2 * g * g;
    p -= a.lr * (m * a.inv_c1) / (sqrtf(v * a.inv_c2) + a.eps);
    p = fminf(fmaxf(p, lower), upper);
}

__global__ __launch_bounds__(ADAM_THREADS) void adam_update_kernel(AdamTensors t, AdamScalars a, const float* __restrict__ scale) {
    const int chunk = blockIdx.x;
    const int i = tensor_of_chunk(t, chunk);
    const long long lo = (long long)(chunk - t.first_chunk[i]) * ADAM_CHUNK;
    const long long hi = lo + ADAM_CHUNK < t.n[i] ? lo + ADAM_CHUNK : t.n[i];
    float* p = t.p[i];
    const float* g = t.g[i];
    float* m = t.m[i];
    float* v = t.v[i];
    const float gs = scale ? scale[0] : 1.f;
    const float lower = t.lower[i], upper = t.upper[i];
    for (long long e = lo + threadIdx.x * 4; e < hi; e += ADAM_THREADS * 4) {
        if (e + 4 <= hi) {
            f4 pp = *reinterpret_cast<f4*>(p + e), mm = *reinterpret_cast<f4*>(m + e), vv = *reinterpret_cast<f4*>(v + e);
            const f4 gg = *reinterpret_cast<const f4*>(g + e);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float pk = pp[k], mk = mm[k], vk = vv[k];
                adam_elem(pk, gg[k] * gs, mk, vk, a, lower, upper);
                pp[k] = pk; mm[k] = mk; vv[k] = vk;
            }
            *reinterpret_cast<f4*>(p + e) = pp;
            *reinterpret_cast<f4*>(m + e) = mm;
            *reinterpret_cast<f4*>(v + e) = vv;
        } else {
            for (long long k = e; k < hi; ++k) adam_elem(p[k], g[k] * gs, m[k], v[k], a, lower, upper);
        }
    }
}

}  // namespace
}  // namespace ver

extern "C" size_t ver_adam_workspace_bytes(void) {
    return (size_t)(ver::ADAM_MAX_CHUNKS + 64) * sizeof(float);
}

extern "C" int ver_adam_step(const ver_adam_cfg* cfg, int32_t n_tensors, float* const* params, const float* const* grads,
                             float* const* exp_avg, float* const* exp_avg_sq, const int64_t* sizes, int64_t step_index,
                             float* grad_norm, void* workspace, size_t workspace_bytes, void* stream) {
    return ver_adam_step_bounded(cfg, n_tensors, params, grads, exp_avg, exp_avg_sq, sizes, nullptr, nullptr, step_index,
                                 grad_norm, workspace, workspace_bytes, stream);
}

extern "C" int ver_adam_step_bounded(const ver_adam_cfg* cfg, int32_t n_tensors, float* const* params,
                                     const float* const* grads, float* const* exp_avg, float* const* exp_avg_sq,
                                     const int64_t* sizes, const float* lower, const float* upper, int64_t step_index,
                                     float* grad_norm, void* workspace, size_t workspace_bytes, void* stream) {
    using namespace ver;
    if (!cfg || !params || !grads || !exp_avg || !exp_avg_sq || !sizes) return VER_EINVAL;
    if (n_tensors < 0 || n_tensors > VER_ADAM_MAX_TENSORS || cfg->total_steps <= 0 || step_index < 0) return VER_EINVAL;
    if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f && cfg->beta2 >= 0.f && cfg->beta2 < 1.f && cfg->eps >= 0.f)) return VER_EINVAL;
    const bool clip = cfg->max_grad_norm > 0.f;
    if (clip && !grad_norm) return VER_EINVAL;
    AdamTensors t;
    t.count = 0;
    int chunks = 0;
    for (int i = 0; i < n_tensors; ++i) {
        if (sizes[i] < 0) return VER_EINVAL;
        const float lo = lower ? lower[i] : -INFINITY, hi = upper ? upper[i] : INFINITY;
        if (!(lo <= hi)) return VER_EINVAL;   // also rejects NaN
        if (sizes[i] == 0) continue;
        if (!params[i] || !grads[i] || !exp_avg[i] || !exp_avg_sq[i]) return VER_EINVAL;
        const long long c = (sizes[i] + ADAM_CHUNK - 1) / ADAM_CHUNK;
        if (chunks + c > ADAM_MAX_CHUNKS) return VER_EUNSUPPORTED;
        t.p[t.count] = params[i]; t.g[t.count] = grads[i]; t.m[t.count] = exp_avg[i]; t.v[t.count] = exp_avg_sq[i];
        t.n[t.count] = sizes[i];
        t.lower[t.count] = lo; t.upper[t.count] = hi;
        t.first_chunk[t.count] = chunks;
        chunks += (int)c;
        ++t.count;
    }
    t.first_chunk[t.count] = chunks;
    if (chunks == 0) return VER_OK;
    const bool want_norm = clip || grad_norm;
    if (want_norm && (!workspace || workspace_bytes < ver_adam_workspace_bytes())) return VER_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // scalars of this step, in double precision on the host
    const long long k = step_index < cfg->total_steps ? step_index : cfg->total_steps;
    const double pi = 3.14159265358979323846;
    const double lr = (double)cfg->lr_final +
                      ((double)cfg->lr0 - (double)cfg->lr_final) * 0.5 * (1.0 + cos(pi * (double)k / (double)cfg->total_steps));
    const double tt = (double)(step_index + 1);
    AdamScalars a;
    a.lr = (float)lr; a.beta1 = cfg->beta1; a.beta2 = cfg->beta2; a.eps = cfg->eps;
    a.omb1 = (float)(1.0 - (double)cfg->beta1);
    a.omb2 = (float)(1.0 - (double)cfg->beta2);
    a.inv_c1 = (float)(1.0 / (1.0 - pow((double)cfg->beta1, tt)));
    a.inv_c2 = (float)(1.0 / (1.0 - pow((double)cfg->beta2, tt)));
    ProfScope prof(VER_PROF_ADAM, s);
    float* scale = nullptr;
    if (want_norm) {
        float* partial = static_cast<float*>(workspace);
        scale = partial + ADAM_MAX_CHUNKS;
        hipLaunchKernelGGL(adam_sumsq_kernel, dim3(chunks), dim3(ADAM_THREADS), 0, s, t, partial);
        hipLaunchKernelGGL(adam_norm_kernel, dim3(1), dim3(ADAM_THREADS), 0, s, partial, chunks, cfg->max_grad_norm, grad_norm, scale);
    }
    hipLaunchKernelGGL(adam_update_kernel, dim3(chunks), dim3(ADAM_THREADS), 0, s, t, a, clip ? scale : (const float*)nullptr);
    return launch_status();
}
