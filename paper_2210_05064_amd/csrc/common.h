// Shared host/device helpers of the VER learner kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/ver.h"

#define VER_WAVE 64

namespace ver {

inline int launch_status() {
    return hipGetLastError() == hipSuccess ? VER_OK : VER_EHIP;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Bump allocator over a caller-provided workspace; every block 256-byte aligned.
struct Carver {
    char* base;
    size_t used;
    explicit Carver(void* p) : base(static_cast<char*>(p)), used(0) {}
    template <typename T>
    T* take(size_t n) {
        T* p = reinterpret_cast<T*>(base + used);
        used += align_up(n * sizeof(T), 256);
        return p;
    }
};

// Loads/stores that are coherent across the whole device (all XCDs): used for
// data exchanged between workgroups inside one kernel.
__device__ __forceinline__ int ld_agent(const int* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(int* p, int v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void fence_release() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }
__device__ __forceinline__ void fence_acquire() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); }

// Largest i in [0, n) with off[i] <= k, given off[0] <= k < off[n] (off non-decreasing).
__device__ __forceinline__ int segment_of(const int32_t* __restrict__ off, int n, int k) {
    int lo = 0, hi = n;  // invariant: off[lo] <= k < off[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (off[mid] <= k) lo = mid; else hi = mid;
    }
    return lo;
}

// Largest e in [0, n) with off[e] <= k (off non-decreasing, off[0] <= k), found by the whole wave: every
// round the 64 lanes probe 64 evenly spaced offsets and a ballot keeps one interval (4 dependent loads for a
// million environments instead of 20).
__device__ __forceinline__ int segment_of_wave(const int32_t* __restrict__ off, int n, int k) {
    const int lane = threadIdx.x & (VER_WAVE - 1);
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int step = (hi - lo + VER_WAVE - 1) / VER_WAVE;
        const int p = lo + lane * step;
        const bool le = p < hi && off[p] <= k;
        const int c = max(1, (int)__popcll(__ballot(le)));   // lanes 0 .. c-1 (lane 0 probes lo, which holds by the invariant)
        lo += (c - 1) * step;
        hi = min(hi, lo + step);
    }
    return lo;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding global
// load and store of the wave, which would put the latency of each prefetch on the critical path; code that
// uses it waits for global memory explicitly where it needs it.
__device__ __forceinline__ void bar_lds() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Fills n 32-bit words with v (used instead of memset nodes so that callers may
// capture the stream into a graph).
__global__ void fill_words_kernel(int32_t* p, size_t n, int32_t v);
void fill_words(int32_t* p, size_t n, int32_t v, hipStream_t s);

// Optional event bracketing of kernel classes (see ver_profile_enable).
extern uint32_t g_prof_mask;
void prof_mark(int cls, bool begin, hipStream_t s);
struct ProfScope {
    int cls; hipStream_t s; bool on;
    ProfScope(int c, hipStream_t st) : cls(c), s(st), on((g_prof_mask >> c) & 1u) { if (on) prof_mark(cls, true, s); }
    ~ProfScope() { if (on) prof_mark(cls, false, s); }
};

}  // namespace ver
