// ver_gae: advantages and value targets over the ragged rollout buffer.
//
// Paper: section 4 "Training" (PPO with Generalized Advantage Estimation,
// gamma/lambda from the hyper-parameter table) applied to the ragged
// per-environment stretches of section 2.2.
//
// The recurrence adv_k = delta_k + c_k * adv_{k+1} is an affine map per step,
// x -> b_k + a_k * x with a_k = gamma*lambda*(1-done_k) (0 at the last step of
// an environment) and b_k = delta_k.  Composition of affine maps is
// associative, so the whole flat buffer is ONE reverse scan; episode ends and
// environment ends simply have a_k = 0.  The scan is single-pass: tiles take
// tickets in launch order, publish their aggregate map, and look back over the
// tiles with lower tickets (which are running or finished, so every wait ends).
// HBM traffic is the algorithmic 17 bytes per step: reward, value, done read
// once (coalesced, staged through LDS), advantage and return written once.
#include "common.h"

namespace ver {
namespace {

constexpr int GAE_THREADS = 256;
constexpr int GAE_ITEMS = 8;
constexpr int GAE_TILE = GAE_THREADS * GAE_ITEMS;
constexpr long long GAE_SPIN_LIMIT = 1LL << 24;  // polls before a wait gives up

// The maps are composed in fp64: the kernel is HBM bound, fp64 costs nothing here,
// and the fp32 outputs then carry one rounding instead of an error that grows
// with the length of the episode (returns = advantage + value cancels heavily
// when the critic is far from the returns).
struct Affine {
    double a, b;  // x -> b + a * x
};
// `first` is applied to the incoming value first (it is later in time), `then` after it.
__device__ __forceinline__ Affine compose(Affine first, Affine then) {
    return Affine{then.a * first.a, then.b + then.a * first.b};
}

struct GaeWs {
    int* ticket;   // [1]
    int* error;    // [1]
    int* flag;     // [ntiles] 0 = nothing, 1 = aggregate, 2 = inclusive value
    double* agg_a;  // [ntiles]
    double* agg_b;  // [ntiles]
    double* inc;    // [ntiles] advantage leaving the tile towards lower k
};

__device__ __forceinline__ Affine wave_shfl_up(Affine v, int d) {
    return Affine{__shfl_up(v.a, d, VER_WAVE), __shfl_up(v.b, d, VER_WAVE)};
}
__device__ __forceinline__ double ld_agent64(const double* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent64(double* p, double v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(GAE_THREADS) void gae_kernel(
    const float* __restrict__ rewards, const float* __restrict__ values,
    const uint8_t* __restrict__ dones, const float* __restrict__ last_values,
    const int32_t* __restrict__ env_off, int N, int S, float gamma, float lambda,
    float* __restrict__ adv, float* __restrict__ ret, GaeWs ws) {
    __shared__ float s_r[GAE_TILE];
    __shared__ float s_v[GAE_TILE + 1];
    __shared__ uint8_t s_d[GAE_TILE];
    __shared__ Affine s_wave[GAE_THREADS / VER_WAVE];
    __shared__ int s_tile;
    __shared__ double s_carry;

    const int tid = threadIdx.x;
    if (tid == 0) s_tile = atomicAdd(ws.ticket, 1);
    __syncthreads();
    const int tile = s_tile;
    // The tile covers flat steps [k_lo, k_hi]; tile 0 is the END of the buffer.
    const int k_hi = S - 1 - tile * GAE_TILE;
    const int k_lo = max(0, k_hi - GAE_TILE + 1);
    const int count = k_hi - k_lo + 1;

    for (int i = tid; i < count; i += GAE_THREADS) {
        s_r[i] = rewards[k_lo + i];
        s_v[i] = values[k_lo + i];
        s_d[i] = dones[k_lo + i];
    }
    if (tid == 0) s_v[count] = (k_hi + 1 < S) ? values[k_hi + 1] : 0.f;
    __syncthreads();

    // Thread tid handles k_top, k_top-1, ... (processing order = time descending).
    const int k_top = k_hi - tid * GAE_ITEMS;
    double a[GAE_ITEMS], b[GAE_ITEMS];
    Affine mine{1.0, 0.0};
    const double gl = (double)gamma * (double)lambda;
    int env = 0;
    if (k_top >= k_lo) env = segment_of(env_off, N, k_top);
#pragma unroll
    for (int i = 0; i < GAE_ITEMS; ++i) {
        const int k = k_top - i;
        a[i] = 1.0;
        b[i] = 0.0;
        if (k >= k_lo) {
            while (k < env_off[env]) --env;
            const int idx = k - k_lo;
            const bool last = (k + 1 == env_off[env + 1]);
            const double nd = s_d[idx] ? 0.0 : 1.0;
            const double v_next = last ? last_values[env] : s_v[idx + 1];
            a[i] = last ? 0.0 : gl * nd;
            b[i] = (double)s_r[idx] + (double)gamma * nd * v_next - (double)s_v[idx];
            mine = compose(mine, Affine{a[i], b[i]});
        }
    }

    // Exclusive scan of the per-thread maps over the tile (thread order = processing order).
    Affine incl = mine;
    const int lane = tid & (VER_WAVE - 1), wave = tid / VER_WAVE;
#pragma unroll
    for (int d = 1; d < VER_WAVE; d <<= 1) {
        Affine up = wave_shfl_up(incl, d);
        if (lane >= d) incl = compose(up, incl);
    }
    if (lane == VER_WAVE - 1) s_wave[wave] = incl;
    __syncthreads();
    Affine before{1.0, 0.0};  // everything in the tile processed before this thread
    for (int w = 0; w < wave; ++w) before = compose(before, s_wave[w]);
    Affine excl_in_wave = wave_shfl_up(incl, 1);
    if (lane > 0) before = compose(before, excl_in_wave);

    // Chained scan across tiles (wave 0).
    if (wave == 0) {
        Affine tile_map{1.0, 0.0};
        for (int w = 0; w < GAE_THREADS / VER_WAVE; ++w) tile_map = compose(tile_map, s_wave[w]);
        if (lane == 0) {
            if (tile == 0 || tile_map.a == 0.0) {
                st_agent64(&ws.inc[tile], tile_map.b);  // incoming value is 0 or irrelevant
                fence_release();
                st_agent(&ws.flag[tile], 2);
            } else {
                st_agent64(&ws.agg_a[tile], tile_map.a);
                st_agent64(&ws.agg_b[tile], tile_map.b);
                fence_release();
                st_agent(&ws.flag[tile], 1);
            }
        }
        double carry = 0.0;  // advantage entering this tile (from step k_hi + 1)
        if (tile > 0) {  // needed even when tile_map.a == 0: steps before the cut still see the carry
            Affine back{1.0, 0.0};  // carry = back.b + back.a * (value entering the window's far end)
            int j0 = tile - 1;
            bool failed = false;
            while (j0 >= 0 && back.a != 0.0 && !failed) {
                const int j = j0 - lane;
                Affine m{1.0, 0.0};
                if (j >= 0) {
                    int f = 0;
                    long long spins = 0;
                    while ((f = ld_agent(&ws.flag[j])) == 0) {
                        if (++spins > GAE_SPIN_LIMIT || ld_agent(ws.error) != 0) { failed = true; break; }
                        __builtin_amdgcn_s_sleep(1);
                    }
                    fence_acquire();
                    if (f == 2) m = Affine{0.0, ld_agent64(&ws.inc[j])};
                    else if (f == 1) m = Affine{ld_agent64(&ws.agg_a[j]), ld_agent64(&ws.agg_b[j])};
                }
                failed = __any(failed);
                // lane 0 is the nearest tile: it is applied LAST, so scan with "nearer then".
                Affine win = m;
#pragma unroll
                for (int d = 1; d < VER_WAVE; d <<= 1) {
                    Affine up = wave_shfl_up(win, d);  // nearer tiles
                    if (lane >= d) win = compose(win, up);
                }
                Affine whole{__shfl(win.a, VER_WAVE - 1, VER_WAVE), __shfl(win.b, VER_WAVE - 1, VER_WAVE)};
                back = compose(whole, back);
                j0 -= VER_WAVE;
            }
            if (failed && lane == 0) st_agent(ws.error, 1);
            carry = back.b;  // beyond tile 0 the incoming advantage is 0
            if (lane == 0 && tile_map.a != 0.0) {
                st_agent64(&ws.inc[tile], tile_map.b + tile_map.a * carry);
                fence_release();
                st_agent(&ws.flag[tile], 2);
            }
        }
        if (lane == 0) s_carry = carry;
    }
    __syncthreads();

    double x = before.b + before.a * s_carry;  // advantage at step k_top + 1
#pragma unroll
    for (int i = 0; i < GAE_ITEMS; ++i) {
        const int k = k_top - i;
        if (k >= k_lo) {
            x = b[i] + a[i] * x;
            const int idx = k - k_lo;
            const float v = s_v[idx];
            s_r[idx] = (float)x;
            s_v[idx] = (float)(x + (double)v);  // only this thread reads s_v[idx] from here on
        }
    }
    __syncthreads();
    for (int i = tid; i < count; i += GAE_THREADS) {
        adv[k_lo + i] = s_r[i];
        ret[k_lo + i] = s_v[i];
    }
}

inline int gae_tiles(int S) { return (S + GAE_TILE - 1) / GAE_TILE; }

}  // namespace
}  // namespace ver

extern "C" size_t ver_gae_workspace_bytes(int32_t S) {
    if (S < 0) return 0;
    size_t t = (size_t)ver::gae_tiles(S);
    return 256 + ver::align_up(t * 4, 256) + 3 * ver::align_up(t * 8, 256);
}

extern "C" int ver_gae(const float* rewards, const float* values, const uint8_t* dones,
                       const float* last_values, const int32_t* env_off, int32_t N, int32_t S,
                       float gamma, float lambda, float* adv, float* ret,
                       void* workspace, size_t workspace_bytes, void* stream) {
    if (N < 0 || S < 0) return VER_EINVAL;
    if (S == 0) return VER_OK;
    if (!rewards || !values || !dones || !last_values || !env_off || !adv || !ret || N == 0) return VER_EINVAL;
    if (!workspace || workspace_bytes < ver_gae_workspace_bytes(S)) return VER_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int tiles = ver::gae_tiles(S);
    ver::Carver cv(workspace);
    int* head = cv.take<int>(64);
    ver::GaeWs ws;
    ws.ticket = head;
    ws.error = head + 1;
    ws.flag = cv.take<int>(tiles);
    ws.agg_a = cv.take<double>(tiles);
    ws.agg_b = cv.take<double>(tiles);
    ws.inc = cv.take<double>(tiles);
    // ticket, error and flags must start at zero: head block + flag block are adjacent
    ver::fill_words(reinterpret_cast<int32_t*>(head), 64 + ver::align_up((size_t)tiles * 4, 256) / 4, 0, s);
    ver::ProfScope prof(VER_PROF_GAE, s);
    hipLaunchKernelGGL(ver::gae_kernel, dim3(tiles), dim3(ver::GAE_THREADS), 0, s, rewards, values, dones,
                       last_values, env_off, N, S, gamma, lambda, adv, ret, ws);
    return ver::launch_status();
}
