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
// What tiles tell each other travels as self-marking 64-bit words (no fences).
// Which steps end an environment is found per tile: two wave-wide searches in
// the offsets for the tile's ends, then the environments in between mark their
// last step in LDS.
// HBM traffic is the algorithmic 17 bytes per step: reward, value, done read
// once (16-byte loads, staged through LDS), advantage and return written once.
#include "common.h"

namespace ver {
namespace {

constexpr int GAE_THREADS = 256;
constexpr int GAE_ITEMS = 8;
constexpr int GAE_TILE = GAE_THREADS * GAE_ITEMS;
constexpr int GAE_LDS = GAE_TILE + GAE_TILE / 8 + 2;   // one unused word after every 8 (see lds_at)
constexpr long long GAE_SPIN_LIMIT = 1LL << 24;  // polls before a wait gives up
constexpr int GAE_MAX_BATCH = 16;      // tiles per ticket at most
constexpr int GAE_BATCH_FROM = 1024;   // one more tile per ticket for every so many tiles

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

// What a tile tells the tiles after it, one 64-bit word per number.  A word carries its own "present" mark:
// 0 (what the workspace is cleared to) means not written yet, anything else is the bits of a double plus one
// (NaNs are made canonical first, so the sum never wraps to 0).  A reader that finds a word non-zero has the
// whole number, whichever order the words arrive in: no flag, no fence, no cache write-back.
struct GaeWs {
    int* ticket;                 // [1]
    int* error;                  // [1]
    unsigned long long* inc;     // [ntiles] advantage leaving the tile towards lower k (final)
    unsigned long long* agg_a;   // [ntiles] the tile's own map, published while inc still waits for the tiles before
    unsigned long long* agg_b;
};
__device__ __forceinline__ unsigned long long word_of(double x) {
    if (x != x) x = __longlong_as_double(0x7FF8000000000000LL);
    return (unsigned long long)__double_as_longlong(x) + 1ull;
}
__device__ __forceinline__ double number_of(unsigned long long w) { return __longlong_as_double((long long)(w - 1ull)); }
__device__ __forceinline__ unsigned long long ld_word(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_word(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ Affine wave_shfl_up(Affine v, int d) {
    return Affine{__shfl_up(v.a, d, VER_WAVE), __shfl_up(v.b, d, VER_WAVE)};
}

// A thread walks 8 consecutive steps, so the lanes of a wave are 8 words apart: with one unused word after
// every 8 they are 9 apart and fall into different LDS banks.
__device__ __forceinline__ int lds_at(int i) { return i + (i >> 3); }

template <bool VEC>
__global__ __launch_bounds__(GAE_THREADS) void gae_kernel(
    const float* __restrict__ rewards, const float* __restrict__ values,
    const uint8_t* __restrict__ dones, const float* __restrict__ last_values,
    const int32_t* __restrict__ env_off, int N, int S, int ntiles, int batch, float gamma, float lambda,
    float* __restrict__ adv, float* __restrict__ ret, GaeWs ws) {
    __shared__ float s_r[GAE_LDS];
    __shared__ float s_v[GAE_LDS];
    __shared__ float s_boot[GAE_LDS];   // value after an environment's last step (only read where s_d says so)
    __shared__ uint8_t s_d[GAE_LDS];    // bit 0: episode ended with this step; bit 1: last step of its environment
    __shared__ Affine s_wave[GAE_THREADS / VER_WAVE];
    __shared__ int s_ticket;
    __shared__ int s_env[2];
    __shared__ double s_carry, s_leaving;

    const int tid = threadIdx.x;
    const int lane = tid & (VER_WAVE - 1), wave = tid / VER_WAVE;
    if (tid == 0) s_ticket = atomicAdd(ws.ticket, 1);
    __syncthreads();
    // A ticket stands for `batch` consecutive tiles, which this workgroup processes one after the other and hands
    // the advantage from one to the next itself (a ticket is an atomic on one address, ~50 ns each across the
    // device: one per 2048 steps would bound the kernel).  Only the first tile of a batch looks back at other
    // workgroups' tiles, namely at the LAST tile of the batch before; so that this one is not the last thing
    // the workgroup before gets to, every workgroup starts with a pass over its last tile that only computes and
    // publishes that tile's map (pass -1; the tile is read once more when its turn comes).
    const int first_tile = s_ticket * batch, n_here = min(batch, ntiles - first_tile);
    double carry_known = 0.0;   // advantage entering the next tile of the batch (valid from its second tile on)
    for (int pass = n_here > 1 ? -1 : 0; pass < n_here; ++pass) {
    const bool map_only = pass < 0;
    const int tile = first_tile + (map_only ? n_here - 1 : pass);
    // Tiles are processed from the END of the buffer: tile number `tile` covers flat steps [k_lo, k_lo + count);
    // tile boundaries are multiples of the tile size from the start, so every tile but the first one
    // processed is whole and all of them start on an aligned address.
    const int k_lo = (ntiles - 1 - tile) * GAE_TILE;
    const int count = min(GAE_TILE, S - k_lo);
    const int k_hi = k_lo + count - 1;

    // environments of the tile's first and last step
    if (wave < 2) {
        const int e = segment_of_wave(env_off, N, wave == 0 ? k_lo : k_hi);
        if (lane == 0) s_env[wave] = e;
    }
    for (int i = tid * 4; i < count; i += GAE_THREADS * 4) {
        if (VEC && i + 4 <= count) {
            const float4 r4 = *reinterpret_cast<const float4*>(rewards + k_lo + i);
            const float4 v4 = *reinterpret_cast<const float4*>(values + k_lo + i);
            const uint32_t d4 = *reinterpret_cast<const uint32_t*>(dones + k_lo + i);
            const int q = lds_at(i);
            s_r[q] = r4.x; s_r[q + 1] = r4.y; s_r[q + 2] = r4.z; s_r[q + 3] = r4.w;
            s_v[q] = v4.x; s_v[q + 1] = v4.y; s_v[q + 2] = v4.z; s_v[q + 3] = v4.w;
            s_d[q] = (d4 & 0xFFu) ? 1 : 0; s_d[q + 1] = (d4 & 0xFF00u) ? 1 : 0;
            s_d[q + 2] = (d4 & 0xFF0000u) ? 1 : 0; s_d[q + 3] = (d4 & 0xFF000000u) ? 1 : 0;
        } else {
            for (int j = i; j < min(i + 4, count); ++j) {
                s_r[lds_at(j)] = rewards[k_lo + j];
                s_v[lds_at(j)] = values[k_lo + j];
                s_d[lds_at(j)] = dones[k_lo + j] ? 1 : 0;
            }
        }
    }
    if (tid == 0) s_v[lds_at(count)] = (k_hi + 1 < S) ? values[k_hi + 1] : 0.f;
    __syncthreads();
    // mark the last step of every environment that ends inside the tile and fetch its bootstrap value
    for (int e = s_env[0] + tid; e <= s_env[1]; e += GAE_THREADS) {
        const int lo = env_off[e], hi = env_off[e + 1];
        const int i = hi - 1 - k_lo;
        if (hi > lo && i >= 0 && i < count) {
            s_d[lds_at(i)] |= 2;
            s_boot[lds_at(i)] = last_values[e];
        }
    }
    __syncthreads();

    // Thread tid handles the steps top, top-1, ... of the tile (processing order = time descending).
    const int top = count - 1 - tid * GAE_ITEMS;
    double a[GAE_ITEMS], b[GAE_ITEMS];
    Affine mine{1.0, 0.0};
    const double gl = (double)gamma * (double)lambda;
#pragma unroll
    for (int i = 0; i < GAE_ITEMS; ++i) {
        const int idx = top - i;
        a[i] = 1.0;
        b[i] = 0.0;
        if (idx >= 0) {
            const int q = lds_at(idx);
            const int f = s_d[q];
            const bool last = (f & 2) != 0;
            const double nd = (f & 1) ? 0.0 : 1.0;
            const double v_next = last ? s_boot[q] : s_v[lds_at(idx + 1)];
            a[i] = last ? 0.0 : gl * nd;
            b[i] = (double)s_r[q] + (double)gamma * nd * v_next - (double)s_v[q];
            mine = compose(mine, Affine{a[i], b[i]});
        }
    }

    // Exclusive scan of the per-thread maps over the tile (thread order = processing order).
    Affine incl = mine;
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
        const bool cut = tile == 0 || tile_map.a == 0.0;   // incoming value is 0 or irrelevant
        if (lane == 0) {
            if (cut) {
                st_word(&ws.inc[tile], word_of(tile_map.b));
            } else {
                st_word(&ws.agg_a[tile], word_of(tile_map.a));
                st_word(&ws.agg_b[tile], word_of(tile_map.b));
            }
        }
        double carry = pass > 0 ? carry_known : 0.0;  // advantage entering this tile (from step k_hi + 1)
        if (!map_only && pass == 0 && tile > 0) {  // needed even when the tile is cut: its steps before the cut still see the carry
            Affine back{1.0, 0.0};  // carry = back.b + back.a * (value entering the window's far end)
            int j0 = tile - 1;
            bool failed = false;
            while (j0 >= 0 && back.a != 0.0 && !failed) {
                // Lane l looks at tile j0 - l.  The wait ends as soon as some lane holds a map with a = 0 (a final
                // value, or a tile cut by an episode or environment end) and every nearer lane holds its map:
                // what lies beyond a cut cannot matter, so tiles that are still far from done are not waited for.
                const int j = j0 - lane;
                Affine m{0.0, 0.0};   // beyond the first tile processed the advantage is 0
                bool ready = j < 0;
                long long spins = 0;
                for (;;) {
                    if (!ready) {
                        const unsigned long long wi = ld_word(&ws.inc[j]);
                        if (wi) {
                            m = Affine{0.0, number_of(wi)};
                            ready = true;
                        } else {
                            const unsigned long long wa = ld_word(&ws.agg_a[j]), wb = ld_word(&ws.agg_b[j]);
                            if (wa && wb) {
                                m = Affine{number_of(wa), number_of(wb)};
                                ready = true;
                            }
                        }
                    }
                    const unsigned long long have = __ballot(ready), cuts = __ballot(ready && m.a == 0.0);
                    if (cuts) {
                        const int c = __ffsll((long long)cuts) - 1;             // nearest cut
                        const unsigned long long nearer = (1ull << c) - 1ull;
                        if ((have & nearer) == nearer) {
                            if (lane > c) m = Affine{1.0, 0.0};
                            break;
                        }
                    } else if (have == ~0ull) {
                        break;
                    }
                    if (++spins > GAE_SPIN_LIMIT || ld_agent(ws.error) != 0) { failed = true; break; }
                    __builtin_amdgcn_s_sleep(1);
                }
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
        }
        if (lane == 0 && !map_only) {
            const double leaving = cut ? tile_map.b : tile_map.b + tile_map.a * carry;
            if (!cut) st_word(&ws.inc[tile], word_of(leaving));
            s_carry = carry;
            s_leaving = leaving;
        }
    }
    __syncthreads();
    if (map_only) continue;   // (uniform; the barrier above also protects the LDS arrays that the next pass refills)
    carry_known = s_leaving;

    double x = before.b + before.a * s_carry;  // advantage at the step after this thread's first
#pragma unroll
    for (int i = 0; i < GAE_ITEMS; ++i) {
        const int idx = top - i;
        if (idx >= 0) {
            x = b[i] + a[i] * x;
            const int q = lds_at(idx);
            const float v = s_v[q];
            s_r[q] = (float)x;
            s_boot[q] = (float)(x + (double)v);
        }
    }
    __syncthreads();
    for (int i = tid * 4; i < count; i += GAE_THREADS * 4) {
        if (VEC && i + 4 <= count) {
            const int q = lds_at(i);
            *reinterpret_cast<float4*>(adv + k_lo + i) = float4{s_r[q], s_r[q + 1], s_r[q + 2], s_r[q + 3]};
            *reinterpret_cast<float4*>(ret + k_lo + i) = float4{s_boot[q], s_boot[q + 1], s_boot[q + 2], s_boot[q + 3]};
        } else {
            for (int j = i; j < min(i + 4, count); ++j) {
                adv[k_lo + j] = s_r[lds_at(j)];
                ret[k_lo + j] = s_boot[lds_at(j)];
            }
        }
    }
    __syncthreads();   // the arrays are refilled by the next tile of the batch
    }
}

inline int gae_tiles(int S) { return (S + GAE_TILE - 1) / GAE_TILE; }
inline int gae_batch(int tiles) {
    const int b = tiles / GAE_BATCH_FROM;
    return b < 1 ? 1 : (b > GAE_MAX_BATCH ? GAE_MAX_BATCH : b);
}

}  // namespace
}  // namespace ver

extern "C" size_t ver_gae_workspace_bytes(int32_t S) {
    if (S < 0) return 0;
    size_t t = (size_t)ver::gae_tiles(S);
    return 256 + 3 * ver::align_up(t * 8, 256);
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
    ws.inc = cv.take<unsigned long long>(tiles);
    ws.agg_a = cv.take<unsigned long long>(tiles);
    ws.agg_b = cv.take<unsigned long long>(tiles);
    // ticket, error and every published word must start at zero (the blocks are adjacent)
    ver::fill_words(reinterpret_cast<int32_t*>(head), cv.used / 4, 0, s);
    ver::ProfScope prof(VER_PROF_GAE, s);
    // 16-byte accesses need 16-byte aligned arrays (tiles start at multiples of the tile size)
    const uintptr_t bits = reinterpret_cast<uintptr_t>(rewards) | reinterpret_cast<uintptr_t>(values) |
                           reinterpret_cast<uintptr_t>(adv) | reinterpret_cast<uintptr_t>(ret) |
                           (reinterpret_cast<uintptr_t>(dones) << 2);
    // tiles per ticket: 1 while tickets are few, up to GAE_MAX_BATCH for buffers of many thousands of tiles
    const int batch = ver::gae_batch(tiles), groups = (tiles + batch - 1) / batch;
    if ((bits & 15) == 0)
        hipLaunchKernelGGL(ver::gae_kernel<true>, dim3(groups), dim3(ver::GAE_THREADS), 0, s, rewards, values, dones,
                           last_values, env_off, N, S, tiles, batch, gamma, lambda, adv, ret, ws);
    else
        hipLaunchKernelGGL(ver::gae_kernel<false>, dim3(groups), dim3(ver::GAE_THREADS), 0, s, rewards, values, dones,
                           last_values, env_off, N, S, tiles, batch, gamma, lambda, adv, ret, ws);
    return ver::launch_status();
}
