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
// once, advantage and return written once, by the thread that works on the 8
// consecutive steps, 16 bytes at a time (nothing is staged through LDS).
#include <mutex>
#include <type_traits>

#include "common.h"

namespace ver {
namespace {

constexpr int GAE_THREADS = 256;
constexpr int GAE_ITEMS = 8;
constexpr int GAE_TILE = GAE_THREADS * GAE_ITEMS;
constexpr long long GAE_SPIN_LIMIT = 1LL << 24;  // polls before a wait gives up
constexpr int GAE_MAX_BATCH = 64;      // tiles per ticket at most (measured on 65536 tiles: 16 -> 0.516 ms, 32 -> 0.506, 64 -> 0.499)
constexpr int GAE_BATCH_FROM = 1024;   // one more tile per ticket for every so many tiles

// A map's offset b is kept in fp64 everywhere: advantages are sums of TD errors that cancel heavily (with
// lambda = 1 they telescope to a discounted reward sum minus a value), so an fp32 sum of a thousand terms of size 1
// leaves an error of 1e-5 of a return of size 0.1; fp64 sums leave the fp32 outputs with one rounding.  Inside a
// tile the slope a (a product of at most 2048 factors gamma * lambda, or 0) is fp32: its rounding, a random walk
// of ~3e-6 relative at most, scales what enters from above only.  From tile to tile both travel as fp64.
struct Affine {
    double a, b;  // x -> b + a * x
};
struct AffineF {
    float a;
    double b;
};
// `first` is applied to the incoming value first (it is later in time), `then` after it.
__device__ __forceinline__ Affine compose(Affine first, Affine then) {
    return Affine{then.a * first.a, then.b + then.a * first.b};
}
__device__ __forceinline__ AffineF compose(AffineF first, AffineF then) {
    return AffineF{then.a * first.a, fma((double)then.a, first.b, then.b)};
}
// The value `v` of the lane that a data-parallel-primitive control selects, `idle` where it selects none: the wave
// scan below moves maps between lanes with these (register-to-register) instead of through the LDS crossbar.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp(float idle, float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(idle), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ AffineF dpp_map(AffineF v) {   // lanes the control leaves out get the identity map
    const unsigned long long bits = (unsigned long long)__double_as_longlong(v.b);
    const float lo = dpp<CTRL, ROW_MASK>(0.f, __uint_as_float((unsigned)bits));
    const float hi = dpp<CTRL, ROW_MASK>(0.f, __uint_as_float((unsigned)(bits >> 32)));
    const unsigned long long moved = ((unsigned long long)__float_as_uint(hi) << 32) | __float_as_uint(lo);
    return AffineF{dpp<CTRL, ROW_MASK>(1.f, v.a), __longlong_as_double((long long)moved)};
}
constexpr int DPP_ROW_SHR = 0x110;      // + n: lane i of a row of 16 reads lane i - n of its row
constexpr int DPP_WAVE_SHR1 = 0x138;    // lane i reads lane i - 1 of the wave
constexpr int DPP_ROW_BCAST15 = 0x142;  // lane 15 of every row to all lanes of the next row
constexpr int DPP_ROW_BCAST31 = 0x143;  // lane 31 to all lanes of rows 2 and 3

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
// Inclusive scan of the wave's maps in lane order (lane l's map is applied after those of the lanes below it).
__device__ __forceinline__ AffineF wave_scan(AffineF m) {
    m = compose(dpp_map<DPP_ROW_SHR + 1, 0xf>(m), m);
    m = compose(dpp_map<DPP_ROW_SHR + 2, 0xf>(m), m);
    m = compose(dpp_map<DPP_ROW_SHR + 4, 0xf>(m), m);
    m = compose(dpp_map<DPP_ROW_SHR + 8, 0xf>(m), m);     // every row of 16 lanes is scanned
    m = compose(dpp_map<DPP_ROW_BCAST15, 0xa>(m), m);     // rows 1 and 3 take in the whole row below
    m = compose(dpp_map<DPP_ROW_BCAST31, 0xc>(m), m);     // rows 2 and 3 take in the lower half of the wave
    return m;
}

static_assert(GAE_ITEMS == 8, "a thread's group of steps: two 16-byte loads per array, one 64-bit word of flags");

template <bool VEC>
__global__ __launch_bounds__(GAE_THREADS) void gae_kernel(
    const float* __restrict__ rewards, const float* __restrict__ values,
    const uint8_t* __restrict__ dones, const float* __restrict__ last_values,
    const int32_t* __restrict__ env_off, int N, int S, int ntiles, int batch, float gamma, float lambda,
    float* __restrict__ adv, float* __restrict__ ret, GaeWs ws) {
    // The tile's steps never pass through LDS: a thread reads the 8 consecutive steps it works on straight into
    // registers (two 16-byte loads per array) and writes its 8 results the same way.  LDS only holds which steps
    // end an environment, and the value after such a step.
    __shared__ float s_boot[GAE_TILE];   // value after an environment's last step (only read where s_last says so)
    __shared__ __attribute__((aligned(8))) uint8_t s_last[GAE_TILE + 8];   // byte i: non-zero if step i of the tile is the last of its environment
    __shared__ AffineF s_wave[GAE_THREADS / VER_WAVE];
    __shared__ int s_ticket;
    __shared__ double s_carry, s_leaving;

    const int tid = threadIdx.x;
    const int lane = tid & (VER_WAVE - 1), wave = tid / VER_WAVE;
    if (tid == 0) s_ticket = atomicAdd(ws.ticket, 1);
    *reinterpret_cast<unsigned long long*>(s_last + tid * 8) = 0ull;   // (every reader clears what it has read)
    if (tid == 0) *reinterpret_cast<unsigned long long*>(s_last + GAE_TILE) = 0ull;
    __syncthreads();
    // A ticket stands for `batch` consecutive tiles, which this workgroup processes one after the other and hands
    // the advantage from one to the next itself (a ticket is an atomic on one address, ~50 ns each across the
    // device: one per 2048 steps would bound the kernel).  Only the first tile of a batch looks back at other
    // workgroups' tiles, namely at the LAST tile of the batch before; so that this one is not the last thing
    // the workgroup before gets to, every workgroup starts with a pass over its last tile that only computes and
    // publishes that tile's map (pass -1; the tile is read once more when its turn comes).
    const int first_tile = s_ticket * batch, n_here = min(batch, ntiles - first_tile);
    double carry_known = 0.0;   // advantage entering the next tile of the batch (valid from its second tile on)
    const int pass0 = n_here > 1 ? -1 : 0;
    int env_first_above = 0;   // first environment of the tile of the pass before
    // One pass over one tile.  FULL (a compile-time flag): the tile is whole and the arrays allow 16-byte accesses,
    // so every thread has a whole group and no step needs a validity check: all tiles but the buffer's ragged
    // last one.  (The checks cost a third of the kernel's vector instructions and a hundred branches.)
    auto do_pass = [&](int pass, auto full_flag) {
    constexpr bool FULL = decltype(full_flag)::value;
    const bool map_only = pass < 0;
    const int tile = first_tile + (map_only ? n_here - 1 : pass);
    // Tiles are processed from the END of the buffer: tile number `tile` covers flat steps [k_lo, k_lo + count);
    // tile boundaries are multiples of the tile size from the start, so every tile but the first one
    // processed is whole and all of them start on an aligned address.
    const int k_lo = (ntiles - 1 - tile) * GAE_TILE;
    const int count = FULL ? GAE_TILE : min(GAE_TILE, S - k_lo);
    const int k_hi = k_lo + count - 1;

    // Thread tid handles group n_groups - 1 - tid of 8 consecutive steps, from its last step down (processing
    // order = time descending; the topmost group of a ragged tile is short).
    const int group = ((count + 7) >> 3) - 1 - tid;
    const int g0 = group * 8;                      // the group's first step inside the tile
    const bool whole = FULL || (VEC && group >= 0 && g0 + 8 <= count);
    // (Fetching the next tile's steps a pass ahead into a second set of registers was measured: no faster, the
    // registers cost a wave per SIMD.)
    float r8[GAE_ITEMS], v8[GAE_ITEMS];
    uint32_t d_lo = 0, d_hi = 0;                   // the 8 done bytes
    float v_after = 0.f;                           // value of the step after the group's last one (0 beyond the buffer)
    if (whole) {
        const float4 ra = *reinterpret_cast<const float4*>(rewards + k_lo + g0), rb = *reinterpret_cast<const float4*>(rewards + k_lo + g0 + 4);
        const float4 va = *reinterpret_cast<const float4*>(values + k_lo + g0), vb = *reinterpret_cast<const float4*>(values + k_lo + g0 + 4);
        d_lo = *reinterpret_cast<const uint32_t*>(dones + k_lo + g0);
        d_hi = *reinterpret_cast<const uint32_t*>(dones + k_lo + g0 + 4);
        r8[0] = ra.x; r8[1] = ra.y; r8[2] = ra.z; r8[3] = ra.w; r8[4] = rb.x; r8[5] = rb.y; r8[6] = rb.z; r8[7] = rb.w;
        v8[0] = va.x; v8[1] = va.y; v8[2] = va.z; v8[3] = va.w; v8[4] = vb.x; v8[5] = vb.y; v8[6] = vb.z; v8[7] = vb.w;
    } else {
#pragma unroll
        for (int j = 0; j < GAE_ITEMS; ++j) {
            r8[j] = v8[j] = 0.f;
            if (!FULL && group >= 0 && g0 + j < count) {
                r8[j] = rewards[k_lo + g0 + j];
                v8[j] = values[k_lo + g0 + j];
                const uint32_t d = dones[k_lo + g0 + j] ? 1u : 0u;
                if (j < 4) d_lo |= d << (8 * j); else d_hi |= d << (8 * (j - 4));
            }
        }
    }
    if (FULL) {
        // the step after this thread's group is the first step of the group of the lane before: taken from its
        // register; only the first lane of a wave fetches it (the first thread of the tile from the tile above)
        if (lane == 0 && k_lo + g0 + 8 < S) v_after = values[k_lo + g0 + 8];
        const float from_lane_before = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v8[0]), DPP_WAVE_SHR1, 0xf, 0xf, false));
        if (lane != 0) v_after = from_lane_before;
    } else if (group >= 0 && k_lo + g0 + 8 < S) {
        v_after = values[k_lo + g0 + 8];
    }

    // Which steps of the tile end an environment (wave 0; the loads above are in flight meanwhile).  Environments
    // of the tile's first and last step: from the second tile of a batch on they follow from the tile before (the
    // one just above in memory): that tile's first environment bounds this one's last, and this one's first is
    // found by walking down from there, 64 offsets at a time (one round of loads instead of four dependent ones).
    if (wave == 0) {
        int e, e_hi;
        if (pass >= 1) {
            e = e_hi = env_first_above;
            for (;;) {
                const int probe = e - lane;
                const unsigned long long ok = __ballot(probe >= 0 && env_off[probe] <= k_lo);   // monotone in the lane
                if (ok) { e -= __ffsll((long long)ok) - 1; break; }
                e -= VER_WAVE;
                if (e < 0) { e = 0; break; }   // (env_off[0] = 0 ends the walk before this; malformed input must not run away)
            }
        } else {
            e = segment_of_wave(env_off, N, k_lo);
            e_hi = segment_of_wave(env_off, N, k_hi);
        }
        env_first_above = e;
        // mark the last step of every environment that ends inside the tile and keep its bootstrap value
        for (int m = e + lane; m <= e_hi; m += VER_WAVE) {
            const int lo = env_off[m], hi = env_off[m + 1];
            const int i = hi - 1 - k_lo;
            if (hi > lo && i >= 0 && i < count) {
                s_last[i] = 1;
                s_boot[i] = last_values[m];
            }
        }
    }
    bar_lds();
    uint32_t l_lo = 0, l_hi = 0;   // the 8 bytes of s_last
    if (FULL || group >= 0) {
        const unsigned long long lasts = *reinterpret_cast<const unsigned long long*>(s_last + g0);
        if (lasts) *reinterpret_cast<unsigned long long*>(s_last + g0) = 0ull;   // clean for the next tile
        l_lo = (uint32_t)lasts;
        l_hi = (uint32_t)(lasts >> 32);
    }

    const double gl = (double)gamma * (double)lambda;
    const float glf = (float)gl;
    // the map of step g0 + 7 - i; across the scan a thread keeps the b of its 8 maps and one bit for each a
    // (which is either 0 or gamma * lambda)
    AffineF mine{1.f, 0.0};
    double b_of[GAE_ITEMS];
    unsigned a_zero = 0;
#pragma unroll
    for (int i = 0; i < GAE_ITEMS; ++i) {
        const int j = GAE_ITEMS - 1 - i;               // position inside the group
        b_of[i] = 0.0;
        if (FULL || (group >= 0 && g0 + j < count)) {
            const bool cut = ((j < 4 ? d_lo >> (8 * j) : d_hi >> (8 * (j - 4))) & 0xFFu) != 0;
            const bool last = ((j < 4 ? l_lo >> (8 * j) : l_hi >> (8 * (j - 4))) & 0xFFu) != 0;
            float v_next = j + 1 < GAE_ITEMS ? v8[j + 1 < GAE_ITEMS ? j + 1 : j] : v_after;
            if (last) v_next = s_boot[g0 + j];
            const AffineF m{(last || cut) ? 0.f : glf, fma(cut ? 0.0 : (double)gamma, (double)v_next, (double)r8[j]) - (double)v8[j]};
            b_of[i] = m.b;
            a_zero |= (m.a == 0.f ? 1u : 0u) << i;
            mine = compose(mine, m);
        }
    }

    // Exclusive scan of the per-thread maps over the tile (thread order = processing order).
    const AffineF incl = wave_scan(mine);
    if (lane == VER_WAVE - 1) s_wave[wave] = incl;
    bar_lds();
    AffineF before{1.f, 0.0};  // everything in the tile processed before this thread
    for (int w = 0; w < wave; ++w) before = compose(before, s_wave[w]);
    before = compose(before, dpp_map<DPP_WAVE_SHR1, 0xf>(incl));   // (lane 0 gets the identity)

    // Chained scan across tiles (wave 0).
    if (wave == 0) {
        Affine tile_map{1.0, 0.0};
        for (int w = 0; w < GAE_THREADS / VER_WAVE; ++w) tile_map = compose(tile_map, Affine{(double)s_wave[w].a, (double)s_wave[w].b});
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
            // beyond tile 0 the incoming advantage is 0.  A wait that gave up (it never should) must not pass for a
            // result: the tile's outputs, and through it those of the tiles that read its word, become NaN
            carry = failed ? __longlong_as_double(0x7FF8000000000000LL) : back.b;
        }
        if (lane == 0 && !map_only) {
            const double leaving = cut ? tile_map.b : tile_map.b + tile_map.a * carry;
            if (!cut) st_word(&ws.inc[tile], word_of(leaving));
            s_carry = carry;
            s_leaving = leaving;
        }
    }
    bar_lds();
    if (map_only) return;   // (uniform)
    carry_known = s_leaving;

    double x = fma((double)before.a, s_carry, before.b);  // advantage at the step after this thread's first
#pragma unroll
    for (int i = 0; i < GAE_ITEMS; ++i) {
        const int j = GAE_ITEMS - 1 - i;
        if (FULL || (group >= 0 && g0 + j < count)) {
            x = fma((a_zero >> i) & 1u ? 0.0 : gl, x, b_of[i]);
            r8[j] = (float)x;                        // advantage
            v8[j] = (float)(x + (double)v8[j]);      // return
        }
    }
    if (whole) {
        *reinterpret_cast<float4*>(adv + k_lo + g0) = float4{r8[0], r8[1], r8[2], r8[3]};
        *reinterpret_cast<float4*>(adv + k_lo + g0 + 4) = float4{r8[4], r8[5], r8[6], r8[7]};
        *reinterpret_cast<float4*>(ret + k_lo + g0) = float4{v8[0], v8[1], v8[2], v8[3]};
        *reinterpret_cast<float4*>(ret + k_lo + g0 + 4) = float4{v8[4], v8[5], v8[6], v8[7]};
    } else {
#pragma unroll
        for (int j = 0; j < GAE_ITEMS; ++j)
            if (group >= 0 && g0 + j < count) {
                adv[k_lo + g0 + j] = r8[j];
                ret[k_lo + g0 + j] = v8[j];
            }
    }
    };
    for (int pass = pass0; pass < n_here; ++pass) {
        const int tile = first_tile + (pass < 0 ? n_here - 1 : pass);
        if (VEC && S - (ntiles - 1 - tile) * GAE_TILE >= GAE_TILE) do_pass(pass, std::true_type{});
        else do_pass(pass, std::false_type{});
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

namespace ver {
namespace {
// Enqueues the scan with `mem` (ver_gae_workspace_bytes(S) bytes of device memory) as its scratch.
int gae_launch(const float* rewards, const float* values, const uint8_t* dones, const float* last_values,
               const int32_t* env_off, int32_t N, int32_t S, float gamma, float lambda, float* adv, float* ret,
               void* mem, hipStream_t s) {
    const int tiles = gae_tiles(S);
    Carver cv(mem);
    int* head = cv.take<int>(64);
    GaeWs ws;
    ws.ticket = head;
    ws.error = head + 1;
    ws.inc = cv.take<unsigned long long>(tiles);
    ws.agg_a = cv.take<unsigned long long>(tiles);
    ws.agg_b = cv.take<unsigned long long>(tiles);
    // ticket, error and every published word must start at zero (the blocks are adjacent)
    fill_words(reinterpret_cast<int32_t*>(head), cv.used / 4, 0, s);
    ProfScope prof(VER_PROF_GAE, s);
    // 16-byte accesses need 16-byte aligned arrays (tiles start at multiples of the tile size)
    const uintptr_t bits = reinterpret_cast<uintptr_t>(rewards) | reinterpret_cast<uintptr_t>(values) |
                           reinterpret_cast<uintptr_t>(adv) | reinterpret_cast<uintptr_t>(ret) |
                           (reinterpret_cast<uintptr_t>(dones) << 2);
    // tiles per ticket: 1 while tickets are few, up to GAE_MAX_BATCH for buffers of many thousands of tiles
    const int batch = gae_batch(tiles), groups = (tiles + batch - 1) / batch;
    if ((bits & 15) == 0)
        hipLaunchKernelGGL(gae_kernel<true>, dim3(groups), dim3(GAE_THREADS), 0, s, rewards, values, dones,
                           last_values, env_off, N, S, tiles, batch, gamma, lambda, adv, ret, ws);
    else
        hipLaunchKernelGGL(gae_kernel<false>, dim3(groups), dim3(GAE_THREADS), 0, s, rewards, values, dones,
                           last_values, env_off, N, S, tiles, batch, gamma, lambda, adv, ret, ws);
    return launch_status();
}
}  // namespace
}  // namespace ver

extern "C" int ver_gae(const float* rewards, const float* values, const uint8_t* dones,
                       const float* last_values, const int32_t* env_off, int32_t N, int32_t S,
                       float gamma, float lambda, float* adv, float* ret,
                       void* workspace, size_t workspace_bytes, void* stream) {
    if (N < 0 || S < 0) return VER_EINVAL;
    if (S == 0) return VER_OK;
    if (!rewards || !values || !dones || !last_values || !env_off || !adv || !ret || N == 0) return VER_EINVAL;
    if (!workspace || workspace_bytes < ver_gae_workspace_bytes(S)) return VER_EWORKSPACE;
    return ver::gae_launch(rewards, values, dones, last_values, env_off, N, S, gamma, lambda, adv, ret, workspace,
                           static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------------------- ver_gae_static
// The same scan for callers that cannot allocate device memory: the ticket, the error word and the words the
// tiles publish live in a file-scope device array instead of a caller workspace.  Every GPU the library runs
// on holds its own copy of the array at its own address, which is looked up once per device.
namespace ver {
namespace {
constexpr size_t GAE_STATIC_TILES = (VER_GAE_STATIC_MAX_STEPS + GAE_TILE - 1) / GAE_TILE;
constexpr size_t GAE_STATIC_BYTES = 256 + 3 * ((GAE_STATIC_TILES * 8 + 255) / 256 * 256);
constexpr int GAE_STATIC_MAX_DEVICES = 64;
}  // namespace
}  // namespace ver

static __device__ __align__(256) unsigned char scratch[ver::GAE_STATIC_BYTES];

namespace ver {
namespace {
std::mutex g_scratch_lock;
void* g_scratch_ptr[GAE_STATIC_MAX_DEVICES];   // device address of `scratch` on every device seen so far

// Address of the current device's copy of `scratch` (the array's name is only a host-side handle of the symbol).
int scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return VER_EHIP;
    if (dev < 0 || dev >= GAE_STATIC_MAX_DEVICES) return VER_EUNSUPPORTED;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return VER_EHIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return VER_OK;
}
}  // namespace
}  // namespace ver

extern "C" int ver_gae_static(const float* rewards, const float* values, const uint8_t* dones,
                              const float* last_values, const int32_t* env_off, int32_t N, int32_t S,
                              float gamma, float lambda, float* adv, float* ret, void* stream) {
    if (N < 0 || S < 0) return VER_EINVAL;
    if (S == 0) return VER_OK;
    if (!rewards || !values || !dones || !last_values || !env_off || !adv || !ret || N == 0) return VER_EINVAL;
    if (S > VER_GAE_STATIC_MAX_STEPS) return VER_ETOOLARGE;
    static_assert(ver::GAE_STATIC_BYTES >= 256 + 3 * 256, "scratch holds at least one tile");
    if (ver_gae_workspace_bytes(S) > ver::GAE_STATIC_BYTES) return VER_ETOOLARGE;
    void* mem = nullptr;
    const int st = ver::scratch_of_current_device(&mem);
    if (st != VER_OK) return st;
    // the launch clears the part of the array it uses (a fill kernel, no memset node), so what the call
    // before left there does not matter
    return ver::gae_launch(rewards, values, dones, last_values, env_off, N, S, gamma, lambda, adv, ret, mem,
                           static_cast<hipStream_t>(stream));
}
