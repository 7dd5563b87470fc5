// ver_ppo_loss: PPO clipped surrogate + value + entropy loss over the packed
// rows of a minibatch, its six scalars and the gradient w.r.t. the heads'
// outputs, in ONE kernel (plus a tiny counter reset).
//
// Paper: section 2.2 "Learning method" (PPO), appendix hyper-parameter table
// (clip 0.2, value coefficient 0.5, no clipped value loss, no advantage
// normalisation) and the fixed entropy coefficient of the benchmark runs; or,
// as in the training runs (section 4 "Training"), the learned coefficient alpha
// read from device memory: the total then carries alpha*(lambda - H) - alpha*H
// and alpha's gradient lambda - H leaves the kernel with the other scalars.
//
// One thread owns a row: the row's head outputs, action, old log-probability,
// advantage and return are read once, its gradients written once (56 B/row
// categorical-4, 156 B/row Gaussian-11: HBM bound); rows of up to 16 head
// outputs travel through LDS so that memory sees whole contiguous blocks.
// Sums are reduced wave -> workgroup -> per-workgroup partials in the
// workspace; the workgroup that finishes last adds the partials in index
// order, so the result does not depend on scheduling.
#include "common.h"

namespace ver {
namespace {

constexpr int LOSS_THREADS = 256;
constexpr int LOSS_MAX_BLOCKS = 768;   // 3 per CU: measured best on rows streamed through LDS (1024: -9 %, 2048: -35 %)
constexpr int LOSS_SCALARS = 5;  // policy, value, entropy, kl, clipped count
constexpr float HALF_LOG_2PI = 0.91893853320467274178f;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int d = VER_WAVE / 2; d > 0; d >>= 1) v += __shfl_down(v, d, VER_WAVE);
    return v;  // valid in lane 0
}

// Sum over the workgroup, valid in thread 0.  s_red has one slot per wave.
__device__ __forceinline__ float block_sum(float v, float* s_red) {
    v = wave_sum(v);
    const int lane = threadIdx.x & (VER_WAVE - 1), wave = threadIdx.x / VER_WAVE;
    __syncthreads();  // s_red may still be read from the previous call
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    float t = 0.f;
    if (threadIdx.x == 0)
        for (int w = 0; w < LOSS_THREADS / VER_WAVE; ++w) t += s_red[w];
    return t;
}

// What every loss kernel ends with: the workgroup's sums (acc: policy, value, entropy, kl, clipped count; s_lsacc:
// per wave, the log-std gradient per dimension) go to the workgroup's slot of `partials`; the workgroup that
// finishes last adds all slots in index order (a fixed order, whatever the schedule was) and writes the scalars.
template <int DIST>
__device__ __forceinline__ void loss_finish(const ver_ppo_cfg& cfg, int M, const float (&acc)[LOSS_SCALARS],
                                            float (*s_lsacc)[64], float* __restrict__ scalars,
                                            float* __restrict__ d_log_std, float* __restrict__ partials,
                                            int* __restrict__ counter, const float* __restrict__ alpha,
                                            float target_entropy, float alpha_sign, float* __restrict__ d_alpha,
                                            float ent_coef) {
    __shared__ float s_red[LOSS_THREADS / VER_WAVE];
    __shared__ int s_last;
    __shared__ float s_out[LOSS_SCALARS];
    __shared__ float s_slot[LOSS_THREADS];
    const int A = cfg.act_dim;
    const int width = LOSS_SCALARS + (DIST == 1 ? A : 0);  // partial sums per workgroup
    const float inv_m = 1.f / (float)M;
    float* my_partial = partials + (size_t)blockIdx.x * width;
    for (int q = 0; q < LOSS_SCALARS; ++q) {
        const float t = block_sum(acc[q], s_red);
        if (threadIdx.x == 0) st_agent(&my_partial[q], t);
    }
    if (DIST == 1) {
        __syncthreads();
        if (threadIdx.x < A) {
            float t = 0.f;
            for (int w = 0; w < LOSS_THREADS / VER_WAVE; ++w) t += s_lsacc[w][threadIdx.x];
            st_agent(&my_partial[LOSS_SCALARS + threadIdx.x], t);
        }
    }

    // Last workgroup to arrive adds the partials in index order.  The partials are written through to memory with
    // device-scope stores whose completion every thread awaits before the workgroup counts itself in, and are read
    // with device-scope loads: no fence.  (A device-scope fence here writes back the whole L2 of the XCD, dirty
    // with megabytes of gradient rows, once per workgroup: a fifth of the kernel's time on 2^24 rows.)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0)
        s_last = (__hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1);
    __syncthreads();
    if (!s_last) return;
    // Column c of the partials is added by T / width threads ("slots"): slot k adds the workgroups k, k + slots, ...
    // with 8 loads in flight, then one thread per column adds the slots in order: a fixed order, whatever the
    // schedule was, and every thread of the workgroup has work (with one thread per column, 16 of 256 had).
    {
        const int G = gridDim.x, slots = LOSS_THREADS / width;   // width <= 69: at least 3 slots
        const int c = threadIdx.x % width, slot = threadIdx.x / width;
        if (slot < slots) {
            float t = 0.f;
            int g = slot;
            for (; g + 7 * slots < G; g += 8 * slots) {
                float x[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) x[k] = ld_agent(&partials[(size_t)(g + k * slots) * width + c]);
#pragma unroll
                for (int k = 0; k < 8; ++k) t += x[k];
            }
            for (; g < G; g += slots) t += ld_agent(&partials[(size_t)g * width + c]);
            s_slot[slot * width + c] = t;
        }
        __syncthreads();
        if (threadIdx.x < width) {
            float t = 0.f;
            for (int k = 0; k < slots; ++k) t += s_slot[k * width + threadIdx.x];
            if (threadIdx.x < LOSS_SCALARS) s_out[threadIdx.x] = t * inv_m;  // means
            else d_log_std[threadIdx.x - LOSS_SCALARS] = t;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const float pol = s_out[0], val = s_out[1], ent = s_out[2];
        float total = pol + cfg.value_coef * val - ent_coef * ent;
        if (alpha) {
            total += ent_coef * (target_entropy - ent);
            d_alpha[0] = alpha_sign * (target_entropy - ent);
        }
        scalars[0] = total;
        scalars[1] = pol;
        scalars[2] = val;
        scalars[3] = ent;
        scalars[4] = s_out[3];
        scalars[5] = s_out[4];
        *counter = 0;
    }
}

constexpr int LOSS_STAGE_MAX_A = 16;   // widest row that is staged through LDS

// STAGED (1: word by word, 2: 16 bytes at a time for 16-byte aligned arrays): the workgroup's 256 rows of head outputs (and Gaussian actions) are contiguous in memory: they are
// copied into LDS with consecutive lanes on consecutive words, every thread then works on its own row there
// (row pitch A words), writes the row's gradient over the head outputs it has consumed, and the block is
// copied out the same way.  Read row by row straight from memory, a wave instruction would touch 64 rows
// A*4 bytes apart.
template <int DIST, int STAGED>
__global__ __launch_bounds__(LOSS_THREADS) void ppo_loss_kernel(
    ver_ppo_cfg cfg, int M, const float* __restrict__ u, const float* __restrict__ value,
    const float* __restrict__ log_std, const void* __restrict__ actions,
    const float* __restrict__ logp_old, const float* __restrict__ adv, const float* __restrict__ ret,
    const float* __restrict__ is_weight, float* __restrict__ scalars, float* __restrict__ d_u,
    float* __restrict__ d_value, float* __restrict__ d_log_std, float* __restrict__ partials,
    int* __restrict__ counter, const float* __restrict__ alpha, float target_entropy, float alpha_sign,
    float* __restrict__ d_alpha) {
    __shared__ float s_ls[64], s_inv_sigma[64];
    __shared__ float s_lsacc[LOSS_THREADS / VER_WAVE][64];   // per wave: running sums of the log-std gradient
    // staged rows: [256][A] head outputs, then (Gaussian) [256][A] actions; sized by the launch
    extern __shared__ __attribute__((aligned(16))) float s_rows[];
    float* s_u = s_rows;
    float* s_a = s_rows + LOSS_THREADS * cfg.act_dim;
    const int A = cfg.act_dim;
    const float inv_m = 1.f / (float)M;
    const int lane = threadIdx.x & (VER_WAVE - 1), wave = threadIdx.x / VER_WAVE;
    // entropy coefficient: the fixed one, or the current value of the learned one (a constant for the policy)
    const float ent_coef = alpha ? alpha[0] : cfg.entropy_coef;
    if (DIST == 1) {
        if (threadIdx.x < A) {
            s_ls[threadIdx.x] = log_std[threadIdx.x];
            s_inv_sigma[threadIdx.x] = expf(-log_std[threadIdx.x]);
        }
        for (int i = threadIdx.x; i < (LOSS_THREADS / VER_WAVE) * 64; i += LOSS_THREADS) (&s_lsacc[0][0])[i] = 0.f;
        __syncthreads();
    }

    float acc[LOSS_SCALARS] = {0.f, 0.f, 0.f, 0.f, 0.f};
    float ls_own[LOSS_STAGE_MAX_A];
#pragma unroll
    for (int d = 0; d < LOSS_STAGE_MAX_A; ++d) ls_own[d] = 0.f;
    const int stride = gridDim.x * LOSS_THREADS;
    const int rounds = (M + stride - 1) / stride;
    for (int round = 0; round < rounds; ++round) {
        const int p0 = round * stride + blockIdx.x * LOSS_THREADS;
        const int p = p0 + threadIdx.x;
        const bool live = p < M;
        const int words = max(0, min(LOSS_THREADS, M - p0)) * A;   // the block's rows, as words
        if (STAGED) {
            if (round > 0) bar_lds();   // the previous block has been copied out
            const float* gu = u + (size_t)p0 * A;
            const float* ga = static_cast<const float*>(actions) + (size_t)p0 * A;
            const int vec_words = STAGED == 2 ? words & ~3 : 0;
            for (int i = threadIdx.x * 4; i < vec_words; i += LOSS_THREADS * 4) {
                *reinterpret_cast<float4*>(s_u + i) = *reinterpret_cast<const float4*>(gu + i);
                if (DIST == 1) *reinterpret_cast<float4*>(s_a + i) = *reinterpret_cast<const float4*>(ga + i);
            }
            for (int i = vec_words + threadIdx.x; i < words; i += LOSS_THREADS) {
                s_u[i] = gu[i];
                if (DIST == 1) s_a[i] = ga[i];
            }
            bar_lds();
        }
        // this row's scalars
        float w = 1.f, lp_old = 0.f, adv_p = 0.f, val_p = 0.f, ret_p = 0.f;
        int act_p = 0;
        if (live) {
            if (DIST == 0) act_p = static_cast<const int32_t*>(actions)[p];
            w = is_weight ? is_weight[p] : 1.f;
            lp_old = logp_old[p]; adv_p = adv[p]; val_p = value[p]; ret_p = ret[p];
        }
        float coef_logp = 0.f, coef_ent = 0.f;
        const float* up = STAGED ? s_u + threadIdx.x * A : u + (size_t)(live ? p : 0) * A;
        float* dp = STAGED ? s_u + threadIdx.x * A : d_u + (size_t)(live ? p : 0) * A;
        const float* ap = nullptr;
        if (DIST == 1) ap = STAGED ? s_a + threadIdx.x * A : static_cast<const float*>(actions) + (size_t)(live ? p : 0) * A;
        if (live) {
            float logp, ent;
            if (DIST == 0) {
                const int a = act_p;
                float mx = up[0];
                for (int j = 1; j < A; ++j) mx = fmaxf(mx, up[j]);
                float se = 0.f;
                for (int j = 0; j < A; ++j) se += expf(up[j] - mx);
                const float lse = mx + logf(se);
                logp = up[a] - lse;
                ent = 0.f;
                for (int j = 0; j < A; ++j) {
                    const float lq = up[j] - lse;
                    ent -= expf(lq) * lq;
                }
                const float rho = expf(logp - lp_old);
                const float s1 = rho * adv_p;
                const float s2 = fminf(fmaxf(rho, 1.f - cfg.clip), 1.f + cfg.clip) * adv_p;
                coef_logp = (s1 <= s2) ? -w * adv_p * rho * inv_m : 0.f;
                coef_ent = -ent_coef * w * inv_m;
                for (int j = 0; j < A; ++j) {   // (a staged row is overwritten in place: up[j] is read first)
                    const float lq = up[j] - lse;
                    const float q = expf(lq);
                    dp[j] = coef_logp * ((j == a ? 1.f : 0.f) - q) - coef_ent * q * (lq + ent);
                }
                acc[0] += -w * fminf(s1, s2);
                acc[3] += lp_old - logp;
                acc[4] += (fabsf(rho - 1.f) > cfg.clip) ? 1.f : 0.f;
            } else {
                logp = 0.f;
                ent = 0.f;
                for (int d = 0; d < A; ++d) {
                    const float zed = (ap[d] - up[d]) * s_inv_sigma[d];
                    logp += -0.5f * zed * zed - s_ls[d] - HALF_LOG_2PI;
                    ent += s_ls[d] + 0.5f + HALF_LOG_2PI;
                }
                const float rho = expf(logp - lp_old);
                const float s1 = rho * adv_p;
                const float s2 = fminf(fmaxf(rho, 1.f - cfg.clip), 1.f + cfg.clip) * adv_p;
                coef_logp = (s1 <= s2) ? -w * adv_p * rho * inv_m : 0.f;
                coef_ent = -ent_coef * w * inv_m;
                acc[0] += -w * fminf(s1, s2);
                acc[3] += lp_old - logp;
                acc[4] += (fabsf(rho - 1.f) > cfg.clip) ? 1.f : 0.f;
            }
            const float dv = val_p - ret_p;
            acc[1] += w * 0.5f * dv * dv;
            acc[2] += w * ent;
            d_value[p] = cfg.value_coef * w * dv * inv_m;
        }
        if (DIST == 1) {
            // gradient of the mean, and d total / d log_std[d] = sum_rows coef_logp * (zed^2 - 1) + coef_ent
            if (STAGED) {
                // a thread adds up its own rows (one register per dimension); the threads are added at the end
#pragma unroll
                for (int d = 0; d < LOSS_STAGE_MAX_A; ++d) {
                    if (d < A && live) {
                        const float diff = ap[d] - up[d], zed = diff * s_inv_sigma[d];
                        ls_own[d] += coef_logp * (zed * zed - 1.f) + coef_ent;
                        dp[d] = coef_logp * diff * s_inv_sigma[d] * s_inv_sigma[d];
                    }
                }
            } else {
                // wider rows: summed over the wave's rows with shuffles and added to the wave's running sum
                for (int d = 0; d < A; ++d) {
                    float term = 0.f;
                    if (live) {
                        const float diff = ap[d] - up[d], zed = diff * s_inv_sigma[d];
                        term = coef_logp * (zed * zed - 1.f) + coef_ent;
                        dp[d] = coef_logp * diff * s_inv_sigma[d] * s_inv_sigma[d];
                    }
                    const float t = wave_sum(term);
                    if (lane == 0) s_lsacc[wave][d] += t;
                }
            }
        }
        if (STAGED) {
            bar_lds();
            float* gd = d_u + (size_t)p0 * A;
            const int vec_words = STAGED == 2 ? words & ~3 : 0;
            for (int i = threadIdx.x * 4; i < vec_words; i += LOSS_THREADS * 4)
                *reinterpret_cast<float4*>(gd + i) = *reinterpret_cast<const float4*>(s_u + i);
            for (int i = vec_words + threadIdx.x; i < words; i += LOSS_THREADS) gd[i] = s_u[i];
        }
    }
    if (DIST == 1 && STAGED) {
#pragma unroll
        for (int d = 0; d < LOSS_STAGE_MAX_A; ++d) {
            if (d < A) {
                const float t = wave_sum(ls_own[d]);
                if (lane == 0) s_lsacc[wave][d] = t;
            }
        }
    }
    loss_finish<DIST>(cfg, M, acc, s_lsacc, scalars, d_log_std, partials, counter, alpha, target_entropy, alpha_sign, d_alpha, ent_coef);
}

// Lanes of one wave hand data to each other through LDS without a barrier (the hardware executes a wave's LDS
// instructions in order).  The compiler, which reasons about one thread, must be told: it proved that a lane never
// reads a word that the same lane wrote as part of a chunk, and kept such words in registers across the loop.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    asm volatile("" ::: "memory");
}

// The same loss for rows of a width A known at compile time (1..16; 16-byte aligned arrays, M * A a multiple of 4):
// loops over the action dimensions unroll (232 vector instructions per 64 rows instead of ~800 and a dozen
// branches), a row lives in registers between its LDS read and its LDS write, log-std terms are per-kernel
// constants.  A wave's 64 rows are contiguous in memory: it copies them into its own part of LDS with consecutive
// lanes on consecutive 16-byte chunks, every lane works on its own row, the gradient goes back through the same LDS
// words and out as chunks.  LDS instructions of one wave execute in order, so the loop has no barrier and the
// waves of a workgroup drift apart freely.
template <int DIST, int A>
__global__ __launch_bounds__(LOSS_THREADS) void ppo_loss_fixed_kernel(
    ver_ppo_cfg cfg, int M, const float* __restrict__ u, const float* __restrict__ value,
    const float* __restrict__ log_std, const void* __restrict__ actions,
    const float* __restrict__ logp_old, const float* __restrict__ adv, const float* __restrict__ ret,
    const float* __restrict__ is_weight, float* __restrict__ scalars, float* __restrict__ d_u,
    float* __restrict__ d_value, float* __restrict__ d_log_std, float* __restrict__ partials,
    int* __restrict__ counter, const float* __restrict__ alpha, float target_entropy, float alpha_sign,
    float* __restrict__ d_alpha) {
    static_assert(A >= 1 && A <= LOSS_STAGE_MAX_A, "row width");
    constexpr int WWORDS = VER_WAVE * A;                       // words of a wave's 64 rows
    constexpr int NCH = (WWORDS / 4 + VER_WAVE - 1) / VER_WAVE; // 16-byte chunks per lane
    __shared__ float s_lsacc[LOSS_THREADS / VER_WAVE][64];
    // staged rows: [256][A] head outputs, then (Gaussian) [256][A] actions
    __shared__ __attribute__((aligned(16))) float s_u[LOSS_THREADS * A];
    __shared__ __attribute__((aligned(16))) float s_a[DIST == 1 ? LOSS_THREADS * A : 4];
    const float inv_m = 1.f / (float)M;
    const int lane = threadIdx.x & (VER_WAVE - 1), wave = threadIdx.x / VER_WAVE;
    const float ent_coef = alpha ? alpha[0] : cfg.entropy_coef;
    float inv_sigma[A], ls_own[A];
    float ls_sum = 0.f;
#pragma unroll
    for (int d = 0; d < A; ++d) {
        ls_own[d] = 0.f;
        inv_sigma[d] = 1.f;
        if (DIST == 1) {
            const float ls = log_std[d];
            inv_sigma[d] = expf(-ls);
            ls_sum += ls;
        }
    }
    const float gauss_ent = ls_sum + (float)A * (0.5f + HALF_LOG_2PI);   // the same for every row
    float acc[LOSS_SCALARS] = {0.f, 0.f, 0.f, 0.f, 0.f};
    const int stride = gridDim.x * LOSS_THREADS;
    const int rounds = (M + stride - 1) / stride;
    float* su = s_u + wave * WWORDS;
    float* sa = s_a + (DIST == 1 ? wave * WWORDS : 0);

    static_assert(NCH <= 4, "chunks per lane");
    for (int round = 0; round < rounds; ++round) {
        const int p0 = round * stride + (int)blockIdx.x * LOSS_THREADS + wave * VER_WAVE;   // the wave's first row
        const int p = p0 + lane;
        const bool live = p < M;
        const int rows = max(0, min(VER_WAVE, M - p0));
        const int vec_words = rows * A;   // a multiple of 4: the host only launches this kernel when M * A is
        // Every load of the round is issued up front and unconditionally (rows and chunks beyond the buffer's end
        // re-read valid words that are never used): with loads under conditions the compiler cannot count what is
        // in flight and waits for everything at once.  (Fetching a round or two ahead into spare registers was
        // measured: no faster, the plain loop already keeps the memory system busy.)
        const int pl = min(p, M - 1);
        int act_p = 0;
        if (DIST == 0) act_p = static_cast<const int32_t*>(actions)[pl];
        const float w = is_weight ? is_weight[pl] : 1.f;
        const float lp_old = logp_old[pl], adv_p = adv[pl], val_p = value[pl], ret_p = ret[pl];
        {
            const size_t row0 = vec_words > 0 ? (size_t)p0 * A : 0;   // a wave without rows re-reads the start of the buffer
            const int last = vec_words > 0 ? vec_words - 4 : 0;       // last whole chunk of the wave's rows (M * A >= 4)
            const float* gu = u + row0;
            const float* ga = static_cast<const float*>(actions) + row0;
            float4 cu[NCH], ca[NCH];
#pragma unroll
            for (int k = 0; k < NCH; ++k) {
                const int i = min((lane + k * VER_WAVE) * 4, last);
                cu[k] = *reinterpret_cast<const float4*>(gu + i);
                if (DIST == 1) ca[k] = *reinterpret_cast<const float4*>(ga + i);
            }
#pragma unroll
            for (int k = 0; k < NCH; ++k) {
                const int i = (lane + k * VER_WAVE) * 4;
                if (i < vec_words) {
                    *reinterpret_cast<float4*>(su + i) = cu[k];
                    if (DIST == 1) *reinterpret_cast<float4*>(sa + i) = ca[k];
                }
            }
        }
        wave_lds_fence();   // the row below was written by other lanes

        // this lane's row, out of LDS
        float ur[A], ar[A];
        if ((A & 3) == 0) {
#pragma unroll
            for (int d = 0; d < A; d += 4) {
                const float4 t = *reinterpret_cast<const float4*>(su + lane * A + d);
                ur[d] = t.x; ur[d + 1] = t.y; ur[d + 2] = t.z; ur[d + 3] = t.w;
                if (DIST == 1) {
                    const float4 t2 = *reinterpret_cast<const float4*>(sa + lane * A + d);
                    ar[d] = t2.x; ar[d + 1] = t2.y; ar[d + 2] = t2.z; ar[d + 3] = t2.w;
                }
            }
        } else {
#pragma unroll
            for (int d = 0; d < A; ++d) {
                ur[d] = su[lane * A + d];
                if (DIST == 1) ar[d] = sa[lane * A + d];
            }
        }
        float gr[A];   // gradient w.r.t. the row's head outputs
#pragma unroll
        for (int d = 0; d < A; ++d) gr[d] = 0.f;
        if (live) {
            float logp, ent, coef_logp, coef_ent;
            if (DIST == 0) {
                float mx = ur[0];
#pragma unroll
                for (int j = 1; j < A; ++j) mx = fmaxf(mx, ur[j]);
                float se = 0.f;
#pragma unroll
                for (int j = 0; j < A; ++j) se += expf(ur[j] - mx);
                const float lse = mx + logf(se);
                float lq[A], q[A];
                logp = 0.f;
                ent = 0.f;
#pragma unroll
                for (int j = 0; j < A; ++j) {
                    lq[j] = ur[j] - lse;
                    q[j] = expf(lq[j]);
                    ent -= q[j] * lq[j];
                    if (j == act_p) logp = lq[j];
                }
                const float rho = expf(logp - lp_old);
                const float s1 = rho * adv_p;
                const float s2 = fminf(fmaxf(rho, 1.f - cfg.clip), 1.f + cfg.clip) * adv_p;
                coef_logp = (s1 <= s2) ? -w * adv_p * rho * inv_m : 0.f;
                coef_ent = -ent_coef * w * inv_m;
#pragma unroll
                for (int j = 0; j < A; ++j)
                    gr[j] = coef_logp * ((j == act_p ? 1.f : 0.f) - q[j]) - coef_ent * q[j] * (lq[j] + ent);
                acc[0] += -w * fminf(s1, s2);
                acc[3] += lp_old - logp;
                acc[4] += (fabsf(rho - 1.f) > cfg.clip) ? 1.f : 0.f;
            } else {
                float diff[A], zed[A];
                logp = 0.f;
#pragma unroll
                for (int d = 0; d < A; ++d) {
                    diff[d] = ar[d] - ur[d];
                    zed[d] = diff[d] * inv_sigma[d];
                    logp += -0.5f * zed[d] * zed[d];
                }
                logp -= ls_sum + (float)A * HALF_LOG_2PI;
                ent = gauss_ent;
                const float rho = expf(logp - lp_old);
                const float s1 = rho * adv_p;
                const float s2 = fminf(fmaxf(rho, 1.f - cfg.clip), 1.f + cfg.clip) * adv_p;
                coef_logp = (s1 <= s2) ? -w * adv_p * rho * inv_m : 0.f;
                coef_ent = -ent_coef * w * inv_m;
                // gradient of the mean, and d total / d log_std[d] = sum_rows coef_logp * (zed^2 - 1) + coef_ent
#pragma unroll
                for (int d = 0; d < A; ++d) {
                    ls_own[d] += coef_logp * (zed[d] * zed[d] - 1.f) + coef_ent;
                    gr[d] = coef_logp * diff[d] * inv_sigma[d] * inv_sigma[d];
                }
                acc[0] += -w * fminf(s1, s2);
                acc[3] += lp_old - logp;
                acc[4] += (fabsf(rho - 1.f) > cfg.clip) ? 1.f : 0.f;
            }
            const float dv = val_p - ret_p;
            acc[1] += w * 0.5f * dv * dv;
            acc[2] += w * ent;
            d_value[p] = cfg.value_coef * w * dv * inv_m;
        }
        // the row's gradient over the head outputs it came from, then the wave's rows out as 16-byte chunks
        if ((A & 3) == 0) {
#pragma unroll
            for (int d = 0; d < A; d += 4) *reinterpret_cast<float4*>(su + lane * A + d) = float4{gr[d], gr[d + 1], gr[d + 2], gr[d + 3]};
        } else {
#pragma unroll
            for (int d = 0; d < A; ++d) su[lane * A + d] = gr[d];
        }
        wave_lds_fence();   // the chunks below were written by other lanes
        float* gd = d_u + (size_t)p0 * A;
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            const int i = (lane + k * VER_WAVE) * 4;
            if (i < vec_words) *reinterpret_cast<float4*>(gd + i) = *reinterpret_cast<const float4*>(su + i);
        }
        wave_lds_fence();   // the next round overwrites what other lanes have just read
    }
    if (DIST == 1) {
#pragma unroll
        for (int d = 0; d < A; ++d) {
            const float t = wave_sum(ls_own[d]);
            if (lane == 0) s_lsacc[wave][d] = t;
        }
    }
    loss_finish<DIST>(cfg, M, acc, s_lsacc, scalars, d_log_std, partials, counter, alpha, target_entropy, alpha_sign, d_alpha, ent_coef);
}

inline int loss_blocks(int M) {
    int b = (M + LOSS_THREADS - 1) / LOSS_THREADS;
    return b > LOSS_MAX_BLOCKS ? LOSS_MAX_BLOCKS : b;
}

}  // namespace
}  // namespace ver

extern "C" size_t ver_ppo_loss_workspace_bytes(int32_t M, int32_t act_dim) {
    if (M <= 0 || act_dim <= 0) return 0;
    return 256 + ver::align_up((size_t)ver::loss_blocks(M) * (ver::LOSS_SCALARS + act_dim) * 4, 256);
}

namespace ver {
namespace {
int ppo_loss_launch(const ver_ppo_cfg* cfg, int32_t M, const float* head_out, const float* value, const float* log_std,
                    const void* actions_packed, const float* logp_old, const float* adv, const float* ret,
                    const float* is_weight, float* scalars, float* d_head_out, float* d_value, float* d_log_std,
                    void* workspace, size_t workspace_bytes, void* stream, const float* alpha, float target_entropy,
                    float alpha_sign, float* d_alpha) {
    if (!cfg || M <= 0 || !head_out || !value || !actions_packed || !logp_old || !adv || !ret || !scalars ||
        !d_head_out || !d_value)
        return VER_EINVAL;
    if (cfg->dist != 0 && cfg->dist != 1) return VER_EINVAL;
    if (cfg->act_dim < 1 || cfg->act_dim > 63) return VER_EUNSUPPORTED;
    if (cfg->dist == 1 && (!log_std || !d_log_std)) return VER_EINVAL;
    if (!workspace || workspace_bytes < ver_ppo_loss_workspace_bytes(M, cfg->act_dim)) return VER_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(workspace);
    int* counter = cv.take<int>(64);
    float* partials = cv.take<float>((size_t)loss_blocks(M) * (LOSS_SCALARS + cfg->act_dim));
    fill_words(counter, 1, 0, s);
    const int blocks = loss_blocks(M);
    ProfScope prof(VER_PROF_LOSS, s);
    // 0: rows read from memory one by one; 1: staged through LDS; 2: staged with 16-byte accesses
    int staged = cfg->act_dim <= LOSS_STAGE_MAX_A ? 1 : 0;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(head_out) | reinterpret_cast<uintptr_t>(d_head_out) |
                           (cfg->dist == 1 ? reinterpret_cast<uintptr_t>(actions_packed) : 0);
    if (staged && (bits & 15) == 0) staged = 2;
    // the fixed-width kernel moves whole 16-byte chunks only
    const bool fixed_width = staged == 2 && ((long long)M * cfg->act_dim) % 4 == 0;
    const size_t lds = staged ? (size_t)LOSS_THREADS * cfg->act_dim * 4 * (cfg->dist == 1 ? 2 : 1) : 0;
#define VER_LOSS_LAUNCH(DIST, STAGED)                                                                                  \
    hipLaunchKernelGGL((ppo_loss_kernel<DIST, STAGED>), dim3(blocks), dim3(LOSS_THREADS), lds, s, *cfg, M, head_out,    \
                       value, log_std, actions_packed, logp_old, adv, ret, is_weight, scalars, d_head_out, d_value,    \
                       d_log_std, partials, counter, alpha, target_entropy, alpha_sign, d_alpha)
#define VER_LOSS_FIXED(DIST, A_)                                                                                        \
    case A_:                                                                                                            \
        hipLaunchKernelGGL((ppo_loss_fixed_kernel<DIST, A_>), dim3(blocks), dim3(LOSS_THREADS), 0, s, *cfg, M, head_out, \
                           value, log_std, actions_packed, logp_old, adv, ret, is_weight, scalars, d_head_out, d_value, \
                           d_log_std, partials, counter, alpha, target_entropy, alpha_sign, d_alpha);                   \
        break;
#define VER_LOSS_FIXED_ALL(DIST)                                                                                        \
    switch (cfg->act_dim) {                                                                                             \
        VER_LOSS_FIXED(DIST, 1) VER_LOSS_FIXED(DIST, 2) VER_LOSS_FIXED(DIST, 3) VER_LOSS_FIXED(DIST, 4)                  \
        VER_LOSS_FIXED(DIST, 5) VER_LOSS_FIXED(DIST, 6) VER_LOSS_FIXED(DIST, 7) VER_LOSS_FIXED(DIST, 8)                  \
        VER_LOSS_FIXED(DIST, 9) VER_LOSS_FIXED(DIST, 10) VER_LOSS_FIXED(DIST, 11) VER_LOSS_FIXED(DIST, 12)               \
        VER_LOSS_FIXED(DIST, 13) VER_LOSS_FIXED(DIST, 14) VER_LOSS_FIXED(DIST, 15) VER_LOSS_FIXED(DIST, 16)              \
        default: return VER_EUNSUPPORTED;                                                                               \
    }
    if (cfg->dist == 0) {
        if (fixed_width) VER_LOSS_FIXED_ALL(0) else if (staged == 2) VER_LOSS_LAUNCH(0, 2); else if (staged) VER_LOSS_LAUNCH(0, 1); else VER_LOSS_LAUNCH(0, 0);
    } else {
        if (fixed_width) VER_LOSS_FIXED_ALL(1) else if (staged == 2) VER_LOSS_LAUNCH(1, 2); else if (staged) VER_LOSS_LAUNCH(1, 1); else VER_LOSS_LAUNCH(1, 0);
    }
#undef VER_LOSS_FIXED_ALL
#undef VER_LOSS_FIXED
#undef VER_LOSS_LAUNCH
    return launch_status();
}
}  // namespace
}  // namespace ver

extern "C" int ver_ppo_loss(const ver_ppo_cfg* cfg, int32_t M, const float* head_out, const float* value,
                            const float* log_std, const void* actions_packed, const float* logp_old,
                            const float* adv, const float* ret, const float* is_weight, float* scalars,
                            float* d_head_out, float* d_value, float* d_log_std, void* workspace,
                            size_t workspace_bytes, void* stream) {
    return ver::ppo_loss_launch(cfg, M, head_out, value, log_std, actions_packed, logp_old, adv, ret, is_weight, scalars,
                                d_head_out, d_value, d_log_std, workspace, workspace_bytes, stream, nullptr, 0.f, 1.f,
                                nullptr);
}

extern "C" int ver_ppo_loss_learned_entropy(const ver_ppo_cfg* cfg, int32_t M, const float* head_out, const float* value,
                                            const float* log_std, const void* actions_packed, const float* logp_old,
                                            const float* adv, const float* ret, const float* is_weight,
                                            const float* alpha, float target_entropy, float alpha_sign, float* scalars,
                                            float* d_head_out, float* d_value, float* d_log_std, float* d_alpha,
                                            void* workspace, size_t workspace_bytes, void* stream) {
    if (!alpha || !d_alpha || !(alpha_sign == 1.f || alpha_sign == -1.f)) return VER_EINVAL;
    return ver::ppo_loss_launch(cfg, M, head_out, value, log_std, actions_packed, logp_old, adv, ret, is_weight, scalars,
                                d_head_out, d_value, d_log_std, workspace, workspace_bytes, stream, alpha,
                                target_entropy, alpha_sign, d_alpha);
}
