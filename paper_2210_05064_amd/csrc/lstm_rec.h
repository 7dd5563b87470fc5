// Persistent recurrent kernels of the packed LSTM (one launch per layer and
// direction).  gfx950 only.
//
// Paper: the policy's LSTM (section 4 "Architecture") evaluated over the packed
// minibatch of section 2.2: at timestep t only the first batch_sizes[t] pieces
// are alive, and row j of timestep t continues row j of timestep t-1.
//
// The time loop is sequential, so its cost is latency, not FLOPs.  Design:
//  * the hidden units are split over G workgroups; each keeps ITS rows of the
//    recurrent weight matrix in LDS for the whole kernel (loaded once), so a
//    timestep touches HBM/L2 only for the h / dz rows that are exchanged;
//  * gate rows are interleaved (row = unit*4 + gate) so that one MFMA output
//    fragment holds the four gates of a unit in one lane: the cell update needs
//    no cross-lane traffic;
//  * 4H (forward) or H (backward) sits on the MFMA M dimension and the alive
//    pieces on N, so a ragged tail of one or two pieces wastes only N padding;
//  * workgroups synchronise once per timestep through a flag array in global
//    memory (release after the h / dz rows are written, acquire before they are
//    read).  Every wait is bounded: on time-out the error word is set and all
//    later waits fall through, so the kernel always terminates.
#pragma once
#include "gemm.h"

namespace ver {

constexpr int REC_THREADS = 256;
constexpr long long REC_SPIN_LIMIT = 1LL << 22;

template <int MODE> struct RecGeom;
template <> struct RecGeom<MODE_BF16> {
    typedef bf16_t E;
    static constexpr int PAD = 8;    // elements; keeps rows 16-byte aligned and spreads LDS banks
    static constexpr int KBLK = 32;  // contraction elements consumed per 16-byte operand pair
    static constexpr int VEC = 8;    // elements per 16 bytes
};
template <> struct RecGeom<MODE_F32> {
    typedef float E;
    static constexpr int PAD = 4;
    static constexpr int KBLK = 16;
    static constexpr int VEC = 4;
};

// acc += A(16 x KBLK) * B(KBLK x 16); each lane passes the 16 bytes it holds of A and B.
// Any fixed assignment of contraction indices to lanes is valid as long as A and B agree.
template <int MODE> __device__ __forceinline__ f32x4_t mfma_block(f32x4_t a_raw, f32x4_t b_raw, f32x4_t acc);
template <> __device__ __forceinline__ f32x4_t mfma_block<MODE_BF16>(f32x4_t a_raw, f32x4_t b_raw, f32x4_t acc) {
    return mfma_bf16_16x16x32(__builtin_bit_cast(u16x8_t, a_raw), __builtin_bit_cast(u16x8_t, b_raw), acc);
}
template <> __device__ __forceinline__ f32x4_t mfma_block<MODE_F32>(f32x4_t a_raw, f32x4_t b_raw, f32x4_t acc) {
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = mfma_f32_16x16x4(a_raw[e], b_raw[e], acc);
    return acc;
}

__device__ __forceinline__ float sigmoidf_(float x) { return 1.f / (1.f + __expf(-x)); }
__device__ __forceinline__ float tanhf_(float x) {
    // tanh(x) = 1 - 2 / (exp(2x) + 1); exact limits at +-inf, ~1e-7 relative elsewhere
    const float e = __expf(2.f * x);
    return 1.f - 2.f / (e + 1.f);
}

// All workgroups have published a value >= target.  Bounded.
__device__ __forceinline__ void rec_wait(const int* flags, int G, int target, int* err) {
    if (threadIdx.x < VER_WAVE) {
        long long spins = 0;
        for (;;) {
            bool ok = true;
            for (int i = threadIdx.x; i < G; i += VER_WAVE) ok = ok && (ld_agent(&flags[i]) >= target);
            if (__all(ok)) break;
            if (++spins > REC_SPIN_LIMIT || ld_agent(err) != 0) {
                if (threadIdx.x == 0) st_agent(err, 1);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
    }
    __syncthreads();
    fence_acquire();
}

__device__ __forceinline__ void rec_publish(int* flags, int value) {
    fence_release();
    __syncthreads();
    if (threadIdx.x == 0) st_agent(&flags[blockIdx.x], value);
}

struct RecFwdArgs {
    const int32_t* info;
    const int32_t* batch_sizes;
    const int32_t* t_off;
    float* gates;       // [M, 4H] in: W_ih x + b (interleaved columns); out: activated gates i,f,g,o
    float* c;           // [M, H]
    float* hout;        // [M, H]
    void* hprev;        // [M, H] operand type: row p = h_{t-1} of the piece in row p
    const void* whh;    // [4H, H] operand type, interleaved rows
    const float* h0;    // [seq_cap, H] of this layer, or NULL
    const float* c0;
    int H, seq_cap;
    int* flags;
    int* err;
};

// MT 16-row tiles of gate rows per workgroup (4*MT hidden units), KS-way split of the contraction.
template <int MODE, int MT, int KS>
__global__ __launch_bounds__(REC_THREADS) void lstm_rec_fwd_kernel(RecFwdArgs a) {
    static_assert(MT * KS * VER_WAVE == REC_THREADS, "one wave per (tile, k-split)");
    typedef typename RecGeom<MODE>::E E;
    constexpr int PAD = RecGeom<MODE>::PAD, KBLK = RecGeom<MODE>::KBLK, VEC = RecGeom<MODE>::VEC;
    constexpr int UH = 4 * MT, ROWS = 16 * MT;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int H = a.H, stride = H + PAD;
    E* sW = reinterpret_cast<E*>(smem);
    f32x4_t* sRed = reinterpret_cast<f32x4_t*>(smem + (size_t)ROWS * stride * sizeof(E));  // [KS][MT][64]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int mt = wave / KS, ks = wave % KS;
    const int lr = lane & 15, lk = lane >> 4;
    const int G = gridDim.x, j0 = blockIdx.x * UH;
    const int n_seq = a.info[0], T = a.info[1];
    E* hprev = static_cast<E*>(a.hprev);

    // recurrent weights of this workgroup's units -> LDS, once
    {
        const E* src = static_cast<const E*>(a.whh) + (size_t)blockIdx.x * ROWS * H;
        const int vec_per_row = H / VEC;
        for (int i = tid; i < ROWS * vec_per_row; i += REC_THREADS) {
            const int r = i / vec_per_row, v = i % vec_per_row;
            *reinterpret_cast<f32x4_t*>(sW + r * stride + v * VEC) =
                *reinterpret_cast<const f32x4_t*>(src + (size_t)r * H + v * VEC);
        }
    }
    // initial hidden state of every piece, this workgroup's columns
    for (int i = tid; i < n_seq * UH; i += REC_THREADS) {
        const int n = i / UH, u = i % UH;
        const float v = (a.h0 && n < a.seq_cap) ? a.h0[(size_t)n * H + j0 + u] : 0.f;
        hprev[(size_t)n * H + j0 + u] = cvt_elem<E>(v);
    }
    rec_publish(a.flags, 1);

    for (int t = 0; t < T; ++t) {
        rec_wait(a.flags, G, t + 1, a.err);
        const int bs = a.batch_sizes[t], base = a.t_off[t];
        const int bs_next = (t + 1 < T) ? a.batch_sizes[t + 1] : 0, base_next = base + bs;
        const int base_prev = (t > 0) ? a.t_off[t - 1] : 0;
        const int n_tiles = (bs + 15) >> 4;
        for (int nt = 0; nt < n_tiles; ++nt) {
            const int n = nt * 16 + lr;
            const E* brow = hprev + (size_t)(base + min(n, bs - 1)) * H;
            const E* arow = sW + (mt * 16 + lr) * stride;
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
            const int k_lo = ks * (H / KS), k_hi = k_lo + H / KS;
#pragma unroll 4
            for (int k0 = k_lo; k0 < k_hi; k0 += KBLK) {
                const f32x4_t av = *reinterpret_cast<const f32x4_t*>(arow + k0 + lk * VEC);
                const f32x4_t bv = *reinterpret_cast<const f32x4_t*>(brow + k0 + lk * VEC);
                acc = mfma_block<MODE>(av, bv, acc);
            }
            if (KS > 1) {
                __syncthreads();  // previous tile's partial sums have been consumed
                sRed[(ks * MT + mt) * 64 + lane] = acc;
                __syncthreads();
                if (ks == 0) {
                    acc = sRed[mt * 64 + lane];
#pragma unroll
                    for (int s = 1; s < KS; ++s) {
                        const f32x4_t o = sRed[(s * MT + mt) * 64 + lane];
                        acc[0] += o[0]; acc[1] += o[1]; acc[2] += o[2]; acc[3] += o[3];
                    }
                }
            }
            // lane holds the 4 gate pre-activations of unit (mt*4 + lk) for piece n
            if (ks == 0 && n < bs) {
                const int j = j0 + mt * 4 + lk;
                const size_t p = (size_t)base + n;
                f32x4_t* gp = reinterpret_cast<f32x4_t*>(a.gates + p * 4 * H + (size_t)j * 4);
                const f32x4_t zin = *gp;
                const float gi = sigmoidf_(acc[0] + zin[0]);
                const float gf = sigmoidf_(acc[1] + zin[1]);
                const float gg = tanhf_(acc[2] + zin[2]);
                const float go = sigmoidf_(acc[3] + zin[3]);
                float c_prev;
                if (t == 0) c_prev = (a.c0 && n < a.seq_cap) ? a.c0[(size_t)n * H + j] : 0.f;
                else c_prev = a.c[((size_t)base_prev + n) * H + j];
                const float cn = gf * c_prev + gi * gg;
                const float hn = go * tanhf_(cn);
                *gp = f32x4_t{gi, gf, gg, go};
                a.c[p * H + j] = cn;
                a.hout[p * H + j] = hn;
                if (n < bs_next) hprev[((size_t)base_next + n) * H + j] = cvt_elem<E>(hn);
            }
        }
        rec_publish(a.flags, t + 2);
    }
}

struct RecBwdArgs {
    const int32_t* info;
    const int32_t* batch_sizes;
    const int32_t* t_off;
    const float* gates;     // [M, 4H] activated gates (interleaved)
    const float* c;         // [M, H]
    const float* c0;        // [seq_cap, H] of this layer or NULL
    const float* dh_above;  // [M, H] gradient arriving at h_t from the layer above / the heads
    void* dz;               // [M, 4H] operand type (out): gradient at the gate pre-activations
    const void* whhT;       // [H, 4H] operand type: row k = column k of the interleaved W_hh
    float* dh_state;        // [n_cap, H] recurrent gradient carried to the previous timestep
    float* dc_state;        // [n_cap, H]
    int H, seq_cap;
    int* flags;
    int* err;
};

template <int MODE> __device__ __forceinline__ void store_dz4(void* dz, size_t idx, float a, float b, float c, float d);
template <> __device__ __forceinline__ void store_dz4<MODE_F32>(void* dz, size_t idx, float a, float b, float c, float d) {
    *reinterpret_cast<f32x4_t*>(static_cast<float*>(dz) + idx) = f32x4_t{a, b, c, d};
}
template <> __device__ __forceinline__ void store_dz4<MODE_BF16>(void* dz, size_t idx, float a, float b, float c, float d) {
    u16x4_t v;
    v.x = to_bf16(a); v.y = to_bf16(b); v.z = to_bf16(c); v.w = to_bf16(d);
    *reinterpret_cast<u16x4_t*>(static_cast<bf16_t*>(dz) + idx) = v;
}

// One 16-unit tile per workgroup, KS = 4 waves split the contraction over the 4H gate rows.
template <int MODE>
__global__ __launch_bounds__(REC_THREADS) void lstm_rec_bwd_kernel(RecBwdArgs a) {
    typedef typename RecGeom<MODE>::E E;
    constexpr int PAD = RecGeom<MODE>::PAD, KBLK = RecGeom<MODE>::KBLK, VEC = RecGeom<MODE>::VEC;
    constexpr int KS = 4, UH = 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int H = a.H, K = 4 * H, stride = K + PAD;
    E* sW = reinterpret_cast<E*>(smem);
    f32x4_t* sRed = reinterpret_cast<f32x4_t*>(smem + (size_t)UH * stride * sizeof(E));  // [KS][64]

    const int tid = threadIdx.x, lane = tid & 63, ks = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;
    const int G = gridDim.x, j0 = blockIdx.x * UH;
    const int T = a.info[1];
    const E* dzr = static_cast<const E*>(a.dz);

    {
        const E* src = static_cast<const E*>(a.whhT) + (size_t)j0 * K;
        const int vec_per_row = K / VEC;
        for (int i = tid; i < UH * vec_per_row; i += REC_THREADS) {
            const int r = i / vec_per_row, v = i % vec_per_row;
            *reinterpret_cast<f32x4_t*>(sW + r * stride + v * VEC) =
                *reinterpret_cast<const f32x4_t*>(src + (size_t)r * K + v * VEC);
        }
    }
    __syncthreads();

    for (int t = T - 1; t >= 0; --t) {
        const int bs = a.batch_sizes[t], base = a.t_off[t];
        const int bs_next = (t + 1 < T) ? a.batch_sizes[t + 1] : 0;
        const int base_prev = (t > 0) ? a.t_off[t - 1] : 0;
        // A. gate gradients of this workgroup's 16 units for every alive piece
        for (int i = tid; i < bs * UH; i += REC_THREADS) {
            const int n = i / UH, j = j0 + (i % UH);
            const size_t p = (size_t)base + n;
            const f32x4_t g4 = *reinterpret_cast<const f32x4_t*>(a.gates + p * K + (size_t)j * 4);
            const float gi = g4[0], gf = g4[1], gg = g4[2], go = g4[3];
            const float cc = a.c[p * H + j];
            float c_prev;
            if (t == 0) c_prev = (a.c0 && n < a.seq_cap) ? a.c0[(size_t)n * H + j] : 0.f;
            else c_prev = a.c[((size_t)base_prev + n) * H + j];
            const bool carried = n < bs_next;  // the piece is still alive at t+1
            const float dh = a.dh_above[p * H + j] + (carried ? a.dh_state[(size_t)n * H + j] : 0.f);
            const float tc = tanhf_(cc);
            const float dc = (carried ? a.dc_state[(size_t)n * H + j] : 0.f) + dh * go * (1.f - tc * tc);
            store_dz4<MODE>(a.dz, p * K + (size_t)j * 4, dc * gg * gi * (1.f - gi), dc * c_prev * gf * (1.f - gf),
                            dc * gi * (1.f - gg * gg), dh * tc * go * (1.f - go));
            a.dc_state[(size_t)n * H + j] = dc * gf;
        }
        if (t == 0) break;  // nothing is carried before the first timestep
        rec_publish(a.flags, T - t);
        rec_wait(a.flags, G, T - t, a.err);
        // B. dh carried to t-1: dh[n][k] = sum_q dz[n][q] * W_hh[q][k] for this workgroup's 16 columns k
        const int n_tiles = (bs + 15) >> 4;
        for (int nt = 0; nt < n_tiles; ++nt) {
            const int n = nt * 16 + lr;
            const E* brow = dzr + (size_t)(base + min(n, bs - 1)) * K;
            const E* arow = sW + lr * stride;
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
            const int k_lo = ks * (K / KS), k_hi = k_lo + K / KS;
#pragma unroll 4
            for (int k0 = k_lo; k0 < k_hi; k0 += KBLK) {
                const f32x4_t av = *reinterpret_cast<const f32x4_t*>(arow + k0 + lk * VEC);
                const f32x4_t bv = *reinterpret_cast<const f32x4_t*>(brow + k0 + lk * VEC);
                acc = mfma_block<MODE>(av, bv, acc);
            }
            __syncthreads();
            sRed[ks * 64 + lane] = acc;
            __syncthreads();
            if (ks == 0 && n < bs) {
#pragma unroll
                for (int s = 1; s < KS; ++s) {
                    const f32x4_t o = sRed[s * 64 + lane];
                    acc[0] += o[0]; acc[1] += o[1]; acc[2] += o[2]; acc[3] += o[3];
                }
                // lane holds units lk*4 .. lk*4+3 of piece n
                *reinterpret_cast<f32x4_t*>(a.dh_state + (size_t)n * H + j0 + lk * 4) = acc;
            }
        }
        __syncthreads();  // dh_state is read by other threads in the next timestep's part A
    }
}

}  // namespace ver
