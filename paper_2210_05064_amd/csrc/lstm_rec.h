// Persistent recurrent kernels of the packed LSTM (one launch per layer and
// direction).  gfx950 only.
//
// Paper: the policy's LSTM (section 4 "Architecture") evaluated over the packed
// minibatch of section 2.2: at timestep t only the first batch_sizes[t] pieces
// are alive, and row j of timestep t continues row j of timestep t-1.
//
// The time loop is sequential, so its cost is latency, not FLOPs.  Design:
//  * the hidden units are split over G workgroups; each wave keeps ITS 16 rows
//    of the recurrent weight matrix in registers, already in MFMA operand
//    layout, for the whole kernel (loaded once), so a timestep touches HBM/L2
//    only for the h / dz rows that are exchanged; those rows are fetched by the
//    whole workgroup in one burst and staged in LDS, from where every wave
//    reads its MFMA operands;
//  * gate rows are interleaved (row = unit*4 + gate) so that one MFMA output
//    fragment holds the four gates of a unit in one lane: the cell update needs
//    no cross-lane traffic;
//  * 4H (forward) or H (backward) sits on the MFMA M dimension and the alive
//    pieces on N, so a ragged tail of one or two pieces wastes only N padding;
//  * workgroups synchronise once per timestep through a flag array in global
//    memory.  Exchanged rows are written with device-coherent write-through
//    stores, the writer waits for their completion before it raises its flag,
//    and readers fetch them with device-coherent loads.  No cache-wide
//    write-back or invalidate is issued: on this chip those cost microseconds
//    per workgroup and serialise within an XCD, far more than the exchange
//    itself.  Every wait is bounded: on time-out the error word is set and all
//    later waits fall through, so the kernel always terminates.
#pragma once
#include "gemm.h"

namespace ver {

// Optional phase timing (build with -DVER_REC_PROF): thread 0 of workgroup 0 adds the core-clock cycles spent
// in each phase of the time loop to prof[phase]; prof[15] counts timesteps.  Off in the product build.
#ifdef VER_REC_PROF
#define REC_PROF_DECL long long prof_t = 0; long long* prof_out = a.prof;
#define REC_PROF_START() do { if (threadIdx.x == 0 && blockIdx.x == 0) prof_t = clock64(); } while (0)
#define REC_PROF_MARK(i) do { if (threadIdx.x == 0 && blockIdx.x == 0) { long long now_ = clock64(); prof_out[i] += now_ - prof_t; prof_t = now_; } } while (0)
#else
#define REC_PROF_DECL
#define REC_PROF_START() do { } while (0)
#define REC_PROF_MARK(i) do { } while (0)
#endif

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
}

// Call after the exchanged rows were written with st_xchg*: waits until this wave's write-through
// stores have completed, then (after the workgroup barrier) raises the workgroup's flag.
__device__ __forceinline__ void rec_publish(int* flags, int value) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) st_agent(&flags[blockIdx.x], value);
}

// Device-coherent 8-byte accesses for rows exchanged between workgroups.
typedef unsigned long long u64_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void st_xchg8(void* p, u64_t v) {
    __hip_atomic_store(static_cast<u64_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64_t ld_xchg8(const void* p) {
    return __hip_atomic_load(static_cast<const u64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Stores 4 consecutive elements of an exchanged row (8 bytes bf16, 16 bytes fp32).
template <typename E> __device__ __forceinline__ void st_xchg_4(E* p, float a, float b, float c, float d);
template <> __device__ __forceinline__ void st_xchg_4<bf16_t>(bf16_t* p, float a, float b, float c, float d) {
    const u64_t v = (u64_t)to_bf16(a) | ((u64_t)to_bf16(b) << 16) | ((u64_t)to_bf16(c) << 32) | ((u64_t)to_bf16(d) << 48);
    st_xchg8(p, v);
}
template <> __device__ __forceinline__ void st_xchg_4<float>(float* p, float a, float b, float c, float d) {
    st_xchg8(p, (u64_t)__float_as_uint(a) | ((u64_t)__float_as_uint(b) << 32));
    st_xchg8(p + 2, (u64_t)__float_as_uint(c) | ((u64_t)__float_as_uint(d) << 32));
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
    int ntc;            // 16-row tiles of staged rows that fit in LDS (1..REC_NTC)
    int ll_rows;        // timesteps with at most this many alive pieces use the low-latency exchange
    u64_t* ll;          // [2][ll_rows][words per row] tagged words, zero before the launch
    int* flags;
    int* err;
    long long* prof;    // [16] phase cycle counters (only read by builds with VER_REC_PROF)
};

constexpr int REC_NTC = 4;   // at most this many 16-piece tiles are staged and multiplied at once
constexpr int REC_NI = 32;   // at most this many 16-byte operand blocks of W per lane (128 VGPRs)

// Copies `rows` rows of `row_elems` elements (16-byte multiples) from global memory into LDS rows of
// `stride` elements.  The whole workgroup takes part; loads are 16-byte device-coherent buffer loads
// (cache policy sc1), which the compiler keeps in flight eight deep per thread.
template <typename E>
__device__ __forceinline__ void stage_rows(const E* __restrict__ src, int rows, int row_elems, E* __restrict__ lds,
                                           int stride) {
    constexpr int VEC = 16 / sizeof(E);
    constexpr int AUX_SC1 = 16;          // cache-policy bit 4: coherent at device scope
    const int vec_per_row = row_elems / VEC;
    const int n = rows * vec_per_row;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<E*>(src), 0, n * 16, 0x00020000);
    constexpr int DEPTH = 8;  // loads in flight per thread; reads past the last row return zero (buffer bounds)
    int r = threadIdx.x / vec_per_row, c = threadIdx.x - r * vec_per_row;   // position of vector v = threadIdx.x
    for (int v0 = threadIdx.x; v0 < n; v0 += DEPTH * REC_THREADS) {
        u32x4_t tmp[DEPTH];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            tmp[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (v0 + u * REC_THREADS) * 16, 0, AUX_SC1);
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            if (v0 + u * REC_THREADS < n) *reinterpret_cast<u32x4_t*>(lds + r * stride + c * VEC) = tmp[u];
            c += REC_THREADS;
            while (c >= vec_per_row) { c -= vec_per_row; ++r; }
        }
    }
}

// ---- Low-latency exchange for timesteps with few alive pieces -------------------------------------
// With a handful of rows, a timestep is pure synchronisation latency.  For those steps every 4 bytes of an
// exchanged row travel in an 8-byte word {data, tag}: the tag (the timestep counter) makes the word
// self-validating, so the writer neither waits for its stores to complete nor raises a flag, and readers
// poll the data itself with coherent loads.  One memory round trip per timestep instead of three.
// Two slots (timestep parity) suffice: a workgroup can only write slot s+2 after it has read every
// workgroup's words of step s+1, which they wrote after they had finished reading slot s.
constexpr int REC_LL_UNITS = 8;   // 16-byte units (two words) a thread fetches per poll at most

// LL words per exchanged row of row_elems elements (4 data bytes per word).
template <typename E> __device__ __forceinline__ int ll_words(int row_elems) { return row_elems * (int)sizeof(E) / 4; }

// Polls `rows` rows of the slot until every word carries `tag`, then unpacks the data into LDS rows of
// `stride` elements.  rows * words_per_row / 2 <= REC_LL_UNITS * REC_THREADS.  Bounded.
template <typename E>
__device__ __forceinline__ void ll_stage(const u64_t* slot, int rows, int row_elems, unsigned tag, E* lds, int stride,
                                         int* err) {
    constexpr int EPW = 4 / sizeof(E);          // elements per word
    constexpr int AUX_SC1 = 16;
    const int upr = ll_words<E>(row_elems) / 2;  // 16-byte units per row
    const int units = rows * upr;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<u64_t*>(slot), 0, units * 16, 0x00020000);
    u32x4_t d[REC_LL_UNITS];
    long long spins = 0;
    for (;;) {
        bool ready = true;
#pragma unroll
        for (int i = 0; i < REC_LL_UNITS; ++i)
            d[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (threadIdx.x + i * REC_THREADS) * 16, 0, AUX_SC1);
#pragma unroll
        for (int i = 0; i < REC_LL_UNITS; ++i)
            if ((int)threadIdx.x + i * REC_THREADS < units) ready = ready && d[i].y == tag && d[i].w == tag;
        if (ready) break;
        if (++spins > REC_SPIN_LIMIT || ld_agent(err) != 0) {
            st_agent(err, 1);
            break;
        }
    }
    __syncthreads();  // every wave is past the previous timestep's reads of the staging rows
#pragma unroll
    for (int i = 0; i < REC_LL_UNITS; ++i) {
        const int u = threadIdx.x + i * REC_THREADS;
        if (u < units) {
            const int r = u / upr, cu = u - r * upr;
            *reinterpret_cast<u64_t*>(lds + r * stride + cu * 2 * EPW) = (u64_t)d[i].x | ((u64_t)d[i].z << 32);
        }
    }
    __syncthreads();
}

// Writes 4 consecutive elements of row `row` (starting at element `col`, a multiple of 4) as tagged words.
template <typename E>
__device__ __forceinline__ void ll_store4(u64_t* slot, int row, int row_elems, int col, unsigned tag, float a, float b,
                                          float c, float d);
template <>
__device__ __forceinline__ void ll_store4<bf16_t>(u64_t* slot, int row, int row_elems, int col, unsigned tag, float a,
                                                  float b, float c, float d) {
    const u32x4_t v = {(unsigned)to_bf16(a) | ((unsigned)to_bf16(b) << 16), tag,
                       (unsigned)to_bf16(c) | ((unsigned)to_bf16(d) << 16), tag};
    u64_t* p = slot + (size_t)row * (row_elems / 2) + col / 2;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(p, 0, 16, 0x00020000);
    __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, 0, 0, 16);
}
template <>
__device__ __forceinline__ void ll_store4<float>(u64_t* slot, int row, int row_elems, int col, unsigned tag, float a,
                                                 float b, float c, float d) {
    u64_t* p = slot + (size_t)row * row_elems + col;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(p, 0, 32, 0x00020000);
    __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{__float_as_uint(a), tag, __float_as_uint(b), tag}, rsrc, 0, 0, 16);
    __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{__float_as_uint(c), tag, __float_as_uint(d), tag}, rsrc, 16, 0, 16);
}

// acc[q] += W(16 x k-range) * B_q(k-range x 16) for NT staged tiles; W blocks come from registers, B from LDS.
// NI > 0: exactly NI blocks, straight-line code (all LDS reads can be issued ahead of the MFMAs).
// NI == 0: ni_rt blocks (<= REC_NI), guarded: the general, slower path.
template <int MODE, int NI, int NT, int NW>
__device__ __forceinline__ void mma_tiles(const f32x4_t (&wreg)[NW], const typename RecGeom<MODE>::E* brow, int stride,
                                          int ni_rt, f32x4_t (&acc)[REC_NTC]) {
    constexpr int KBLK = RecGeom<MODE>::KBLK;
    if (NI > 0) {
        // with few tiles, split the contraction over CH independent accumulator chains per tile so that
        // consecutive MFMAs do not wait for each other's result
        constexpr int CH = (NT == 1 && NI >= 4) ? 4 : ((NT == 2 && NI >= 2) ? 2 : 1);
        f32x4_t part[NT][CH];
#pragma unroll
        for (int q = 0; q < NT; ++q)
#pragma unroll
            for (int c = 0; c < CH; ++c) part[q][c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int q = 0; q < NT; ++q)
                part[q][i % CH] = mfma_block<MODE>(
                    wreg[i], *reinterpret_cast<const f32x4_t*>(brow + q * 16 * stride + i * KBLK), part[q][i % CH]);
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            f32x4_t sum = part[q][0];
#pragma unroll
            for (int c = 1; c < CH; ++c) {
                sum[0] += part[q][c][0]; sum[1] += part[q][c][1]; sum[2] += part[q][c][2]; sum[3] += part[q][c][3];
            }
            acc[q] = sum;
        }
    } else {
#pragma unroll
        for (int i = 0; i < NW; ++i)
            if (i < ni_rt) {
#pragma unroll
                for (int q = 0; q < NT; ++q)
                    acc[q] = mfma_block<MODE>(wreg[i],
                                              *reinterpret_cast<const f32x4_t*>(brow + q * 16 * stride + i * KBLK), acc[q]);
            }
    }
}
template <int MODE, int NI, int NW>
__device__ __forceinline__ void mma_dispatch(const f32x4_t (&wreg)[NW], const typename RecGeom<MODE>::E* brow, int stride,
                                             int ni_rt, int rows, f32x4_t (&acc)[REC_NTC]) {
    if (rows <= 16) mma_tiles<MODE, NI, 1, NW>(wreg, brow, stride, ni_rt, acc);
    else if (rows <= 32) mma_tiles<MODE, NI, 2, NW>(wreg, brow, stride, ni_rt, acc);
    else if (rows <= 48) mma_tiles<MODE, NI, 3, NW>(wreg, brow, stride, ni_rt, acc);
    else mma_tiles<MODE, NI, 4, NW>(wreg, brow, stride, ni_rt, acc);
}

// MT 16-row tiles of gate rows per workgroup (4*MT hidden units), KS-way split of the contraction.
// NI: 16-byte blocks of W per lane when known at compile time (fast path), 0 = general path.
template <int MODE, int MT, int KS, int NI>
__global__ __launch_bounds__(REC_THREADS) __attribute__((amdgpu_waves_per_eu(1, 1))) void lstm_rec_fwd_kernel(RecFwdArgs a) {
    constexpr int NW = NI > 0 ? NI : REC_NI;
    static_assert(MT * KS * VER_WAVE == REC_THREADS, "one wave per (tile, k-split)");
    typedef typename RecGeom<MODE>::E E;
    constexpr int PAD = RecGeom<MODE>::PAD, KBLK = RecGeom<MODE>::KBLK, VEC = RecGeom<MODE>::VEC;
    constexpr int UH = 4 * MT, ROWS = 16 * MT;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int H = a.H, stride = H + PAD, ntc = a.ntc;
    E* sB = reinterpret_cast<E*>(smem);                                                   // staged h rows
    f32x4_t* sRed = reinterpret_cast<f32x4_t*>(smem + (size_t)ntc * 16 * stride * sizeof(E));  // [KS][MT][NTC][64]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int mt = wave / KS, ks = wave % KS;
    const int lr = lane & 15, lk = lane >> 4;
    const int G = gridDim.x, j0 = blockIdx.x * UH;
    const int n_seq = a.info[0], T = a.info[1];
    E* hprev = static_cast<E*>(a.hprev);
    const int k_lo = ks * (H / KS);
    const int ni = (H / KS) / KBLK;

    // this wave's 16 rows of W_hh (its share of the contraction) -> registers, in MFMA operand layout
    f32x4_t wreg[NW];
    {
        const E* wrow = static_cast<const E*>(a.whh) + ((size_t)blockIdx.x * ROWS + mt * 16 + lr) * H + k_lo + lk * VEC;
#pragma unroll
        for (int i = 0; i < NW; ++i)
            wreg[i] = (i < ni) ? *reinterpret_cast<const f32x4_t*>(wrow + i * KBLK) : f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    // initial hidden state of every piece, this workgroup's columns
    for (int i = tid; i < n_seq * (UH / 4); i += REC_THREADS) {
        const int n = i / (UH / 4), u = (i % (UH / 4)) * 4;
        f32x4_t v = {0.f, 0.f, 0.f, 0.f};
        if (a.h0 && n < a.seq_cap) v = *reinterpret_cast<const f32x4_t*>(a.h0 + (size_t)n * H + j0 + u);
        st_xchg_4<E>(hprev + (size_t)n * H + j0 + u, v[0], v[1], v[2], v[3]);
    }
    rec_publish(a.flags, 1);
    REC_PROF_DECL
    REC_PROF_START();
    float creg[REC_NTC] = {0.f, 0.f, 0.f, 0.f};  // cell state of the pieces in this lane's first REC_NTC tiles

    for (int t = 0; t < T; ++t) {
        const int bs = a.batch_sizes[t], base = a.t_off[t];
        const int bs_next = (t + 1 < T) ? a.batch_sizes[t + 1] : 0, base_next = base + bs;
        const int base_prev = (t > 0) ? a.t_off[t - 1] : 0;
        // The input projections of the first REC_NTC tiles do not depend on other workgroups: fetch them
        // before waiting, so that their latency overlaps the wait and the exchange.
        f32x4_t zpre[REC_NTC];
        if (ks == 0) {
#pragma unroll
            for (int q = 0; q < REC_NTC; ++q) {
                const int n = q * 16 + lr;
                if (n < bs)
                    zpre[q] = *reinterpret_cast<const f32x4_t*>(a.gates + ((size_t)base + n) * 4 * H +
                                                                  (size_t)(j0 + mt * 4 + lk) * 4);
            }
        }
        const bool in_ll = t > 0 && bs <= a.ll_rows;                // how h_{t-1} reaches this timestep
        const bool out_ll = bs_next > 0 && bs_next <= a.ll_rows;   // how h_t leaves it
        const int ll_row_words = ll_words<E>(H);
        u64_t* ll_out = a.ll + (size_t)((t + 1) & 1) * a.ll_rows * ll_row_words;
        if (!in_ll) rec_wait(a.flags, G, t + 1, a.err);
        REC_PROF_MARK(0);
        for (int c0 = 0; c0 < bs; c0 += 16 * ntc) {
            const int rows = min(bs - c0, 16 * ntc);
            if (in_ll) {
                ll_stage<E>(a.ll + (size_t)(t & 1) * a.ll_rows * ll_row_words, rows, H, (unsigned)t, sB, stride, a.err);
            } else {
                if (c0 > 0) __syncthreads();  // the previous chunk's rows have been consumed
                stage_rows<E>(hprev + (size_t)(base + c0) * H, rows, H, sB, stride);
                __syncthreads();
            }
            REC_PROF_MARK(1);
            f32x4_t acc[REC_NTC];
#pragma unroll
            for (int q = 0; q < REC_NTC; ++q) acc[q] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            mma_dispatch<MODE, NI, NW>(wreg, sB + lr * stride + k_lo + lk * VEC, stride, ni, rows, acc);
            if (KS > 1) {
#pragma unroll
                for (int q = 0; q < REC_NTC; ++q)
                    if (q * 16 < rows) sRed[((ks * MT + mt) * REC_NTC + q) * 64 + lane] = acc[q];
                __syncthreads();
                if (ks == 0) {
#pragma unroll
                    for (int q = 0; q < REC_NTC; ++q)
                        if (q * 16 < rows) {
#pragma unroll
                            for (int s = 1; s < KS; ++s) {
                                const f32x4_t o = sRed[((s * MT + mt) * REC_NTC + q) * 64 + lane];
                                acc[q][0] += o[0]; acc[q][1] += o[1]; acc[q][2] += o[2]; acc[q][3] += o[3];
                            }
                        }
                }
            }
            REC_PROF_MARK(2);
            // lane holds the 4 gate pre-activations of unit (mt*4 + lk) for piece c0 + q*16 + lr
            if (ks == 0) {
                const int j = j0 + mt * 4 + lk;
#pragma unroll
                for (int q = 0; q < REC_NTC; ++q) {
                    const int n = c0 + q * 16 + lr;
                    float hn = 0.f;
                    if (q * 16 < rows && n < bs) {
                        const size_t p = (size_t)base + n;
                        f32x4_t* gp = reinterpret_cast<f32x4_t*>(a.gates + p * 4 * H + (size_t)j * 4);
                        const f32x4_t zin = (c0 == 0) ? zpre[q] : *gp;
                        const float gi = sigmoidf_(acc[q][0] + zin[0]);
                        const float gf = sigmoidf_(acc[q][1] + zin[1]);
                        const float gg = tanhf_(acc[q][2] + zin[2]);
                        const float go = sigmoidf_(acc[q][3] + zin[3]);
                        float c_prev;
                        if (t == 0) c_prev = (a.c0 && n < a.seq_cap) ? a.c0[(size_t)n * H + j] : 0.f;
                        else if (c0 == 0) c_prev = creg[q];   // this lane computed it one timestep ago
                        else c_prev = a.c[((size_t)base_prev + n) * H + j];
                        const float cn = gf * c_prev + gi * gg;
                        if (c0 == 0) creg[q] = cn;
                        hn = go * tanhf_(cn);
                        *gp = f32x4_t{gi, gf, gg, go};
                        a.c[p * H + j] = cn;
                        a.hout[p * H + j] = hn;
                    }
                    if (q * 16 < rows) {
                        // the 4 lanes with equal lr hold units mt*4 .. mt*4+3 of piece n: one coherent store
                        const float h1 = __shfl(hn, lr + 16, VER_WAVE), h2 = __shfl(hn, lr + 32, VER_WAVE),
                                    h3 = __shfl(hn, lr + 48, VER_WAVE);
                        if (lk == 0 && n < bs_next) {
                            st_xchg_4<E>(hprev + ((size_t)base_next + n) * H + j0 + mt * 4, hn, h1, h2, h3);
                            if (out_ll) ll_store4<E>(ll_out, n, H, j0 + mt * 4, (unsigned)(t + 1), hn, h1, h2, h3);
                        }
                    }
                }
            }
        }
        REC_PROF_MARK(3);
        if (!out_ll && t + 1 < T) rec_publish(a.flags, t + 2);
        REC_PROF_MARK(4);
#ifdef VER_REC_PROF
        if (threadIdx.x == 0 && blockIdx.x == 0) prof_out[15] += 1;
#endif
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
    int ntc;
    int ll_rows;
    u64_t* ll;          // [2][ll_rows][words per dz row]
    int* flags;
    int* err;
    long long* prof;
};


// What the gate-gradient step needs from the forward pass for one (piece, unit).
struct BwdSaved {
    f32x4_t g4;   // activated gates i, f, g, o
    float c, c_prev, dh_above;
};
__device__ __forceinline__ BwdSaved load_saved(const RecBwdArgs& a, int t, int base, int base_prev, int n, int j, int H) {
    BwdSaved s;
    const size_t p = (size_t)base + n;
    s.g4 = *reinterpret_cast<const f32x4_t*>(a.gates + p * 4 * H + (size_t)j * 4);
    s.c = a.c[p * H + j];
    if (t == 0) s.c_prev = (a.c0 && n < a.seq_cap) ? a.c0[(size_t)n * H + j] : 0.f;
    else s.c_prev = a.c[((size_t)base_prev + n) * H + j];
    s.dh_above = a.dh_above[p * H + j];
    return s;
}

// One 16-unit tile per workgroup, KS = 4 waves split the contraction over the 4H gate rows.
template <int MODE, int NI>
__global__ __launch_bounds__(REC_THREADS) __attribute__((amdgpu_waves_per_eu(1, 1))) void lstm_rec_bwd_kernel(RecBwdArgs a) {
    constexpr int NW = NI > 0 ? NI : REC_NI;
    typedef typename RecGeom<MODE>::E E;
    constexpr int PAD = RecGeom<MODE>::PAD, KBLK = RecGeom<MODE>::KBLK, VEC = RecGeom<MODE>::VEC;
    constexpr int KS = 4, UH = 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int H = a.H, K = 4 * H, stride = K + PAD, ntc = a.ntc;
    E* sB = reinterpret_cast<E*>(smem);                                                       // staged dz rows
    f32x4_t* sRed = reinterpret_cast<f32x4_t*>(smem + (size_t)ntc * 16 * stride * sizeof(E));  // [KS][NTC][64]

    const int tid = threadIdx.x, lane = tid & 63, ks = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;
    const int G = gridDim.x, j0 = blockIdx.x * UH;
    const int T = a.info[1];
    const E* dzr = static_cast<const E*>(a.dz);
    const int k_lo = ks * H;      // this wave's quarter of the 4H contraction
    const int ni = H / KBLK;

    f32x4_t wreg[NW];
    {
        const E* wrow = static_cast<const E*>(a.whhT) + ((size_t)j0 + lr) * K + k_lo + lk * VEC;
#pragma unroll
        for (int i = 0; i < NW; ++i)
            wreg[i] = (i < ni) ? *reinterpret_cast<const f32x4_t*>(wrow + i * KBLK) : f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    BwdSaved pre;
    pre.g4 = f32x4_t{0.f, 0.f, 0.f, 0.f};
    pre.c = pre.c_prev = pre.dh_above = 0.f;
    if (T > 0) {
        const int bs_l = a.batch_sizes[T - 1], base_l = a.t_off[T - 1];
        if (tid < bs_l * UH)
            pre = load_saved(a, T - 1, base_l, (T > 1) ? a.t_off[T - 2] : 0, tid / UH, j0 + (tid % UH), H);
    }
    REC_PROF_DECL
    REC_PROF_START();
    for (int t = T - 1; t >= 0; --t) {
        const int bs = a.batch_sizes[t], base = a.t_off[t];
        const int bs_next = (t + 1 < T) ? a.batch_sizes[t + 1] : 0;
        const int base_prev = (t > 0) ? a.t_off[t - 1] : 0;
        const bool use_ll = bs <= a.ll_rows;   // few alive pieces: exchange dz_t through tagged words
        u64_t* ll_slot = a.ll + (size_t)((T - t) & 1) * a.ll_rows * ll_words<E>(K);
        // A. gate gradients of this workgroup's 16 units for every alive piece
        for (int i = tid; i < bs * UH; i += REC_THREADS) {
            const int n = i / UH, j = j0 + (i % UH);
            const size_t p = (size_t)base + n;
            const BwdSaved sv = (i == tid) ? pre : load_saved(a, t, base, base_prev, n, j, H);
            const float gi = sv.g4[0], gf = sv.g4[1], gg = sv.g4[2], go = sv.g4[3];
            const bool carried = n < bs_next;  // the piece is still alive at t+1
            const float dh = sv.dh_above + (carried ? a.dh_state[(size_t)n * H + j] : 0.f);
            const float tc = tanhf_(sv.c);
            const float dc = (carried ? a.dc_state[(size_t)n * H + j] : 0.f) + dh * go * (1.f - tc * tc);
            const float dzi = dc * gg * gi * (1.f - gi), dzf = dc * sv.c_prev * gf * (1.f - gf),
                        dzg = dc * gi * (1.f - gg * gg), dzo = dh * tc * go * (1.f - go);
            st_xchg_4<E>(static_cast<E*>(a.dz) + p * K + (size_t)j * 4, dzi, dzf, dzg, dzo);
            if (use_ll && t > 0) ll_store4<E>(ll_slot, n, K, j * 4, (unsigned)(T - t), dzi, dzf, dzg, dzo);
            a.dc_state[(size_t)n * H + j] = dc * gf;
        }
        if (t == 0) break;  // nothing is carried before the first timestep
        {   // saved activations of this thread's first item of timestep t-1: in flight during the exchange
            const int bs_p = a.batch_sizes[t - 1], base_p = a.t_off[t - 1];
            if (tid < bs_p * UH)
                pre = load_saved(a, t - 1, base_p, (t > 1) ? a.t_off[t - 2] : 0, tid / UH, j0 + (tid % UH), H);
        }
        REC_PROF_MARK(8);
        if (!use_ll) {
            rec_publish(a.flags, T - t);
            REC_PROF_MARK(9);
            rec_wait(a.flags, G, T - t, a.err);
        }
        REC_PROF_MARK(10);
        // B. dh carried to t-1: dh[n][k] = sum_q dz[n][q] * W_hh[q][k] for this workgroup's 16 columns k
        for (int c0 = 0; c0 < bs; c0 += 16 * ntc) {
            const int rows = min(bs - c0, 16 * ntc);
            if (use_ll) {
                ll_stage<E>(ll_slot, rows, K, (unsigned)(T - t), sB, stride, a.err);
            } else {
                if (c0 > 0) __syncthreads();
                stage_rows<E>(dzr + (size_t)(base + c0) * K, rows, K, sB, stride);
                __syncthreads();
            }
            REC_PROF_MARK(11);
            f32x4_t acc[REC_NTC];
#pragma unroll
            for (int q = 0; q < REC_NTC; ++q) acc[q] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            mma_dispatch<MODE, NI, NW>(wreg, sB + lr * stride + k_lo + lk * VEC, stride, ni, rows, acc);
#pragma unroll
            for (int q = 0; q < REC_NTC; ++q)
                if (q * 16 < rows) sRed[(ks * REC_NTC + q) * 64 + lane] = acc[q];
            __syncthreads();
            // wave q of the workgroup adds the four partial sums of tile q: lane holds units lk*4..lk*4+3 of piece n
            if (ks * 16 < rows) {
                const int n = c0 + ks * 16 + lr;
                f32x4_t sum = sRed[(0 * REC_NTC + ks) * 64 + lane];
#pragma unroll
                for (int s = 1; s < KS; ++s) {
                    const f32x4_t o = sRed[(s * REC_NTC + ks) * 64 + lane];
                    sum[0] += o[0]; sum[1] += o[1]; sum[2] += o[2]; sum[3] += o[3];
                }
                if (n < bs) *reinterpret_cast<f32x4_t*>(a.dh_state + (size_t)n * H + j0 + lk * 4) = sum;
            }
        }
        __syncthreads();  // dh_state is read by other threads in the next timestep's part A
        REC_PROF_MARK(12);
#ifdef VER_REC_PROF
        if (threadIdx.x == 0 && blockIdx.x == 0) prof_out[15] += 1;
#endif
    }
}

}  // namespace ver
