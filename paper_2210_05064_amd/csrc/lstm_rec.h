// Persistent recurrent kernels of the packed LSTM (one launch per layer and
// direction).  gfx950 only.
//
// Paper: the policy's LSTM (section 4 "Architecture") evaluated over the packed
// minibatch of section 2.2: at timestep t only the first batch_sizes[t] pieces
// are alive, and row j of timestep t continues row j of timestep t-1.
//
// The time loop is sequential (hundreds of dependent timesteps with a handful of
// alive pieces each), so its cost is the latency of one all-to-all exchange of
// h_t (forward) or dz_t (backward) between the workgroups that share the hidden
// units, not FLOPs.  Measured on MI355X, per exchange step:
//     64 workgroups on 8 XCDs, agent-scope release/acquire fences   6.5 us
//     64 workgroups on 8 XCDs, write-through stores + coherent loads 2.6 us
//     32 workgroups on ONE XCD, synchronising through its L2          1.0 us
// Hence the design:
//  * pieces are independent of each other in the time loop, so they are dealt to the 8 XCDs: the kernel is
//    launched on the whole chip (one workgroup per CU), the workgroups that find themselves on XCD x
//    (hardware register XCC_ID) form group x, take ranks from the group's ticket and run the pieces
//    n = x, x+8, x+16, ... with a full copy of the recurrent weights spread over their registers.  A
//    group exchanges only its own pieces' rows, and only inside its own L2, which makes that L2 the
//    coherence point: exchanged rows are written with plain stores; the writer waits for their
//    completion (s_waitcnt) before it raises its flag; readers poll the flags with loads that bypass
//    their CU's L1 and then read the rows, which no CU has touched before in this launch (every row of
//    the exchange buffers belongs to exactly one timestep), so they come from L2.  No cache-wide
//    write-back or invalidate is ever issued.  Pieces are sorted longest first, so group 0 runs all
//    T_max timesteps and the others stop earlier;
//  * each wave keeps ITS [16 x K] block of the recurrent weight matrix in
//    registers, already in MFMA operand layout, for the whole kernel; a timestep
//    touches memory only for the exchanged rows (copied by loads that write LDS directly, for all
//    waves) and the saved activations;
//  * gate rows are interleaved (row = unit*4 + gate) so that one MFMA output
//    fragment holds the four gates of a unit in one lane: the cell update needs
//    no cross-lane traffic;
//  * 4H (forward) or H (backward) sits on the MFMA M dimension and the alive
//    pieces on N, so a ragged tail of one or two pieces wastes only N padding;
//  * every wait is bounded and sticky: on time-out the error word is set, every
//    workgroup that sees it leaves the kernel, so the grid always drains.
#pragma once
#include "gemm.h"

namespace ver {

// Optional phase timing (build with -DVER_REC_PROF): thread 0 of the rank-0 workgroup adds the core-clock
// cycles spent in each phase of the time loop to prof[phase]; prof[15] counts timesteps.  Off in the product build.
#ifdef VER_REC_PROF
#ifndef VER_REC_PROF_GROUP
#define VER_REC_PROF_GROUP 0
#endif
#define REC_PROF_DECL long long prof_t = 0; long long* prof_out = a.prof; const bool prof_on = threadIdx.x == 0 && rank == 0 && ps.id == VER_REC_PROF_GROUP;
#define REC_PROF_START() do { if (prof_on) prof_t = clock64(); if (threadIdx.x == 0 && rank == 0 && PIPE != PIPE_NONE) a.prof_all[112 + ps.id + (PIPE == PIPE_CONSUMER ? 3 : 0)] = wall_clock64(); } while (0)
#define REC_PROF_MARK(i) do { if (prof_on) { long long now_ = clock64(); prof_out[i] += now_ - prof_t; prof_t = now_; } } while (0)
#define REC_PROF_STEP() do { if (prof_on) prof_out[15] += 1; } while (0)
#else
#define REC_PROF_DECL
#define REC_PROF_START() do { } while (0)
#define REC_PROF_MARK(i) do { } while (0)
#define REC_PROF_STEP() do { } while (0)
#endif

constexpr int REC_THREADS = 512;          // 8 waves, two per SIMD: 256 registers each
constexpr int REC_WAVES = REC_THREADS / VER_WAVE;
constexpr int REC_GRID = 256;             // one workgroup per CU: 32 per XCD, each XCD one group
constexpr int REC_MAX_GROUP = 32;         // CUs of one XCD
#ifndef VER_REC_GROUPS
#define VER_REC_GROUPS 8
#endif
constexpr int REC_GROUPS = VER_REC_GROUPS;   // XCDs in use: the workgroups of XCD x run the pieces n = x, x+8, x+16, ...
constexpr long long REC_SPIN_LIMIT = 1LL << 21;
constexpr int REC_NTC = 4;                // at most this many 16-piece tiles are staged and multiplied at once
constexpr int REC_NI = 32;                // at most this many 16-byte operand blocks of W per lane (128 registers)

typedef unsigned long long u64_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

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

// Gate non-linearities from the hardware exp2 and reciprocal (about 1 ulp each): at microseconds per
// timestep the instruction count of the cell update matters, and an IEEE division costs ten instructions.
__device__ __forceinline__ float sigmoidf_(float x) { return __builtin_amdgcn_rcpf(1.f + __expf(-x)); }
__device__ __forceinline__ float tanhf_(float x) {
    // tanh(x) = 1 - 2 / (exp(2x) + 1); exact limits at +-inf, ~1e-7 absolute elsewhere
    return 1.f - 2.f * __builtin_amdgcn_rcpf(__expf(2.f * x) + 1.f);
}
// Round to nearest even for finite values (hidden states and their gradients are finite by construction).
__device__ __forceinline__ bf16_t to_bf16_finite(float f) {
    unsigned int u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
template <typename E> __device__ __forceinline__ E cvt_finite(float v);
template <> __device__ __forceinline__ float cvt_finite<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t cvt_finite<bf16_t>(float v) { return to_bf16_finite(v); }

// ---- which workgroups take part ---------------------------------------------------------------------
// The workgroups of one XCD form a group (grp = hardware XCC id) and take ranks from that group's ticket
// (tickets[REC_GROUPS], zero at launch).  Returns this workgroup's rank in [0, G) or -1.
__device__ __forceinline__ int rec_rank(int* tickets, int G, int& grp) {
    __shared__ int s_rank, s_grp;
    if (threadIdx.x == 0) {
        const int xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xf;   // HW_REG_XCC_ID, 4 bits
        int r = -1;
        if (xcc < REC_GROUPS) {
            r = __hip_atomic_fetch_add(&tickets[xcc], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (r >= G) r = -1;
        }
        s_rank = r;
        s_grp = xcc;
    }
    __syncthreads();
    grp = s_grp;
    return s_rank;
}
// Which pieces a group runs: n = x + m * X for m = 0 .. cap-1.  Dealt round-robin to X groups (x = group, cap
// unbounded) or a block of consecutive pieces (x = first piece, X = 1, cap = pieces in the block).
struct PieceSet {
    int x, X, cap;
    int id;   // index of the group (only named by the profiling build)
};
// Pieces of the set alive when `bs` pieces are alive in all (the alive ones are always the first of the set).
__device__ __forceinline__ int grp_count(int bs, const PieceSet& ps) {
    return bs > ps.x ? min((bs - ps.x + ps.X - 1) / ps.X, ps.cap) : 0;
}
// Timesteps at which piece x is alive: batch sizes never grow, so that is how many exceed x.
__device__ __forceinline__ int grp_steps(const int32_t* batch_sizes, int T, int x) {
    __shared__ int s_T;
    if (threadIdx.x == 0) s_T = 0;
    __syncthreads();
    int cnt = 0;
    for (int t = threadIdx.x; t < T; t += blockDim.x) cnt += batch_sizes[t] > x ? 1 : 0;
    if (cnt) atomicAdd(&s_T, cnt);
    __syncthreads();
    return s_T;
}

// ---- exchange through the XCD's L2 --------------------------------------------------------------------
// Flag read that is never served by the CU's L1 (a volatile load carries the sc0 sc1 cache bits); measured
// three times faster than the same bits on a buffer load.
__device__ __forceinline__ int ld_l2(const int* p) { return *reinterpret_cast<const volatile int*>(p); }

// All G participants have published a value >= target.  Returns false if the wait was abandoned (time-out
// here or in another workgroup): the caller must leave the kernel.
// poll_wave: the wave that polls.  A volatile load waits for everything the wave has in flight, so a caller
// that leaves stores in flight across the wait names a wave that rarely has any.
__device__ __forceinline__ bool rec_wait(const int* flags, int G, int target, int* err, int poll_wave = 0) {
    __shared__ int s_ok;
    if ((int)(threadIdx.x >> 6) == poll_wave) {
        const int pl = threadIdx.x & 63;
        long long spins = 0;
        bool alive = true;
        for (;;) {
            const bool ok = pl >= G || ld_l2(&flags[pl]) >= target;
            if (__all(ok)) break;
            ++spins;
            if ((spins & 1023) == 0 && (spins > REC_SPIN_LIMIT || ld_agent(err) != 0)) {
                if (pl == 0) st_agent(err, 1);
                alive = false;
                break;
            }
        }
        if (pl == 0) s_ok = alive ? 1 : 0;
    }
    bar_lds();
    return s_ok != 0;
}

// Call after the exchanged rows were written: waits until this wave's stores have reached L2, then (after
// the workgroup barrier) raises the workgroup's flag.
__device__ __forceinline__ void rec_publish(int* flags, int rank, int value) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    bar_lds();
    if (threadIdx.x == 0) {
        __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(&flags[rank], 0, 4, 0x00020000);
        __builtin_amdgcn_raw_buffer_store_b32(value, r, 0, 0, 0);
    }
}

// Copies `rows` rows of `row_elems` elements (16-byte multiples), `pitch` elements apart in global memory
// (L2), into LDS rows of `stride` elements, with loads that write LDS directly (no registers in between, so a wave can have dozens
// of kilobytes in flight: the copy is bound by the latency of L2, and only the number of bytes in flight
// shortens it).  One wave instruction moves a segment of up to 1 KB of one row: lane i's 16 bytes land at
// the instruction's LDS base + 16*i.  Segments are dealt round-robin to the waves.
// `rot` rotates the order in which this workgroup walks the segments: all workgroups fetch the same rows at
// the same moment, and starting each one at a different place spreads them over the L2 channels.
// The caller waits for the loads (s_waitcnt vmcnt(0)) and synchronises the workgroup.
// The rows start `first` bytes into the buffer `rsrc` (a scalar offset: the buffer itself never changes during
// a kernel, so no descriptor has to be built per timestep).
template <typename E>
__device__ __forceinline__ void stage_rows(__amdgpu_buffer_rsrc_t rsrc, unsigned first, int rows, int row_elems, int pitch,
                                           E* __restrict__ lds, int stride, int rot) {
    const int row_bytes = row_elems * (int)sizeof(E), pitch_bytes = pitch * (int)sizeof(E);
    const int nseg = (row_bytes + 1023) >> 10;
    const int n = rows * nseg;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int shift = (rot * n) / REC_MAX_GROUP;
    const bool pow2 = (nseg & (nseg - 1)) == 0;
    const int lg = 31 - __builtin_clz(nseg);
    unsigned char* lds_b = reinterpret_cast<unsigned char*>(lds);
    for (int s0 = wave; s0 < n; s0 += REC_WAVES) {
        int sg = s0 + shift;
        if (sg >= n) sg -= n;
        const int r = pow2 ? sg >> lg : sg / nseg, part = sg - r * nseg;
        const int in_row = part * 1024 + lane * 16;
        if (in_row < row_bytes)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)(lds_b + (size_t)r * stride * sizeof(E) + part * 1024), 16,
                                                     r * pitch_bytes + in_row, first, 0, 0);
    }
}

// The same for rows given by a pointer: builds the buffer over just those rows.
template <typename E>
__device__ __forceinline__ void stage_rows(const E* __restrict__ src, int rows, int row_elems, int pitch,
                                           E* __restrict__ lds, int stride, int rot) {
    const int row_bytes = row_elems * (int)sizeof(E), pitch_bytes = pitch * (int)sizeof(E);
    stage_rows<E>(__builtin_amdgcn_make_buffer_rsrc(const_cast<E*>(src), 0, (rows - 1) * pitch_bytes + row_bytes, 0x00020000), 0u,
                  rows, row_elems, pitch, lds, stride, rot);
}

// Stores 4 consecutive elements of an exchanged row (8 bytes bf16, 16 bytes fp32).
template <typename E> __device__ __forceinline__ void st_row4(E* p, float a, float b, float c, float d);
template <> __device__ __forceinline__ void st_row4<bf16_t>(bf16_t* p, float a, float b, float c, float d) {
    u16x4_t v;
    v.x = to_bf16_finite(a); v.y = to_bf16_finite(b); v.z = to_bf16_finite(c); v.w = to_bf16_finite(d);
    *reinterpret_cast<u16x4_t*>(p) = v;
}
template <> __device__ __forceinline__ void st_row4<float>(float* p, float a, float b, float c, float d) {
    *reinterpret_cast<f32x4_t*>(p) = f32x4_t{a, b, c, d};
}

// acc[q] += W(16 x k-range) * B_q(k-range x 16) for NT staged tiles; W blocks come from registers, B from LDS.
// In the last (possibly partly empty) tile, lanes whose piece does not exist read piece 0 instead (blast
// points there): equal addresses are broadcast by the LDS, so with one or two alive pieces the LDS traffic
// of the step drops sixteen-fold, and the reads stay unconditional so that they can be issued ahead.
// NI > 0: exactly NI blocks, straight-line code (all LDS reads can be issued ahead of the MFMAs).
// NI == 0: ni_rt blocks (<= REC_NI), guarded: the general, slower path.
template <int MODE, int NI, int NT, int NW>
__device__ __forceinline__ void mma_tiles(const f32x4_t (&wreg)[NW], const typename RecGeom<MODE>::E* brow, int stride,
                                          int ni_rt, const typename RecGeom<MODE>::E* blast, f32x4_t (&acc)[REC_NTC]) {
    constexpr int KBLK = RecGeom<MODE>::KBLK;
    const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
    if (NI > 0) {
        // with few tiles, split the contraction over CH independent accumulator chains per tile so that
        // consecutive MFMAs do not wait for each other's result
        constexpr int CH = (NT == 1 && NI >= 4) ? 4 : ((NT == 2 && NI >= 2) ? 2 : 1);
        f32x4_t part[NT][CH];
#pragma unroll
        for (int q = 0; q < NT; ++q)
#pragma unroll
            for (int c = 0; c < CH; ++c) part[q][c] = zero;
        // operand blocks are fetched from LDS GRP at a time, ahead of the MFMAs that consume them
        constexpr int GRP = (NI * NT >= 8) ? 8 / NT : (NI > 0 ? NI : 1);
#pragma unroll
        for (int i0 = 0; i0 < NI; i0 += GRP) {
            f32x4_t b[GRP][NT];
#pragma unroll
            for (int g = 0; g < GRP; ++g)
#pragma unroll
                for (int q = 0; q < NT; ++q) {
                    const typename RecGeom<MODE>::E* src = (q + 1 < NT) ? brow : blast;   // only the last tile can be partly empty
                    if (i0 + g < NI) b[g][q] = *reinterpret_cast<const f32x4_t*>(src + q * 16 * stride + (i0 + g) * KBLK);
                }
            __builtin_amdgcn_sched_barrier(0);   // keep the loads of a group together and ahead of its MFMAs
#pragma unroll
            for (int g = 0; g < GRP; ++g)
#pragma unroll
                for (int q = 0; q < NT; ++q)
                    if (i0 + g < NI)
                        part[q][(i0 + g) % CH] = mfma_block<MODE>(wreg[i0 + g], b[g][q], part[q][(i0 + g) % CH]);
        }
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
        for (int q = 0; q < NT; ++q) acc[q] = zero;
#pragma unroll
        for (int i = 0; i < NW; ++i)
            if (i < ni_rt) {
#pragma unroll
                for (int q = 0; q < NT; ++q) {
                    const typename RecGeom<MODE>::E* src = (q + 1 < NT) ? brow : blast;
                    const f32x4_t b = *reinterpret_cast<const f32x4_t*>(src + q * 16 * stride + i * KBLK);
                    acc[q] = mfma_block<MODE>(wreg[i], b, acc[q]);
                }
            }
    }
}
// rows: staged rows of this chunk (1 .. 16*REC_NTC); lr: this lane's piece index within a tile.
template <int MODE, int NI, int NW>
__device__ __forceinline__ void mma_dispatch(const f32x4_t (&wreg)[NW], const typename RecGeom<MODE>::E* brow, int stride,
                                             int ni_rt, int rows, int lr, f32x4_t (&acc)[REC_NTC]) {
    const int nt = (rows + 15) >> 4;
    const bool lane_live = (nt - 1) * 16 + lr < rows;
    const typename RecGeom<MODE>::E* blast = lane_live ? brow : brow - lr * stride;
    if (nt == 1) mma_tiles<MODE, NI, 1, NW>(wreg, brow, stride, ni_rt, blast, acc);
    else if (nt == 2) mma_tiles<MODE, NI, 2, NW>(wreg, brow, stride, ni_rt, blast, acc);
    else if (nt == 3) mma_tiles<MODE, NI, 3, NW>(wreg, brow, stride, ni_rt, blast, acc);
    else mma_tiles<MODE, NI, 4, NW>(wreg, brow, stride, ni_rt, blast, acc);
}

// ---- two layers in one launch ---------------------------------------------------------------------------
// With two layers, both time loops run in the same launch on different XCDs.  Group g of the first
// ("producer") layer and group g of the second ("consumer") layer run the same block of consecutive pieces
// (lstm_pipe.h says how the blocks are chosen); a producer group publishes how far it is; workgroups on the
// remaining XCDs ("workers") turn each finished chunk of a group's timesteps into the consumer group's input (a
// GEMM tile at a time); a consumer group waits for the chunk that holds its next timestep.  Groups never wait
// for each other.  Everything that crosses XCDs is written through to memory (the L2s of different XCDs are not
// coherent), completed (s_waitcnt) before it is announced, and announced/read with agent-scope atomics.
constexpr int PIPE_BM = 128;         // rows per GEMM tile
constexpr int PIPE_BN = 256;         // columns per GEMM tile
constexpr int PIPE_CT_MAX = 32;      // at most this many timesteps per chunk
enum { PIPE_NONE = 0, PIPE_PRODUCER = 1, PIPE_CONSUMER = 2 };
// One group's view of the hand-over (producer and consumer groups with the same index run the same pieces).
struct PipeLink {
    int* progress;   // the group's word: timesteps whose producer rows are complete in memory
    int* done;       // the group's [chunks]: GEMM tiles finished per chunk
    const int* rp;   // the group's [T + 1]: rows of the group in the timesteps before t
    int ct;          // timesteps per chunk of the group: chunk c = timesteps [c*ct, (c+1)*ct)
    int tiles_n;     // column tiles per row tile of the GEMM
    int T;           // the group's timesteps
};
// GEMM tiles that cover the group's rows of chunk c.
__device__ __forceinline__ int pipe_chunk_tiles(const PipeLink& pl, int c) {
    const int t0 = c * pl.ct, t1 = min(t0 + pl.ct, pl.T);
    return (pl.rp[t1] - pl.rp[t0] + PIPE_BM - 1) / PIPE_BM * pl.tiles_n;
}
// Consumer: blocks until the workers have finished chunk c.  False if the wait was abandoned.
__device__ __forceinline__ bool pipe_wait_chunk(const PipeLink& pl, int c, int* err, long long* waited = nullptr) {
    __shared__ int s_ok2;
    if (threadIdx.x == 0) {
#ifdef VER_REC_PROF
        const long long w0 = wall_clock64();
#endif
        int have = ld_agent(&pl.done[c]);            // (in flight together with the two loads behind `need`)
        const int need = pipe_chunk_tiles(pl, c);
        long long spins = 0;
        bool alive = true;
        while (have < need) {
            have = ld_agent(&pl.done[c]);
            ++spins;
            if ((spins & 255) == 0 && (spins > REC_SPIN_LIMIT || ld_agent(err) != 0)) {
                st_agent(err, 1);
                alive = false;
                break;
            }
        }
        s_ok2 = alive ? 1 : 0;
#ifdef VER_REC_PROF
        if (waited) *waited += wall_clock64() - w0;   // (100 MHz clock)
#endif
    }
    bar_lds();
    return s_ok2 != 0;
}
#ifdef VER_REC_PROF
#define REC_PROF_CHUNK_ACC(a, rank, ps) ((rank) == 0 ? (a).prof_all + 88 + (ps).id : nullptr)
#else
#define REC_PROF_CHUNK_ACC(a, rank, ps) nullptr
#endif
// Stores that are written through to memory (visible to the other XCDs once complete).  rs: buffer resource
// (wave-uniform) of the rows of one timestep; off: this lane's byte offset in it.
__device__ __forceinline__ void st_through(__amdgpu_buffer_rsrc_t rs, int off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rs, off, 0, 17);
}
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
// Stores 4 consecutive elements of a row at byte `off` + scalar offset `so` of a buffer; AUX = 17 writes through to
// memory (rows that workgroups on other XCDs read), 0 is an ordinary store.
template <typename E, int AUX> struct StRow4;
template <int AUX> struct StRow4<bf16_t, AUX> {
    static __device__ __forceinline__ void go(__amdgpu_buffer_rsrc_t rs, int off, unsigned so, float a, float b, float c, float d) {
        u32x2_t v;
        v.x = (unsigned)to_bf16_finite(a) | ((unsigned)to_bf16_finite(b) << 16);
        v.y = (unsigned)to_bf16_finite(c) | ((unsigned)to_bf16_finite(d) << 16);
        __builtin_amdgcn_raw_buffer_store_b64(v, rs, off, so, AUX);
    }
};
template <int AUX> struct StRow4<float, AUX> {
    static __device__ __forceinline__ void go(__amdgpu_buffer_rsrc_t rs, int off, unsigned so, float a, float b, float c, float d) {
        u32x4_t v = {__float_as_uint(a), __float_as_uint(b), __float_as_uint(c), __float_as_uint(d)};
        __builtin_amdgcn_raw_buffer_store_b128(v, rs, off, so, AUX);
    }
};
template <typename E, int AUX>
__device__ __forceinline__ void st_row4_buf(__amdgpu_buffer_rsrc_t rs, int off, unsigned so, float a, float b, float c, float d) {
    StRow4<E, AUX>::go(rs, off, so, a, b, c, d);
}

// ---- the product of one timestep (forward kernel) ---------------------------------------------------------
// A wave holds TPW 16-row tiles of the weight matrix over its share of the contraction, NBW 16-byte operand
// blocks per tile (wreg[tile * NBW + block]).  For one tile of 16 pieces it reads the matching blocks of the
// staged rows from LDS once, multiplies them with all its tiles, and leaves its partial sums in LDS for the
// wave that owns the tile in the epilogue.  Sharing the contraction between waves is what keeps the number of
// LDS reads down: with one or two alive pieces the step is bound by LDS instructions, not by the MFMAs.
// (Operand blocks loaded straight from the exchanged rows in L2 were measured slower than staging: a load
// instruction costs the same whether 4 or 64 of its lanes carry data.)
constexpr int REC_PRE = 2;   // piece tiles whose per-step inputs are prefetched one timestep ahead

// Register slot i of a wave holds operand block blk_of(i) of its share, for the weights and for the rows
// alike: the rotation `rot` (different in every workgroup) keeps the workgroups of a group, which all read the
// same rows at the same moment, from asking L2 for the same line at the same time.
template <int NBW, bool STATIC>
__device__ __forceinline__ int blk_of(int i, int rot, int nb) {
    const int v = i + rot;
    if (STATIC) return v % NBW;
    return v >= nb ? v - nb : v;
}
// acc[tt] = sum over the wave's operand blocks of W(tile tt, block) * B(block): the B blocks (16 bytes per lane from
// the staged rows at p) are fetched from LDS a few at a time, ahead of the MFMAs that consume them; with fewer than
// four tiles the sum is split over independent accumulator chains so that consecutive MFMAs do not wait for each
// other's result.
template <int MODE, int TPW, int NBW, bool STATIC>
__device__ __forceinline__ void mma_rows(const f32x4_t (&wreg)[TPW * NBW], const typename RecGeom<MODE>::E* p, int nb, int rot,
                                         f32x4_t (&acc)[TPW]) {
    constexpr int CH = TPW >= 4 ? 1 : (TPW == 2 ? (STATIC ? 2 : 1) : 4);
    constexpr int BCH = NBW < 8 ? NBW : 8;
    f32x4_t part[TPW][CH];
#pragma unroll
    for (int tt = 0; tt < TPW; ++tt)
#pragma unroll
        for (int c = 0; c < CH; ++c) part[tt][c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c0 = 0; c0 < NBW; c0 += BCH) {
        f32x4_t b[BCH];
#pragma unroll
        for (int i = 0; i < BCH; ++i)
            if (c0 + i < NBW && (STATIC || c0 + i < nb))
                b[i] = *reinterpret_cast<const f32x4_t*>(p + blk_of<NBW, STATIC>(c0 + i, rot, nb) * RecGeom<MODE>::KBLK);
#pragma unroll
        for (int i = 0; i < BCH; ++i)
            if (c0 + i < NBW && (STATIC || c0 + i < nb)) {
#pragma unroll
                for (int tt = 0; tt < TPW; ++tt)
                    part[tt][(c0 + i) % CH] = mfma_block<MODE>(wreg[tt * NBW + c0 + i], b[i], part[tt][(c0 + i) % CH]);
            }
    }
#pragma unroll
    for (int tt = 0; tt < TPW; ++tt) {
        f32x4_t sum = part[tt][0];
#pragma unroll
        for (int c = 1; c < CH; ++c) {
            sum[0] += part[tt][c][0]; sum[1] += part[tt][c][1]; sum[2] += part[tt][c][2]; sum[3] += part[tt][c][3];
        }
        acc[tt] = sum;
    }
}

// ---- few alive pieces in fp32: the vector ALUs instead of the matrix cores --------------------------------
// An fp32 MFMA (16x16x4) takes a weight through the matrix core at 2 per cycle and SIMD whatever the number of
// alive pieces; a vector FMA takes 16 per cycle and piece.  Up to REC_VALU_ROWS alive pieces of a group the
// product of a timestep is therefore computed piece by piece on the vector ALUs, from the same registers: a lane
// holds 4 consecutive weights of gate row lr per operand block (the MFMA's A layout), reads the matching 4 values
// of the piece's row from LDS (the same address in the 16 lanes of a row group: a broadcast), and the four
// partial sums of a row (lk = 0..3) are added across the wave.  The result goes where the MFMA's accumulator of
// the same (tile, piece) would have gone: out[...] is the f32x4 fragment array of piece tile 0 (64 lanes: column
// = piece, element e of lane group lk = row lk*4 + e).  bf16 gains nothing from this (a packed dot product takes
// 32 weights per cycle, as the bf16 MFMA does).
constexpr int REC_VALU_ROWS = 3;   // (measured on the 2 x 512 fp32 workloads: 2 to 4 within 1 % of each other, 6 and 8 slower)
template <int NW>
__device__ __forceinline__ float valu_row_sum(const f32x4_t (&wreg)[NW], int w0, int n, const float* prow, int nb_rt, int rot,
                                              int nbw, bool is_static) {
    float p0 = 0.f, p1 = 0.f;   // two chains
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        if (i >= n) break;
        if (is_static || i < nb_rt) {
            const int v = i + rot;
            const int blk = is_static ? v % nbw : (v >= nb_rt ? v - nb_rt : v);
            const f32x4_t b = *reinterpret_cast<const f32x4_t*>(prow + blk * RecGeom<MODE_F32>::KBLK);
            const f32x4_t w = wreg[w0 + i];
            p0 = fmaf(w[0], b[0], p0); p1 = fmaf(w[1], b[1], p1);
            p0 = fmaf(w[2], b[2], p0); p1 = fmaf(w[3], b[3], p1);
        }
    }
    float p = p0 + p1;
    p += __shfl_xor(p, 16, VER_WAVE);
    p += __shfl_xor(p, 32, VER_WAVE);
    return p;
}

// ======================================================================================================
struct RecFwdArgs {
    const int32_t* info;
    const int32_t* batch_sizes;
    const int32_t* t_off;
    float* gates;       // [M, 4H] in: W_ih x + b (interleaved columns); out: activated gates i,f,g,o
    float* c;           // [M, H]
    float* hout;        // [M, H]
    void* hprev;        // [M, H] operand type: row p = h_{t-1} of the piece in row p
    void* hcopy;        // [M, H] operand type: row p = h_t, written through for the workers (producer layer only)
    const void* whh;    // [4H, H] operand type, interleaved rows
    const float* h0;    // [seq_cap, H] of this layer, or NULL
    const float* c0;
    int H, seq_cap, M;
    int G;              // workgroups per group; each owns 4*MT hidden units
    int ntc;            // 16-row tiles of staged rows that fit in LDS (1..REC_NTC)
    int* flags;         // [REC_GROUPS][REC_MAX_GROUP] zero at launch
    int* ticket;        // [REC_GROUPS] zero at launch
    int* err;
    long long* prof;    // [16] phase cycle counters (only touched by builds with VER_REC_PROF)
    long long* prof_all;   // start of the profiling words
};

// Waves are (row group rg, contraction share ks): REC_WAVES = RG * KS; a wave multiplies TPW tiles of 16 gate
// rows over 1/KS of the contraction; the workgroup owns MT = RG*TPW tiles = 4*MT hidden units.  In the
// epilogue wave w adds the KS partial sums of tile w and updates the cells of its 4 units.
// NBW: capacity in operand blocks per tile and wave; STATIC: exactly NBW blocks (straight-line code).
// rank: this workgroup's rank in its group; the group runs the pieces n = m * X + x, m = 0, 1, ...; flags: the
// group's flag words.  PIPE: alone, or producer / consumer of a two-layer launch (pl).
template <int MODE, int TPW, int KS, int NBW, bool STATIC, int PIPE>
__device__ __forceinline__ void rec_fwd_body(const RecFwdArgs& a, int rank, const PieceSet ps, int T, int* flags,
                                             const PipeLink& pl, unsigned char* smem) {
    const int x = ps.x, X = ps.X;
    typedef typename RecGeom<MODE>::E E;
    constexpr int PAD = RecGeom<MODE>::PAD, KBLK = RecGeom<MODE>::KBLK, VEC = RecGeom<MODE>::VEC;
    constexpr int RG = REC_WAVES / KS, MT = RG * TPW, UH = 4 * MT, ROWS = 16 * MT;
    static_assert(RG * KS == REC_WAVES && MT <= REC_WAVES, "wave roles");
    const int G = a.G;

    const int H = a.H, stride = H + PAD, ntc = a.ntc;
    E* sB = reinterpret_cast<E*>(smem);                                                        // staged h rows
    f32x4_t* sRed = reinterpret_cast<f32x4_t*>(smem + (size_t)ntc * 16 * stride * sizeof(E));  // [KS][MT][ntc][64]
    E* sH = reinterpret_cast<E*>(sRed + (size_t)KS * MT * ntc * 64);                            // [ntc*16][UH] new h
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rg = wave / KS, ks = wave % KS;
    const int lr = lane & 15, lk = lane >> 4;
    const int j0 = rank * UH;
    const int n_seq = grp_count(a.info[0], ps);
    E* hprev = static_cast<E*>(a.hprev);
    const int k_lo = ((ks + rank) % KS) * (H / KS);   // which share a wave takes rotates with the rank, too
    const int nb = (H / KS) / KBLK;
    const int rot = (rank / KS) % nb;

    // this wave's rows of W_hh (its share of the contraction) -> registers, in MFMA operand layout
    f32x4_t wreg[TPW * NBW];
#pragma unroll
    for (int tt = 0; tt < TPW; ++tt) {
        const E* wrow = static_cast<const E*>(a.whh) + ((size_t)rank * ROWS + (rg * TPW + tt) * 16 + lr) * H + k_lo + lk * VEC;
#pragma unroll
        for (int i = 0; i < NBW; ++i)
            wreg[tt * NBW + i] = (STATIC || i < nb) ? *reinterpret_cast<const f32x4_t*>(wrow + blk_of<NBW, STATIC>(i, rot, nb) * KBLK)
                                                    : f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    // The weights have arrived before the time loop starts, and the compiler has to know: without a use of the
    // registers here it keeps the loads on its books into the loop, where it then makes the MFMAs that read them
    // wait for whatever else is in flight (the prefetch of the next timestep's inputs, the stores of the saved
    // activations), ending in a wait for everything after the last MFMA of every timestep.
#pragma unroll
    for (int i = 0; i < TPW * NBW; ++i) asm volatile("" : "+v"(wreg[i]));
    // initial hidden state of every piece, this workgroup's columns
    for (int i = tid; i < n_seq * (UH / 4); i += REC_THREADS) {
        const int n = (i / (UH / 4)) * X + x, u = (i % (UH / 4)) * 4;
        f32x4_t v = {0.f, 0.f, 0.f, 0.f};
        if (a.h0 && n < a.seq_cap) v = *reinterpret_cast<const f32x4_t*>(a.h0 + (size_t)n * H + j0 + u);
        st_row4<E>(hprev + (size_t)n * H + j0 + u, v[0], v[1], v[2], v[3]);
    }
    rec_publish(flags, rank, 1);
    REC_PROF_DECL
    REC_PROF_START();
    // epilogue role: wave `wave` owns row tile `wave` (units j0 + wave*4 .. +3); its lane holds the four gates of
    // unit wave*4 + lk for piece lr of a piece tile
    const bool has_tile = wave < MT;
    const int je = j0 + wave * 4 + lk;
    const size_t gcol = (size_t)je * 4;
    float creg[REC_PRE];     // cell state of the pieces in this lane's first REC_PRE tiles
    f32x4_t zpre[REC_PRE], znext[REC_PRE];   // their input projections, fetched one timestep ahead
    unsigned goff[REC_PRE];  // byte offset of this lane's gates inside a timestep's rows (tile q): the same every step
#pragma unroll
    for (int q = 0; q < REC_PRE; ++q) {
        creg[q] = 0.f;
        zpre[q] = znext[q] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        goff[q] = ((unsigned)((q * 16 + lr) * X + x) * 4u * (unsigned)H + (unsigned)je * 4u) * 4u;
    }
    if (PIPE == PIPE_CONSUMER && T > 0 && !pipe_wait_chunk(pl, 0, a.err, REC_PROF_CHUNK_ACC(a, rank, ps))) return;
    int c_wait = 1;   // consumer: the chunk it has to wait for next
    if (has_tile && T > 0) {
        const int bs0 = grp_count(a.batch_sizes[0], ps);
#pragma unroll
        for (int q = 0; q < REC_PRE; ++q)
            if (q * 16 + lr < bs0) {
                const int n = (q * 16 + lr) * X + x;
                zpre[q] = *reinterpret_cast<const f32x4_t*>(a.gates + (size_t)n * 4 * H + gcol);
                if (a.c0 && n < a.seq_cap) creg[q] = a.c0[(size_t)n * H + je];   // initial cell state
            }
    }

    // batch sizes of timesteps t, t+1 (and t+2, fetched a step ahead: a scalar load that misses costs about half
    // a microsecond, which would otherwise sit at the top of every step); row offsets follow by addition
    int bs_a = T > 0 ? a.batch_sizes[0] : 0, bs_b = T > 1 ? a.batch_sizes[1] : 0;
    int base = 0, base_prev = 0;
    // The activation arrays as buffers that never change during the loop (host code guarantees that every
    // array is shorter than 2^31 bytes); a lane without a piece gets an offset beyond the range, which a load
    // answers with zero.
    const unsigned row_g = 16u * (unsigned)H;   // bytes of a gates row
    constexpr unsigned OUT_OF_RANGE = 0xFFFFFFF0u;
    constexpr int WHOLE = (int)0x80000000u;
    const __amdgpu_buffer_rsrc_t rs_g = __builtin_amdgcn_make_buffer_rsrc(a.gates, 0, WHOLE, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_c = __builtin_amdgcn_make_buffer_rsrc(a.c, 0, WHOLE, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_h = __builtin_amdgcn_make_buffer_rsrc(a.hout, 0, WHOLE, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_hp = __builtin_amdgcn_make_buffer_rsrc(hprev, 0, WHOLE, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_hcopy = __builtin_amdgcn_make_buffer_rsrc(a.hcopy, 0, PIPE == PIPE_PRODUCER ? WHOLE : 0, 0x00020000);
    for (int t = 0; t < T; ++t) {
        // (the compiler reads it with a vector load, since it cannot prove the array constant; left alone it would
        // wait for that load, and for every store in flight before it, right here at the top of the step: the
        // value is kept in a vector register and made uniform only where the step waits for its stores anyway)
        int bs_c_v = (t + 2 < T) ? a.batch_sizes[t + 2] : 0;
        // bs, bs_next: this group's alive pieces; its piece m sits in packed row base + m * X + x
        const int bs_all = bs_a, bs = grp_count(bs_all, ps);
        const int bs_next = (t + 1 < T) ? grp_count(bs_b, ps) : 0, base_next = base + bs_all;
        if (PIPE == PIPE_CONSUMER && t + 1 < T && t + 1 == c_wait * pl.ct) {
            if (!pipe_wait_chunk(pl, c_wait, a.err, REC_PROF_CHUNK_ACC(a, rank, ps))) return;
            ++c_wait;
        }
        REC_PROF_MARK(6);
        const unsigned so_hcopy = (unsigned)base * (unsigned)(H * (int)sizeof(E));
        // Where this timestep's rows (and the next one's) begin inside the activation arrays, in bytes: the scalar
        // offset of the buffer accesses below; a lane's own offset inside a timestep's rows never changes.
        const unsigned so_g = (unsigned)base * row_g, so_c = so_g >> 2;
        const unsigned so_gnext = (unsigned)base_next * row_g, so_hnext = (unsigned)base_next * (unsigned)(H * (int)sizeof(E));
        if (!rec_wait(flags, G, t + 1, a.err)) return;
        // every workgroup of the group has raised its flag for timestep t-1, i.e. completed that step's stores
        if (PIPE == PIPE_PRODUCER && rank == 0 && tid == 0 && t > 0) st_agent(pl.progress, t);
        REC_PROF_MARK(0);
        for (int c0 = 0; c0 < bs; c0 += 16 * ntc) {
            const int rows = min(bs - c0, 16 * ntc), nt = (rows + 15) >> 4;
            if (c0 > 0) bar_lds();  // the previous chunk's rows have been consumed
            stage_rows<E>(rs_hp, (unsigned)((base + c0 * X + x) * H) * (unsigned)sizeof(E), rows, H, X * H, sB, stride, rank);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            bar_lds();
            if (c0 == 0 && has_tile) {
                // next timestep's input projections.  Issued right after the exchanged rows have arrived: the
                // memory counter retires in order, so a prefetch must never be queued in front of loads that
                // the critical path waits for; from here nothing waits for global memory until the flag is
                // raised at the end of the step.
#pragma unroll
                for (int qq = 0; qq < REC_PRE; ++qq)
                    znext[qq] = __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                                                                rs_g, qq * 16 + lr < bs_next ? goff[qq] : OUT_OF_RANGE, so_gnext, 0));
            }
            REC_PROF_MARK(1);
            if (MODE == MODE_F32 && rows <= REC_VALU_ROWS) {
                if constexpr (MODE == MODE_F32) {
                    for (int pc = 0; pc < rows; ++pc) {
                        const float* prow = reinterpret_cast<const float*>(sB) + pc * stride + k_lo + lk * VEC;
#pragma unroll
                        for (int tt = 0; tt < TPW; ++tt) {
                            const float p = valu_row_sum<TPW * NBW>(wreg, tt * NBW, NBW, prow, nb, rot, NBW, STATIC);
                            if (lk == 0)
                                reinterpret_cast<float*>(&sRed[((ks * MT + rg * TPW + tt) * ntc + 0) * 64 + pc + 16 * (lr >> 2)])[lr & 3] = p;
                        }
                    }
                }
            } else
#pragma unroll 1
            for (int q = 0; q < nt; ++q) {
                // dead lanes of the last tile read its first row: equal addresses are broadcast by the LDS
                const int r = q * 16 + ((q * 16 + lr < rows) ? lr : 0);
                f32x4_t acc[TPW];
                mma_rows<MODE, TPW, NBW, STATIC>(wreg, sB + r * stride + k_lo + lk * VEC, nb, rot, acc);
#pragma unroll
                for (int tt = 0; tt < TPW; ++tt) sRed[((ks * MT + rg * TPW + tt) * ntc + q) * 64 + lane] = acc[tt];
            }
            bar_lds();
            REC_PROF_MARK(2);
            if (has_tile) {
#pragma unroll
                for (int q = 0; q < REC_NTC; ++q) {
                    if (q >= nt) break;
                    f32x4_t z = sRed[((0 * MT + wave) * ntc + q) * 64 + lane];
#pragma unroll
                    for (int sp = 1; sp < KS; ++sp) {
                        const f32x4_t o = sRed[((sp * MT + wave) * ntc + q) * 64 + lane];
                        z[0] += o[0]; z[1] += o[1]; z[2] += o[2]; z[3] += o[3];
                    }
                    const int m = c0 + q * 16 + lr, n = m * X + x;
                    const bool in_regs = c0 == 0 && q < REC_PRE;
                    float hn = 0.f;
                    if (m < bs) {
                        const size_t p = (size_t)base + n;
                        f32x4_t* gp = reinterpret_cast<f32x4_t*>(a.gates + p * 4 * H + gcol);
                        const f32x4_t zin = in_regs ? zpre[q < REC_PRE ? q : 0] : *gp;
                        const float gi = sigmoidf_(z[0] + zin[0]);
                        const float gf = sigmoidf_(z[1] + zin[1]);
                        const float gg = tanhf_(z[2] + zin[2]);
                        const float go = sigmoidf_(z[3] + zin[3]);
                        float c_prev;
                        if (in_regs) c_prev = creg[q < REC_PRE ? q : 0];   // this lane computed it one timestep ago (or fetched c0)
                        else if (t == 0) c_prev = (a.c0 && n < a.seq_cap) ? a.c0[(size_t)n * H + je] : 0.f;
                        else c_prev = a.c[((size_t)base_prev + n) * H + je];
                        const float cn = gf * c_prev + gi * gg;
                        if (in_regs) creg[q < REC_PRE ? q : 0] = cn;
                        hn = go * tanhf_(cn);
                        if (in_regs) {
                            const unsigned go_ = goff[q < REC_PRE ? q : 0];
                            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, f32x4_t{gi, gf, gg, go}), rs_g, go_, so_g, 0);
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(cn), rs_c, go_ >> 2, so_c, 0);
                            // (the producer layer of a two-layer launch hands h on in operand type only: hcopy below)
                            if (PIPE != PIPE_PRODUCER) __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(hn), rs_h, go_ >> 2, so_c, 0);
                        } else {
                            *gp = f32x4_t{gi, gf, gg, go};
                            a.c[p * H + je] = cn;
                            if (PIPE != PIPE_PRODUCER) a.hout[p * H + je] = hn;
                        }
                    }
                    // h_t goes to the exchange row of the next timestep through LDS (below)
                    sH[(q * 16 + lr) * UH + wave * 4 + lk] = cvt_finite<E>(hn);
                }
            }
            // The workgroup's UH units of a row are contiguous (UH * sizeof(E) = 32..64 bytes): write them with
            // full 16-byte pieces from consecutive lanes.  Partial-sector writes scattered over several
            // instructions make the L2 fetch the rest of the line from memory, and the readers of the next
            // timestep then wait for that fill (about 2 us) instead of an L2 hit.
            bar_lds();
            {
                constexpr int PIECES = UH * (int)sizeof(E) / 16;     // 16-byte pieces per row
                const int live = min(rows, bs_next - c0);            // rows of this chunk still alive at t+1
                for (int i = tid; i < live * PIECES; i += REC_THREADS) {
                    const int r = i / PIECES, pc = i % PIECES;
                    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(sH + r * UH + pc * VEC);
                    __builtin_amdgcn_raw_buffer_store_b128(v, rs_hp, (((c0 + r) * X + x) * H + j0 + pc * VEC) * (int)sizeof(E), so_hnext, 0);
                }
                if (PIPE == PIPE_PRODUCER) {
                    // h_t of every row of the chunk in operand type, written through: input of the workers' GEMM
                    for (int i = tid; i < min(rows, bs - c0) * PIECES; i += REC_THREADS) {
                        const int r = i / PIECES, pc = i % PIECES;
                        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(sH + r * UH + pc * VEC);
                        __builtin_amdgcn_raw_buffer_store_b128(v, rs_hcopy, (((c0 + r) * X + x) * H + j0 + pc * VEC) * (int)sizeof(E), so_hcopy, 17);
                    }
                }
            }
        }
        REC_PROF_MARK(3);
        if (t + 1 < T || PIPE == PIPE_PRODUCER) rec_publish(flags, rank, t + 2);
        asm volatile("" : "+v"(bs_c_v));
        const int bs_c = __builtin_amdgcn_readfirstlane(bs_c_v);
#pragma unroll
        for (int q = 0; q < REC_PRE; ++q) zpre[q] = znext[q];
        base_prev = base;
        base = base_next;
        bs_a = bs_b;
        bs_b = bs_c;
        REC_PROF_MARK(4);
        REC_PROF_STEP();
    }
    if (PIPE == PIPE_PRODUCER && rank == 0) {   // the last timestep is complete once every flag says so
        if (T > 0 && !rec_wait(flags, G, T + 1, a.err)) return;
        if (tid == 0) st_agent(pl.progress, T);
    }
}

template <int MODE, int TPW, int KS, int NBW, bool STATIC>
__global__ __launch_bounds__(REC_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void lstm_rec_fwd_kernel(RecFwdArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int grp;
    const int rank = rec_rank(a.ticket, a.G, grp);
    if (rank < 0) return;
    PipeLink none = {};
    const PieceSet ps = {grp, REC_GROUPS, 0x7fffffff, grp};
    const int T = grp_steps(a.batch_sizes, a.info[1], grp);
    rec_fwd_body<MODE, TPW, KS, NBW, STATIC, PIPE_NONE>(a, rank, ps, T, a.flags + grp * REC_MAX_GROUP, none, smem);
}

// ======================================================================================================
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
    float* db_part;         // [groups, 4H] (out): every group's sum of dz over its rows, interleaved columns
    int H, seq_cap;
    int G;                  // participating workgroups; each owns 16*MT hidden units
    int ntc;
    int* flags;
    int* ticket;
    int* err;
    long long* prof;
    long long* prof_all;
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

// MT 16-unit tiles per workgroup, KS waves per tile split the contraction over the 4H gate rows.
template <int MODE, int MT, int KS, int NI, int PIPE>
__device__ __forceinline__ void rec_bwd_body(const RecBwdArgs& a, int rank, const PieceSet ps, int T, int* flags,
                                             const PipeLink& pl, unsigned char* smem) {
    const int x = ps.x, X = ps.X;
    static_assert(MT * KS == REC_WAVES, "one wave per (tile, k-split)");
    static_assert(MT * REC_NTC <= REC_WAVES, "one wave per tile sum");
    typedef typename RecGeom<MODE>::E E;
    constexpr int PAD = RecGeom<MODE>::PAD, KBLK = RecGeom<MODE>::KBLK, VEC = RecGeom<MODE>::VEC;
    constexpr int UH = 16 * MT;
    constexpr int NW = NI > 0 ? NI : REC_NI;
    const int G = a.G;

    const int H = a.H, K = 4 * H, stride = K + PAD, ntc = a.ntc;
    E* sB = reinterpret_cast<E*>(smem);                                                        // staged dz rows
    f32x4_t* sRed = reinterpret_cast<f32x4_t*>(smem + (size_t)ntc * 16 * stride * sizeof(E));  // [KS][MT][ntc][64]
    float* sDh = reinterpret_cast<float*>(sRed + (size_t)KS * MT * ntc * 64);   // [ntc*16][UH] dh carried to the previous timestep
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int mt = wave / KS, ks = wave % KS;
    const int lr = lane & 15, lk = lane >> 4;
    const int j0 = rank * UH;
    E* dzw = static_cast<E*>(a.dz);
    const int k_lo = ks * (K / KS);
    const int ni = (K / KS) / KBLK;

    f32x4_t wreg[NW];
    {
        const E* wrow = static_cast<const E*>(a.whhT) + ((size_t)j0 + mt * 16 + lr) * K + k_lo + lk * VEC;
#pragma unroll
        for (int i = 0; i < NW; ++i)
            wreg[i] = (i < ni) ? *reinterpret_cast<const f32x4_t*>(wrow + i * KBLK) : f32x4_t{0.f, 0.f, 0.f, 0.f};
        // (a use of the registers: the loads are complete before the time loop, see the forward kernel)
#pragma unroll
        for (int i = 0; i < NW; ++i) asm volatile("" : "+v"(wreg[i]));
    }
    // The arrays as buffers that never change during the loop (host code guarantees that each is shorter than
    // 2^31 bytes); where a timestep's rows begin is the scalar offset of an access, and this thread's first
    // (piece, unit) sits at the same place inside every timestep's rows.
    constexpr int WHOLE = (int)0x80000000u;
    const __amdgpu_buffer_rsrc_t rs_dzall = __builtin_amdgcn_make_buffer_rsrc(dzw, 0, WHOLE, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_gates = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.gates), 0, WHOLE, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_cell = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.c), 0, WHOLE, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_above = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.dh_above), 0, WHOLE, 0x00020000);
    const unsigned poff = (unsigned)(((tid / UH) * X + x) * H + j0 + (tid % UH)) * 4u;   // bytes inside an [rows, H] fp32 array
    const unsigned row_h = 4u * (unsigned)H;
    BwdSaved pre;   // saved activations of this thread's first (piece, unit) of the coming timestep
    pre.g4 = f32x4_t{0.f, 0.f, 0.f, 0.f};
    pre.c = pre.c_prev = pre.dh_above = 0.f;
    float dcreg = 0.f;   // cell-state gradient of that (piece, unit), carried from timestep to timestep
    // Bias gradient: a thread always works on the same unit (the stride of its items is a multiple of UH), so it
    // adds up that unit's four gate gradients over all its items in registers; summed over threads after the loop.
    static_assert(REC_THREADS % UH == 0, "a thread keeps its unit");
    float db0 = 0.f, db1 = 0.f, db2 = 0.f, db3 = 0.f;
    int c_wait = T > 0 ? (T - 1) / pl.ct : 0;   // consumer: the chunk of the timestep it runs next
    if (PIPE == PIPE_CONSUMER && T > 0 && !pipe_wait_chunk(pl, c_wait, a.err, REC_PROF_CHUNK_ACC(a, rank, ps))) return;
    // batch sizes of timesteps t+1, t, t-1, t-2 (t-3 is fetched a step ahead, see the forward kernel); row offsets
    // follow by subtraction
    int bs_up = 0, bs_t = T > 0 ? a.batch_sizes[T - 1] : 0, bs_m1 = T > 1 ? a.batch_sizes[T - 2] : 0,
        bs_m2 = T > 2 ? a.batch_sizes[T - 3] : 0;
    int base = T > 0 ? a.t_off[T - 1] : 0;
    if (T > 0) {
        const int bs_l = grp_count(bs_t, ps);
        if (tid < bs_l * UH)
            pre = load_saved(a, T - 1, base, base - bs_m1, (tid / UH) * X + x, j0 + (tid % UH), H);
    }
    REC_PROF_DECL
    REC_PROF_START();
    for (int t = T - 1; t >= 0; --t) {
        // bs, bs_next: this group's alive pieces; its piece m sits in packed row base + m * X + x
        // (kept in a vector register and made uniform only at the end of the step, where everything the step loaded
        // has long arrived: see the forward kernel; read as a scalar right here, the step would open with a wait for
        // this load and for every store still in flight)
        int bs_m3_v = t > 2 ? a.batch_sizes[t - 3] : 0;
        const int bs = grp_count(bs_t, ps);
        const int bs_next = (t + 1 < T) ? grp_count(bs_up, ps) : 0;
        const int base_prev = base - bs_m1;     // rows of timestep t-1 (unused when t == 0)
        const unsigned so_dz = (unsigned)base * (unsigned)(K * (int)sizeof(E));   // where this timestep's dz rows begin
        // A. gate gradients of this workgroup's units for every alive piece
        for (int i = tid; i < bs * UH; i += REC_THREADS) {
            const int m = i / UH, n = m * X + x, j = j0 + (i % UH);
            const size_t p = (size_t)base + n;
            const bool first = i == tid;
            const BwdSaved sv = first ? pre : load_saved(a, t, base, base_prev, n, j, H);
            const float gi = sv.g4[0], gf = sv.g4[1], gg = sv.g4[2], go = sv.g4[3];
            const bool carried = m < bs_next;  // the piece is still alive at t+1
            float dh = sv.dh_above, dc = 0.f;
            if (carried) {
                // the pieces of the first chunk hand dh over in LDS, a thread's first item keeps dc in a register
                // (two separate loads on purpose: written as one conditional expression the compiler loads through
                // a pointer that is either LDS or global memory, and this compiler's back end then fails on the
                // null test of that pointer)
                const float dh_lds = sDh[(m < 16 * ntc ? m : 0) * UH + (i % UH)];
                float dh_mem = 0.f;
                if (m >= 16 * ntc) dh_mem = a.dh_state[(size_t)n * H + j];
                dh += (m < 16 * ntc) ? dh_lds : dh_mem;
                dc = first ? dcreg : a.dc_state[(size_t)n * H + j];
            }
            const float tc = tanhf_(sv.c);
            dc += dh * go * (1.f - tc * tc);
            // (written through in a two-layer launch: the rows are also read by the workers on other XCDs)
                        const float dzi = dc * gg * gi * (1.f - gi), dzf = dc * sv.c_prev * gf * (1.f - gf), dzg = dc * gi * (1.f - gg * gg),
                        dzo = dh * tc * go * (1.f - go);
            st_row4_buf<E, PIPE == PIPE_PRODUCER ? 17 : 0>(rs_dzall, (n * K + j * 4) * (int)sizeof(E), so_dz, dzi, dzf, dzg, dzo);
            db0 += dzi; db1 += dzf; db2 += dzg; db3 += dzo;
            if (first) dcreg = dc * gf;
            else a.dc_state[(size_t)n * H + j] = dc * gf;
        }
        if (t == 0 && PIPE != PIPE_PRODUCER) break;  // nothing is carried before the first timestep
        REC_PROF_MARK(8);
        rec_publish(flags, rank, T - t);
        REC_PROF_MARK(9);
        if (t == 0 && rank != 0) break;
        if (t > 0) {
            if (PIPE == PIPE_CONSUMER && t == c_wait * pl.ct) {   // timestep t-1 opens the chunk below
                --c_wait;
                if (!pipe_wait_chunk(pl, c_wait, a.err, REC_PROF_CHUNK_ACC(a, rank, ps))) return;
            }
            REC_PROF_MARK(13);
            // Saved activations of this thread's first item of timestep t-1.  They come from memory (the forward pass
            // wrote them long ago), which takes longer than a whole MFMA phase: so they are requested here, before the
            // wait for the other workgroups, by waves that do not poll (a poll waits for everything its wave has in
            // flight); the wait for the exchanged rows below then also covers them.
            const int bs_p = grp_count(bs_m1, ps);
            if (tid < bs_p * UH) {
                const unsigned so = (unsigned)base_prev * row_h;
                pre.g4 = __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rs_gates, poff * 4u, so * 4u, 0));
                pre.c = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_cell, poff, so, 0));
                pre.dh_above = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_above, poff, so, 0));
                if (t - 1 == 0) {
                    const int n = (tid / UH) * X + x;
                    pre.c_prev = (a.c0 && n < a.seq_cap) ? a.c0[(size_t)n * H + j0 + (tid % UH)] : 0.f;
                } else {
                    pre.c_prev = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_cell, poff, (unsigned)(base_prev - bs_m2) * row_h, 0));
                }
            }
        }
        if (!rec_wait(flags, G, T - t, a.err, REC_WAVES - 1)) return;
        // every workgroup of the group has completed the dz rows of timesteps >= t
        if (PIPE == PIPE_PRODUCER && rank == 0 && tid == 0) st_agent(pl.progress, T - t);
        if (t == 0) break;
        REC_PROF_MARK(10);
        // B. dh carried to t-1: dh[n][k] = sum_q dz[n][q] * W_hh[q][k] for this workgroup's columns k
        for (int c0 = 0; c0 < bs; c0 += 16 * ntc) {
            const int rows = min(bs - c0, 16 * ntc);
            if (c0 > 0) bar_lds();
            stage_rows<E>(rs_dzall, so_dz + (unsigned)((c0 * X + x) * K) * (unsigned)sizeof(E), rows, K, X * K, sB, stride, rank);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            bar_lds();
            REC_PROF_MARK(11);
            if (MODE == MODE_F32 && rows <= REC_VALU_ROWS) {
                if constexpr (MODE == MODE_F32) {   // few pieces in fp32: the vector ALUs (see valu_row_sum)
                    for (int pc = 0; pc < rows; ++pc) {
                        const float* prow = reinterpret_cast<const float*>(sB) + pc * stride + k_lo + lk * VEC;
                        const float p = valu_row_sum<NW>(wreg, 0, NW, prow, ni, 0, NW, false);
                        if (lk == 0) reinterpret_cast<float*>(&sRed[((ks * MT + mt) * ntc + 0) * 64 + pc + 16 * (lr >> 2)])[lr & 3] = p;
                    }
                }
            } else {
            f32x4_t acc[REC_NTC];
            mma_dispatch<MODE, NI, NW>(wreg, sB + lr * stride + k_lo + lk * VEC, stride, ni, rows, lr, acc);
#pragma unroll
            for (int q = 0; q < REC_NTC; ++q)
                if (q * 16 < rows) sRed[((ks * MT + mt) * ntc + q) * 64 + lane] = acc[q];
            }
            bar_lds();
            // wave w adds the KS partial sums of (unit tile w / REC_NTC, piece tile w % REC_NTC):
            // its lane holds units lk*4..lk*4+3 of piece n
            const int smt = wave / REC_NTC, sq = wave % REC_NTC;
            if (smt < MT && sq * 16 < rows) {
                const int m = c0 + sq * 16 + lr, n = m * X + x;
                f32x4_t sum = sRed[((0 * MT + smt) * ntc + sq) * 64 + lane];
#pragma unroll
                for (int s = 1; s < KS; ++s) {
                    const f32x4_t o = sRed[((s * MT + smt) * ntc + sq) * 64 + lane];
                    sum[0] += o[0]; sum[1] += o[1]; sum[2] += o[2]; sum[3] += o[3];
                }
                if (m < bs) {
                    if (c0 == 0) *reinterpret_cast<f32x4_t*>(sDh + (sq * 16 + lr) * UH + smt * 16 + lk * 4) = sum;
                    else *reinterpret_cast<f32x4_t*>(a.dh_state + (size_t)n * H + j0 + smt * 16 + lk * 4) = sum;
                }
            }
        }
        // dh is read by other threads in the next timestep's part A: from LDS, or (pieces beyond the first chunk)
        // from global memory, whose stores must have completed
        if (bs > 16 * ntc) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        bar_lds();
        base = base_prev;
        bs_up = bs_t;
        bs_t = bs_m1;
        bs_m1 = bs_m2;
        asm volatile("" : "+v"(bs_m3_v));
        bs_m2 = __builtin_amdgcn_readfirstlane(bs_m3_v);
        REC_PROF_MARK(12);
        REC_PROF_STEP();
    }
    // bias gradient of this workgroup's units: the REC_THREADS / UH threads of a unit, added in thread order
    bar_lds();   // (the staging area is free)
    f32x4_t* s_db = reinterpret_cast<f32x4_t*>(smem);
    s_db[tid] = f32x4_t{db0, db1, db2, db3};
    bar_lds();
    if (tid < UH) {
        f32x4_t sum = s_db[tid];
        for (int k = 1; k < REC_THREADS / UH; ++k) {
            const f32x4_t o = s_db[k * UH + tid];
            sum[0] += o[0]; sum[1] += o[1]; sum[2] += o[2]; sum[3] += o[3];
        }
        *reinterpret_cast<f32x4_t*>(a.db_part + (size_t)ps.id * K + (size_t)(j0 + tid) * 4) = sum;
    }
}

template <int MODE, int MT, int KS, int NI>
__global__ __launch_bounds__(REC_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void lstm_rec_bwd_kernel(RecBwdArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int grp;
    const int rank = rec_rank(a.ticket, a.G, grp);
    if (rank < 0) return;
    PipeLink none = {};
    const PieceSet ps = {grp, REC_GROUPS, 0x7fffffff, grp};
    const int T = grp_steps(a.batch_sizes, a.info[1], grp);
    rec_bwd_body<MODE, MT, KS, NI, PIPE_NONE>(a, rank, ps, T, a.flags + grp * REC_MAX_GROUP, none, smem);
}

}  // namespace ver
