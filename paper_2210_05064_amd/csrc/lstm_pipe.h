// Two LSTM layers in one launch.  gfx950 only.
//
// Paper: the policy is a multi-layer LSTM (section 4 "Architecture") evaluated over packed minibatches
// (section 2.2).  The time loop of a layer is a chain of hundreds of dependent steps that leaves most of the
// chip idle, and the second layer's step t only needs the first layer's output of step t: so the two time
// loops run side by side, a few timesteps apart, instead of one after the other.
//
//   XCD 0..2   time loop of the producer layer (forward: layer 0; backward: layer 1), pieces dealt to 3 groups
//   XCD 3..5   time loop of the consumer layer, same dealing (backward: XCD 3..6, 4 groups)
//   the rest   workers: for every finished chunk of PIPE_CT timesteps, the GEMM that turns the producer's rows
//              into the consumer's input (forward: gates_1 = h_0 W_ih1^T + b; backward: dh_0 = dz_1 W_ih1),
//              one 128 x 256 tile at a time from a shared queue, in the order the consumer needs them
//
// Hand-over (lstm_rec.h, PipeLink): producer rows are written through to memory and their completion is
// published per group; a worker waits for all producer groups before it reads a chunk's rows with loads that
// bypass the non-coherent caches, writes its tile through, waits for the stores and counts the tile in
// done[chunk]; a consumer group waits until done[chunk] has reached the number of tiles of the chunk.  Waiting
// only ever points backwards along producer -> worker -> consumer and the queue is ordered by chunk, so the
// launch cannot deadlock; every wait is bounded and raises the shared error word on time-out.
#pragma once
#include "lstm_rec.h"

namespace ver {

constexpr int PIPE_GROUPS = 3;        // groups (XCDs) of the producer layer
constexpr int PIPE_GROUPS_C_FWD = 3;  // groups of the consumer layer, forward: two XCDs of workers
constexpr int PIPE_GROUPS_C_BWD = 4;  // backward (heavier steps, lighter GEMM): one XCD of workers (measured best)
constexpr int PIPE_XCDS = 8;         // XCDs of the chip: those beyond the two layers' groups are workers

struct PipeWork {
    const void* A;      // producer rows [M, K], operand type (forward: h, backward: dz)
    const void* B;      // [N, K] operand type, K contiguous
    float* C;           // [M, N]
    const float* bias;  // [N] or NULL
    int K, N;
    const int32_t* batch_sizes;
    const int32_t* t_off;
    int* queue;         // next item, zero at launch
    int* err;
};

template <typename E, typename T> __device__ __forceinline__ Quad<E> load_quad_coh(__amdgpu_buffer_rsrc_t r, int byte_off);
template <> __device__ __forceinline__ Quad<float> load_quad_coh<float, float>(__amdgpu_buffer_rsrc_t r, int byte_off) {
    const u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 17);
    return Quad<float>{{__uint_as_float(t[0]), __uint_as_float(t[1]), __uint_as_float(t[2]), __uint_as_float(t[3])}};
}
template <> __device__ __forceinline__ Quad<bf16_t> load_quad_coh<bf16_t, bf16_t>(__amdgpu_buffer_rsrc_t r, int byte_off) {
    const u32x2_t t = __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, 17);
    return Quad<bf16_t>{{(bf16_t)(t.x & 0xffff), (bf16_t)(t.x >> 16), (bf16_t)(t.y & 0xffff), (bf16_t)(t.y >> 16)}};
}

// One 128 x 256 tile of C = A B^T (+ bias) for rows [row0, row_end) and columns from col0, by 8 waves (2 x 4
// of 64 x 64).  Same K-tile pipeline as gemm_kernel: the next K-tile's global loads are in flight while the
// current one is multiplied out of LDS.
template <int MODE, typename TA>
__device__ __forceinline__ void pipe_gemm_tile(const PipeWork& w, int row0, int row_end, int col0, unsigned char* smem) {
    typedef typename LdsElem<MODE>::type E;
    constexpr int BK = GemmGeom<MODE>::BK, STRIDE = GemmGeom<MODE>::LDS_STRIDE;
    constexpr int CPR = BK / 4, RPP = REC_THREADS / CPR, QA = PIPE_BM / RPP, QB = PIPE_BN / RPP;
    E* sA = reinterpret_cast<E*>(smem);
    E* sB = sA + PIPE_BM * STRIDE;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 2) * 64, wn = (wave & 3) * 64;
    const int lr = lane & 15, lk = lane >> 4;
    const int c = tid % CPR, r = tid / CPR;
    const int K = w.K, N = w.N;
    __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<TA*>(static_cast<const TA*>(w.A)) + (size_t)row0 * K, 0,
                                                                   (row_end - row0) * K * (int)sizeof(TA), 0x00020000);
    const E* Bp = static_cast<const E*>(w.B);

    f32x4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    Quad<E> ra[QA], rb[QB];
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int i = 0; i < QA; ++i) {
            const int lrow = r + i * RPP;   // rows past the end of the chunk read zero (buffer bounds)
            ra[i] = load_quad_coh<E, TA>(rsA, (lrow * K + k0 + c * 4) * (int)sizeof(TA));
        }
#pragma unroll
        for (int i = 0; i < QB; ++i) {
            const int n = col0 + r + i * RPP;
            rb[i] = n < N ? load_quad<E, E>(Bp + (size_t)n * K + k0 + c * 4) : zero_quad<E>();
        }
    };
    load_tiles(0);
    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int i = 0; i < QA; ++i) store_quad(sA + (r + i * RPP) * STRIDE + c * 4, ra[i]);
#pragma unroll
        for (int i = 0; i < QB; ++i) store_quad(sB + (r + i * RPP) * STRIDE + c * 4, rb[i]);
        bar_lds();
        if (k0 + BK < K) load_tiles(k0 + BK);
        if (MODE == MODE_BF16) {
#pragma unroll
            for (int ks = 0; ks < BK; ks += 32) {
                u16x8_t a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    a[i] = *reinterpret_cast<const u16x8_t*>(reinterpret_cast<const bf16_t*>(sA) + (wm + i * 16 + lr) * STRIDE + ks + lk * 8);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    b[j] = *reinterpret_cast<const u16x8_t*>(reinterpret_cast<const bf16_t*>(sB) + (wn + j * 16 + lr) * STRIDE + ks + lk * 8);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = mfma_bf16_16x16x32(a[i], b[j], acc[i][j]);
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < BK; ks += 16) {
                f32x4_t a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    a[i] = *reinterpret_cast<const f32x4_t*>(reinterpret_cast<const float*>(sA) + (wm + i * 16 + lr) * STRIDE + ks + lk * 4);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    b[j] = *reinterpret_cast<const f32x4_t*>(reinterpret_cast<const float*>(sB) + (wn + j * 16 + lr) * STRIDE + ks + lk * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[i][j] = mfma_f32_16x16x4(a[i][e], b[j][e], acc[i][j]);
            }
        }
        bar_lds();
    }
    // C fragment: element e of lane l is row (l / 16) * 4 + e, column l % 16 of the 16x16 tile; written through
    __amdgpu_buffer_rsrc_t rsC = __builtin_amdgcn_make_buffer_rsrc(w.C + (size_t)row0 * N, 0, (row_end - row0) * N * 4, 0x00020000);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = col0 + wn + j * 16 + lr;
            if (n >= N) continue;
            const float bv = w.bias ? w.bias[n] : 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int lrow = wm + i * 16 + lk * 4 + e;   // rows past the end of the chunk are dropped (buffer bounds)
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][e] + bv), rsC, (lrow * N + n) * 4, 0, 17);
            }
        }
}

// The same tile for bf16 operands on both sides, built for a workgroup that has the CU to itself: K-tiles of
// 64 go from global memory straight into LDS (three stages, two K-tiles in flight while one is multiplied,
// one barrier per K-tile, no registers or LDS stores in between).  An LDS row is the 128 bytes of a tile row,
// as 8 chunks of 16 bytes; chunk position p of row r holds chunk p ^ ((r >> 1) & 7), which makes the 16-byte
// MFMA operand reads of 16 consecutive rows hit all banks once.  A load instruction fills 8 rows (lane -> row
// lane / 8, position lane % 8), so the swizzle is applied on the global side.
constexpr int PIPE_STAGES = 3;
constexpr int PIPE_STAGE_BYTES = (PIPE_BM + PIPE_BN) * 128;
// K need not be a multiple of 64 (it is a multiple of 4): the last K-tile then also fetches what follows the rows'
// ends (the next row, or zeros past the end of the arrays), and the A operand is cleared beyond K in registers, so
// that whatever was fetched on the B side is multiplied by zero.
// COHERENT: A is being written by other XCDs during this launch and C is read by them (loads and stores that
// bypass the non-coherent caches); false for a launch of its own.
template <bool COHERENT>
__device__ __forceinline__ void pipe_gemm_tile_dma(const PipeWork& w, int row0, int row_end, int col0, unsigned char* smem) {
    constexpr int BK = 64;
    constexpr int AUX = COHERENT ? 17 : 0;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave >> 2) * 64, wn = (wave & 3) * 64;
    const int lr = lane & 15, lk = lane >> 4;
    const int K = w.K, N = w.N, nk = (K + BK - 1) / BK, k_tail = K % BK;
    const int ncols = min(N - col0, PIPE_BN);
    __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(static_cast<const bf16_t*>(w.A)) + (size_t)row0 * K, 0, (row_end - row0) * K * 2, 0x00020000);
    __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(static_cast<const bf16_t*>(w.B)) + (size_t)col0 * K, 0, ncols * K * 2, 0x00020000);
    // source offsets of this lane in the 2 (A) + 4 (B) load instructions of this wave per K-tile
    int voffA[2], voffB[4];
    const int row_in = lane >> 3, pos = lane & 7;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int row = (wave * 2 + j) * 8 + row_in;
        voffA[j] = row * K * 2 + ((pos ^ ((row >> 1) & 7)) << 4);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = (wave * 4 + j) * 8 + row_in;
        voffB[j] = row * K * 2 + ((pos ^ ((row >> 1) & 7)) << 4);
    }
    auto issue = [&](int kt) {
        unsigned char* st = smem + (kt % PIPE_STAGES) * PIPE_STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < 2; ++j)   // producer rows: written by other XCDs during this launch
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (lds_ptr_t)(st + (wave * 2 + j) * 1024), 16, voffA[j], kt * BK * 2, 0, AUX);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (lds_ptr_t)(st + PIPE_BM * 128 + (wave * 4 + j) * 1024), 16, voffB[j],
                                                     kt * BK * 2, 0, 0);
    };
    // operand read offsets: row byte offset and swizzle of this lane's row in each 16-row tile
    int arow[4], asw[4], brow[4], bsw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int ra_ = wm + i * 16 + lr, rb_ = wn + i * 16 + lr;
        arow[i] = ra_ * 128; asw[i] = (ra_ >> 1) & 7;
        brow[i] = PIPE_BM * 128 + rb_ * 128; bsw[i] = (rb_ >> 1) & 7;
    }
    f32x4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    issue(0);
    if (nk > 1) issue(1);
    for (int kt = 0; kt < nk; ++kt) {
        // this wave's loads of stage kt have landed (the 6 of stage kt+1 may still be in flight) ...
        if (kt + 1 < nk) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        bar_lds();   // ... and so have everyone's; everyone has also finished reading stage kt-1
        if (kt + 2 < nk) issue(kt + 2);   // into the stage that was read in iteration kt-1
        const unsigned char* st = smem + (kt % PIPE_STAGES) * PIPE_STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            u16x8_t a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                a[i] = *reinterpret_cast<const u16x8_t*>(st + arow[i] + (((ks * 4 + lk) ^ asw[i]) << 4));
            if (k_tail != 0 && kt == nk - 1) {
                // this lane's 8 elements start at ks * 32 + lk * 8 of the K-tile: clear the pairs beyond K
                const int e0 = ks * 32 + lk * 8;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    u32x4_t v = __builtin_bit_cast(u32x4_t, a[i]);
#pragma unroll
                    for (int q = 0; q < 4; ++q) v[q] = e0 + 2 * q < k_tail ? v[q] : 0u;
                    a[i] = __builtin_bit_cast(u16x8_t, v);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                b[j] = *reinterpret_cast<const u16x8_t*>(st + brow[j] + (((ks * 4 + lk) ^ bsw[j]) << 4));
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = mfma_bf16_16x16x32(a[i], b[j], acc[i][j]);
        }
    }
    // C fragment: element e of lane l is row (l / 16) * 4 + e, column l % 16 of the 16x16 tile; written through
    __amdgpu_buffer_rsrc_t rsC = __builtin_amdgcn_make_buffer_rsrc(w.C + (size_t)row0 * N, 0, (row_end - row0) * N * 4, 0x00020000);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = col0 + wn + j * 16 + lr;
            if (n >= N) continue;
            const float bv = w.bias ? w.bias[n] : 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int lrow = wm + i * 16 + lk * 4 + e;   // rows past the end of the chunk are dropped (buffer bounds)
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][e] + bv), rsC, (lrow * N + n) * 4, 0, AUX);
            }
        }
}

// The same tiles as a launch of its own: C[M, N] = A[M, K] B[N, K]^T + bias, bf16 operands (the input projection
// of the first layer).  One workgroup per tile; consecutive workgroups (dealt round-robin to the XCDs) take the
// column tiles of one row tile, so that a row tile of A is fetched from memory by one round of workgroups.
__global__ __launch_bounds__(REC_THREADS) void lstm_proj_dma_kernel(PipeWork w, int M, int tiles_n) {
    extern __shared__ __attribute__((aligned(16))) unsigned char proj_smem[];
    const int rt = blockIdx.x / tiles_n, ct = blockIdx.x % tiles_n;
    pipe_gemm_tile_dma<false>(w, rt * PIPE_BM, min(M, (rt + 1) * PIPE_BM), ct * PIPE_BN, proj_smem);
}

// Worker loop.  Items are the tiles of all chunks in the order the consumer needs the chunks (DESCEND: last
// chunk first); item -> (chunk, row tile, column tile) is found by walking the chunks, which a worker only ever
// does forwards because the queue hands out increasing items.
template <int MODE, bool DESCEND>
__device__ __forceinline__ void pipe_worker(const PipeWork& w, const PipeLink& pl, unsigned char* smem) {
    __shared__ int s_item[4];    // chunk, local tile, ok
    __shared__ int s_Tg[PIPE_GROUPS];
    const int T_all = pl.T_all;
    for (int g = 0; g < PIPE_GROUPS; ++g) {
        const int tg = grp_steps(w.batch_sizes, T_all, g);
        if (threadIdx.x == 0) s_Tg[g] = tg;
    }
    const int n_chunks = (T_all + PIPE_CT - 1) / PIPE_CT;
    int cur = 0, prefix = 0;     // thread 0's cursor: chunks [0, cur) in queue order hold items [0, prefix)
    for (;;) {
        if (threadIdx.x == 0) {
            const int item = __hip_atomic_fetch_add(w.queue, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int ok = 0, c = 0, local = 0;
            while (cur < n_chunks) {
                c = DESCEND ? n_chunks - 1 - cur : cur;
                const int tiles = pipe_chunk_tiles(w.t_off, pl, c);
                if (item < prefix + tiles) { local = item - prefix; ok = 1; break; }
                prefix += tiles;
                ++cur;
            }
            if (ok) {
                // all producer groups must have completed the chunk's timesteps
                const int t_lo = c * PIPE_CT, t_hi = min(t_lo + PIPE_CT, T_all);
                long long spins = 0;
                for (int g = 0; g < PIPE_GROUPS && ok == 1; ++g) {
                    const int tg = s_Tg[g];
                    const int need = DESCEND ? tg - min(t_lo, tg) : min(t_hi, tg);
                    while (ld_agent(&pl.progress[g]) < need) {
                        ++spins;
                        if ((spins & 255) == 0 && (spins > REC_SPIN_LIMIT || ld_agent(w.err) != 0)) {
                            st_agent(w.err, 1);
                            ok = 0;
                            break;
                        }
                    }
                }
            }
            s_item[0] = c; s_item[1] = local; s_item[2] = ok;
        }
        bar_lds();
        const int c = s_item[0], local = s_item[1], ok = s_item[2];
        bar_lds();                      // s_item may be rewritten from here on
        if (!ok) return;
        const int row0 = pipe_chunk_row0(w.t_off, c), rows = pipe_chunk_rows(w.t_off, T_all, c);
        const int rt = local / pl.tiles_n, ct = local % pl.tiles_n;
        if constexpr (MODE == MODE_BF16)
            pipe_gemm_tile_dma<true>(w, row0 + rt * PIPE_BM, min(row0 + rows, row0 + (rt + 1) * PIPE_BM), ct * PIPE_BN, smem);
        else
            pipe_gemm_tile<MODE, typename LdsElem<MODE>::type>(w, row0 + rt * PIPE_BM, min(row0 + rows, row0 + (rt + 1) * PIPE_BM),
                                                                ct * PIPE_BN, smem);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        bar_lds();
        if (threadIdx.x == 0) __hip_atomic_fetch_add(&pl.done[c], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// This workgroup's XCD and its ticket there (tickets[PIPE_XCDS], zero at launch).
__device__ __forceinline__ int xcc_ticket(int* tickets, int& xcc) {
    __shared__ int s_t, s_x;
    if (threadIdx.x == 0) {
        const int id = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xf;   // HW_REG_XCC_ID, 4 bits
        s_x = id;
        s_t = id < PIPE_XCDS ? __hip_atomic_fetch_add(&tickets[id], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : REC_MAX_GROUP;
    }
    __syncthreads();
    xcc = s_x;
    return s_t;
}

struct PipeFwdArgs {
    RecFwdArgs l0, l1;   // producer (layer 0) and consumer (layer 1)
    PipeLink link;
    PipeWork work;
};
template <int MODE, int TPW, int KS, int NBW, bool STATIC>
__global__ __launch_bounds__(REC_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void lstm_pipe_fwd_kernel(PipeFwdArgs p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int xcc;
    const int rank = xcc_ticket(p.l0.ticket, xcc);
    PipeLink link = p.link;
    link.T_all = p.l0.info[1];
#ifdef VER_REC_PROF
    const bool stamp = threadIdx.x == 0 && rank == 0 && (xcc == 0 || xcc == PIPE_GROUPS || xcc == PIPE_GROUPS + PIPE_GROUPS_C_FWD);
    long long* tl = p.l0.prof + 64 + (xcc == 0 ? 0 : (xcc == PIPE_GROUPS ? 2 : 4));
    if (stamp) tl[0] = wall_clock64();
#endif
    if (xcc < PIPE_GROUPS) {
        if (rank < p.l0.G)
            rec_fwd_body<MODE, TPW, KS, NBW, STATIC, PIPE_PRODUCER>(p.l0, rank, xcc, PIPE_GROUPS, p.l0.flags + xcc * REC_MAX_GROUP,
                                                                    link, smem);
    } else if (xcc < PIPE_GROUPS + PIPE_GROUPS_C_FWD) {
        if (rank < p.l1.G)
            rec_fwd_body<MODE, TPW, KS, NBW, STATIC, PIPE_CONSUMER>(p.l1, rank, xcc - PIPE_GROUPS, PIPE_GROUPS_C_FWD,
                                                                    p.l1.flags + xcc * REC_MAX_GROUP, link, smem);
    } else if (xcc < PIPE_XCDS) {
        pipe_worker<MODE, false>(p.work, link, smem);
    }
#ifdef VER_REC_PROF
    if (stamp) tl[1] = wall_clock64();
#endif
}

struct PipeBwdArgs {
    RecBwdArgs l1, l0;   // producer (layer 1) and consumer (layer 0)
    PipeLink link;
    PipeWork work;
};
template <int MODE, int MT, int KS, int NI>
__global__ __launch_bounds__(REC_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void lstm_pipe_bwd_kernel(PipeBwdArgs p) {
    typedef typename RecGeom<MODE>::E E;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int xcc;
    const int rank = xcc_ticket(p.l1.ticket, xcc);
    PipeLink link = p.link;
    link.T_all = p.l1.info[1];
    if (xcc < PIPE_GROUPS) {
        if (rank < p.l1.G)
            rec_bwd_body<MODE, MT, KS, NI, PIPE_PRODUCER>(p.l1, rank, xcc, PIPE_GROUPS, p.l1.flags + xcc * REC_MAX_GROUP, link, smem);
    } else if (xcc < PIPE_GROUPS + PIPE_GROUPS_C_BWD) {
        if (rank < p.l0.G)
            rec_bwd_body<MODE, MT, KS, NI, PIPE_CONSUMER>(p.l0, rank, xcc - PIPE_GROUPS, PIPE_GROUPS_C_BWD,
                                                          p.l0.flags + xcc * REC_MAX_GROUP, link, smem);
    } else if (xcc < PIPE_XCDS) {
        pipe_worker<MODE, true>(p.work, link, smem);
    }
}

}  // namespace ver
