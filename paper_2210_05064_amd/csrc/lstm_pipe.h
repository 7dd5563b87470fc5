// Two LSTM layers in one launch.  gfx950 only.
//
// Paper: the policy is a multi-layer LSTM (section 4 "Architecture") evaluated over packed minibatches
// (section 2.2).  The time loop of a layer is a chain of hundreds of dependent steps that leaves most of the
// chip idle, and the second layer's step t only needs the first layer's output of step t: so the two time
// loops run side by side, a few timesteps apart, instead of one after the other.
//
//   XCD 0..2   time loop of the producer layer (forward: layer 0; backward: layer 1), one group per XCD
//   XCD 3..5   time loop of the consumer layer, group g on XCD 3 + g
//   XCD 6..7   workers: for every finished chunk of a group's timesteps, the GEMM that turns the producer's rows
//              into the consumer's input (forward: gates_1 = h_0 W_ih1^T + b; backward: dh_0 = dz_1 W_ih1),
//              one 128 x 256 tile at a time
//
// Which pieces a group runs.  A timestep of a time loop costs a fixed latency (one exchange between the group's
// workgroups, ~3 us) plus a little per alive piece, and the launch lasts as long as its slowest group.  The
// pieces are sorted longest first, so they are cut into three blocks of consecutive pieces: group 0 gets the few
// longest ones (its chain of T_max dependent steps is what bounds the launch, so its steps should be the
// cheapest), the last group the many short ones (few steps, each with many pieces).  lstm_pipe_plan_kernel
// picks the two cuts that minimise the largest predicted group time
//     sum over the group's timesteps of (step + piece * b_t + tile * (ceil(b_t / 16) - 1)),   b_t = alive pieces of the group
// (a time loop works through the alive pieces 16 at a time: the MFMA's columns), which it evaluates per candidate
// from the pieces' lengths: sum_t b_t = sum of the block's lengths (a prefix sum), and the timesteps with more
// than 16 k alive pieces are those of the block's piece number 16 k.  Producer and
// consumer group g run the same block, and everything between them is per group: chunks of the group's own
// timesteps, tiles over the group's own rows (gathered: a group's rows of a timestep are consecutive, those of
// a chunk are not), a queue and completion counters of its own.  So a group never waits for another one: with
// the pieces dealt round-robin all groups had to march in step, and every step paid for a third of all alive pieces.
//
// Hand-over (lstm_rec.h, PipeLink): producer rows are written through to memory and their completion is
// published per group; a worker takes the next tile of a group's queue, waits for that group's producer, reads
// the chunk's rows with loads that bypass the non-coherent caches, writes its tile through, waits for the stores
// and counts the tile in done[group][chunk]; the consumer group waits until that count has reached the number of
// tiles of the chunk.  Waiting only ever points backwards along producer -> worker -> consumer and a queue hands
// out a group's tiles in the order its consumer needs them, so the launch cannot deadlock; every wait is bounded
// and raises the shared error word on time-out.
#pragma once
#include "lstm_rec.h"

namespace ver {

constexpr int PIPE_GROUPS = 3;       // groups (XCDs) per layer
constexpr int PIPE_XCDS = 8;         // XCDs of the chip: those beyond the two layers' groups are workers
constexpr int PIPE_WORKERS = (PIPE_XCDS - 2 * PIPE_GROUPS) * REC_MAX_GROUP;
static_assert(PIPE_XCDS - 2 * PIPE_GROUPS == 2, "the workers split the column tiles between two XCDs");

// The plan of a launch (ints in global memory, written by lstm_pipe_plan_kernel):
constexpr int PLAN_KB = 0;           // [PIPE_GROUPS + 1] first piece of every group's block, then the number of pieces
constexpr int PLAN_T = 8;            // [PIPE_GROUPS] timesteps of the group (those of its first piece; 0 if it has none)
constexpr int PLAN_CT = 12;          // [PIPE_GROUPS] timesteps per chunk
constexpr int PLAN_HDR = 16;         // then rp[PIPE_GROUPS][M + 1]: rows of the group in the timesteps before t
inline __host__ __device__ size_t plan_words(int M) { return PLAN_HDR + (size_t)PIPE_GROUPS * ((size_t)M + 1); }
inline __host__ __device__ size_t plan_scratch_floats(int M) { return 2 * ((size_t)M + 1); }
// The words a launch synchronises through (zero at launch): progress[g] at g, queue[g][half] at 8 + g + PIPE_GROUPS * half, then
// done[g][chunk] from 16 with PIPE_GROUPS rows of pipe_done_stride(M) words.
constexpr int PIPE_CT_MIN = 4;
inline __host__ __device__ int pipe_done_stride(int M) { return M / PIPE_CT_MIN + 2; }
inline __host__ __device__ int pipe_sync_words(int M) { return 16 + PIPE_GROUPS * pipe_done_stride(M); }

// Predicted microseconds of a timestep: step + piece * b + tile * (ceil(b / 16) - 1) (b alive pieces of the group;
// least-squares fit to the measured times of the groups of 16 minibatches of the paper's largest configuration:
// residual 26 us (forward) and 31 us (backward) rms on group times of 0.8-2 ms), and the timesteps per chunk: at most ct0 for group 0 (every timestep of a chunk delays the
// end of the launch once), at most ct for the other groups (which have time to spare: fewer, fuller tiles), and
// no more than chunk_rows / (pieces of the group): the consumer of a group ends one chunk of GEMM tiles and one
// chunk of its own steps after the producer, and starts as much later.
struct PlanCost {
    float step, piece, tile;
    int ct0, ct, chunk_rows;
};
#ifndef VER_PLAN_CT0
#define VER_PLAN_CT0 8
#endif
#ifndef VER_PLAN_CT
#define VER_PLAN_CT 16
#endif
#ifndef VER_PLAN_CHUNK_ROWS
#define VER_PLAN_CHUNK_ROWS 256
#endif
constexpr PlanCost PLAN_COST_FWD = {2.96f, 0.082f, 1.48f, VER_PLAN_CT0, VER_PLAN_CT, VER_PLAN_CHUNK_ROWS};
#ifndef VER_PLAN_CT0_BWD
#define VER_PLAN_CT0_BWD VER_PLAN_CT0
#endif
constexpr PlanCost PLAN_COST_BWD = {2.83f, 0.167f, 1.95f, VER_PLAN_CT0_BWD, VER_PLAN_CT, VER_PLAN_CHUNK_ROWS};

struct PipeWork {
    const void* A;      // producer rows [M, K], operand type (forward: h, backward: dz)
    const void* B;      // [N, K] operand type, K contiguous
    float* C;           // [M, N]
    const float* bias;  // [N] or NULL
    int K, N, M;
    const int32_t* t_off;
    const int* plan;
    int* sync;          // progress, queues, done counters (see above)
    int* err;
    long long* prof_all;   // profiling words (only touched by builds with VER_REC_PROF)
};

constexpr int PLAN_THREADS = 1024;
// Exclusive prefix sums of N values per thread over the 1024 threads of the block (thread order); total: the sums.
// s_w: 16 * N words of LDS.
template <typename T, int N>
__device__ __forceinline__ void plan_scan(T (&v)[N], T* s_w, T (&total)[N]) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    T inc[N];
#pragma unroll
    for (int i = 0; i < N; ++i) inc[i] = v[i];
#pragma unroll
    for (int d = 1; d < 64; d <<= 1)
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const T o = __shfl_up(inc[i], d, VER_WAVE);
            if (lane >= d) inc[i] += o;
        }
    if (lane == 63)
#pragma unroll
        for (int i = 0; i < N; ++i) s_w[wave * N + i] = inc[i];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < N; ++i) {
        T off = 0, tot = 0;
        for (int w = 0; w < PLAN_THREADS / 64; ++w) {
            const T x = s_w[w * N + i];
            if (w < wave) off += x;
            tot += x;
        }
        total[i] = tot;
        v[i] = off + inc[i] - v[i];
    }
    __syncthreads();
}

// The plans of the forward and of the backward launch of one minibatch (the same packing, two cost models).
// IN_LDS: the batch sizes and the per-piece arrays (lengths and their prefix sums) live in LDS (up to PLAN_LDS_N
// pieces and timesteps: the search for the cuts is a chain of dependent reads of them), else in global memory.
constexpr int PLAN_LDS_N = 4096;
constexpr int PLAN_DIRS = 2;
template <bool IN_LDS>
__device__ __forceinline__ void plan_body(const int32_t* __restrict__ batch_sizes, int M, int n_seq, int T, int* __restrict__ plan_fwd,
                                          int* __restrict__ plan_bwd, float* __restrict__ scratch, int* s_bs, float* s_len, float* s_S1,
                                          const PlanCost& pc_fwd, const PlanCost& pc_bwd) {
    constexpr int WAVES = PLAN_THREADS / 64, NR = PLAN_DIRS * PIPE_GROUPS;
    __shared__ float s_wf[WAVES];
    __shared__ int s_wi[WAVES * NR];
    __shared__ float s_obj[WAVES];
    __shared__ int s_k1[WAVES], s_k2[WAVES];
    __shared__ int s_kb[PLAN_DIRS][PIPE_GROUPS + 1];
    const int tid = threadIdx.x;
    const int32_t* bs = batch_sizes;
    if (IN_LDS) {
        for (int t = tid; t < T; t += PLAN_THREADS) s_bs[t] = batch_sizes[t];
        __syncthreads();
        bs = s_bs;
    }
    float* len = IN_LDS ? s_len : scratch;          // [n_seq] timesteps of piece n
    float* S1 = IN_LDS ? s_S1 : scratch + M + 1;    // [n_seq + 1] sum of len[j], j < n
    for (int t = tid; t < T; t += PLAN_THREADS) {
        const int hi = min(bs[t], n_seq), lo = t + 1 < T ? min(bs[t + 1], n_seq) : 0;
        for (int n = lo; n < hi; ++n) len[n] = (float)(t + 1);   // the pieces that end with timestep t
    }
    __syncthreads();
    float c1 = 0.f;
    for (int b0 = 0; b0 < n_seq; b0 += PLAN_THREADS) {
        const int n = b0 + tid;
        float l[1] = {n < n_seq ? len[n] : 0.f}, t1[1];
        plan_scan<float, 1>(l, s_wf, t1);
        if (n < n_seq) S1[n] = c1 + l[0];
        c1 += t1[0];
    }
    if (tid == 0) S1[n_seq] = c1;
    __syncthreads();
    // The first half of the block searches the cuts of the forward plan, the second half those of the backward plan.
    const int dir = tid / (PLAN_THREADS / PLAN_DIRS), rank = tid % (PLAN_THREADS / PLAN_DIRS);
    const PlanCost pc = dir == 0 ? pc_fwd : pc_bwd;
    // predicted time of a group that runs the pieces [lo, hi)
    auto cost = [&](int lo, int hi) -> float {
        if (hi <= lo) return 0.f;
        // timesteps with more than 16, 32, ... alive pieces; beyond 64 such terms the rest by the midpoint rule
        float P = 0.f;
        int k = lo + 16;
        for (int i = 0; i < 64 && k < hi; ++i, k += 16) P += len[k];
        if (k < hi) P += (S1[hi] - S1[k - 8]) * (1.f / 16.f);
        return pc.step * len[lo] + pc.piece * (S1[hi] - S1[lo]) + pc.tile * P;
    };
    // every first cut k1 with the second cut that balances the two remaining groups; ties go to the smaller cuts
    float best = 3.0e38f;
    int bk1 = n_seq, bk2 = n_seq;
    for (int k1 = 1 + rank; k1 <= n_seq; k1 += PLAN_THREADS / PLAN_DIRS) {
        int lo = k1, hi = n_seq;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (cost(k1, mid) >= cost(mid, n_seq)) hi = mid; else lo = mid + 1;
        }
        const float c0 = cost(0, k1);
        for (int k2 = max(lo - 1, k1); k2 <= lo; ++k2) {
            const float obj = fmaxf(c0, fmaxf(cost(k1, k2), cost(k2, n_seq)));
            if (obj < best) { best = obj; bk1 = k1; bk2 = k2; }
        }
    }
    // smallest (objective, k1, k2) of each half: inside the waves by shuffles, then over the half's waves
    auto better = [](float o, int o1, int o2, float m, int m1, int m2) { return o < m || (o == m && (o1 < m1 || (o1 == m1 && o2 < m2))); };
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const float o = __shfl_xor(best, d, VER_WAVE);
        const int o1 = __shfl_xor(bk1, d, VER_WAVE), o2 = __shfl_xor(bk2, d, VER_WAVE);
        if (better(o, o1, o2, best, bk1, bk2)) { best = o; bk1 = o1; bk2 = o2; }
    }
    if ((tid & 63) == 0) { s_obj[tid >> 6] = best; s_k1[tid >> 6] = bk1; s_k2[tid >> 6] = bk2; }
    __syncthreads();
    if (rank == 0) {
        for (int w = dir * (WAVES / PLAN_DIRS) + 1; w < (dir + 1) * (WAVES / PLAN_DIRS); ++w)
            if (better(s_obj[w], s_k1[w], s_k2[w], best, bk1, bk2)) { best = s_obj[w]; bk1 = s_k1[w]; bk2 = s_k2[w]; }
        s_kb[dir][0] = 0; s_kb[dir][1] = bk1; s_kb[dir][2] = bk2; s_kb[dir][3] = n_seq;
        int* plan = dir == 0 ? plan_fwd : plan_bwd;
        for (int g = 0; g <= PIPE_GROUPS; ++g) plan[PLAN_KB + g] = s_kb[dir][g];
    }
    __syncthreads();
    // per plan and group: its timesteps, its chunk length, and its rows before every timestep (all six prefix sums at once)
    int lo_[NR], cap_[NR], Tg_[NR], carry[NR];
    int Tmax = 0;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const int d = r / PIPE_GROUPS, g = r % PIPE_GROUPS;
        lo_[r] = s_kb[d][g];
        cap_[r] = s_kb[d][g + 1] - lo_[r];
        Tg_[r] = cap_[r] > 0 ? (int)len[lo_[r]] : 0;
        carry[r] = 0;
        Tmax = max(Tmax, Tg_[r]);
        if (tid == 0) {
            int* plan = d == 0 ? plan_fwd : plan_bwd;
            const PlanCost& c = d == 0 ? pc_fwd : pc_bwd;
            plan[PLAN_T + g] = Tg_[r];
            plan[PLAN_CT + g] = min(g == 0 ? c.ct0 : c.ct, max(PIPE_CT_MIN, c.chunk_rows / max(cap_[r], 1)));
        }
    }
    for (int b0 = 0; b0 < Tmax; b0 += PLAN_THREADS) {
        const int t = b0 + tid;
        const int b = t < Tmax ? bs[t] : 0;
        int cnt[NR], tot[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) cnt[r] = t < Tg_[r] ? min(max(b - lo_[r], 0), cap_[r]) : 0;
        plan_scan<int, NR>(cnt, s_wi, tot);
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            int* rp = (r / PIPE_GROUPS == 0 ? plan_fwd : plan_bwd) + PLAN_HDR + (size_t)(r % PIPE_GROUPS) * ((size_t)M + 1);
            if (t < Tg_[r]) rp[t] = carry[r] + cnt[r];
            carry[r] += tot[r];
        }
    }
    if (tid == 0)
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            int* rp = (r / PIPE_GROUPS == 0 ? plan_fwd : plan_bwd) + PLAN_HDR + (size_t)(r % PIPE_GROUPS) * ((size_t)M + 1);
            rp[Tg_[r]] = carry[r];
        }
}

// One workgroup, in front of the forward launch: clears that launch's synchronisation words and writes the plans of
// the forward and of the backward launch (see the top of this file).  scratch: plan_scratch_floats(M) floats.
__global__ __launch_bounds__(PLAN_THREADS) void lstm_pipe_plan_kernel(const int32_t* __restrict__ info, const int32_t* __restrict__ batch_sizes,
                                                                      int M, int* __restrict__ plan_fwd, int* __restrict__ plan_bwd,
                                                                      float* __restrict__ scratch, int* __restrict__ clear_first, int n_clear,
                                                                      PlanCost pc_fwd, PlanCost pc_bwd) {
    __shared__ int s_bs[PLAN_LDS_N];
    __shared__ float s_len[PLAN_LDS_N], s_S1[PLAN_LDS_N + 1];
    const int n_seq = min(max(info[0], 0), M), T = min(max(info[1], 0), M);
    for (int i = threadIdx.x; i < n_clear; i += PLAN_THREADS) clear_first[i] = 0;
    if (n_seq <= PLAN_LDS_N && T <= PLAN_LDS_N)
        plan_body<true>(batch_sizes, M, n_seq, T, plan_fwd, plan_bwd, scratch, s_bs, s_len, s_S1, pc_fwd, pc_bwd);
    else
        plan_body<false>(batch_sizes, M, n_seq, T, plan_fwd, plan_bwd, scratch, s_bs, s_len, s_S1, pc_fwd, pc_bwd);
}

template <typename E, typename T> __device__ __forceinline__ Quad<E> load_quad_coh(__amdgpu_buffer_rsrc_t r, int byte_off);
template <> __device__ __forceinline__ Quad<float> load_quad_coh<float, float>(__amdgpu_buffer_rsrc_t r, int byte_off) {
    const u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 17);
    return Quad<float>{{__uint_as_float(t[0]), __uint_as_float(t[1]), __uint_as_float(t[2]), __uint_as_float(t[3])}};
}
template <> __device__ __forceinline__ Quad<bf16_t> load_quad_coh<bf16_t, bf16_t>(__amdgpu_buffer_rsrc_t r, int byte_off) {
    const u32x2_t t = __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, 17);
    return Quad<bf16_t>{{(bf16_t)(t.x & 0xffff), (bf16_t)(t.x >> 16), (bf16_t)(t.y & 0xffff), (bf16_t)(t.y >> 16)}};
}

// A row that a tile does not have: an offset beyond every buffer (loads return zero, stores are dropped), which
// stays there when a K-tile's offset is added.
constexpr int PIPE_NO_ROW = (int)0x80000000u;

// One 128 x 256 tile of C = A B^T (+ bias) for the rows rowmap[0 .. 127] (LDS; -1: none) and columns from col0,
// by 8 waves (2 x 4 of 64 x 64).  Same K-tile pipeline as gemm_kernel: the next K-tile's global loads are in
// flight while the current one is multiplied out of LDS.
// nrows: the tile's rows are its first nrows; a wave whose 64 rows hold none of them does not multiply, one that holds
// at most 16 multiplies only its first 16-row tile (an fp32 tile is bound by its MFMAs, 16 times slower per FLOP
// than bf16 ones: the tiles of a group with one or two pieces would otherwise cost as much as full ones).
template <int MODE, typename TA>
__device__ __forceinline__ void pipe_gemm_tile(const PipeWork& w, const int* rowmap, int nrows, int col0, unsigned char* smem) {
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
    __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<TA*>(static_cast<const TA*>(w.A)), 0,
                                                                   w.M * K * (int)sizeof(TA), 0x00020000);
    const E* Bp = static_cast<const E*>(w.B);
    int rowoff[QA];
#pragma unroll
    for (int i = 0; i < QA; ++i) {
        const int g = rowmap[r + i * RPP];
        rowoff[i] = g >= 0 ? g * K * (int)sizeof(TA) : PIPE_NO_ROW;
    }

    f32x4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    Quad<E> ra[QA], rb[QB];
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int i = 0; i < QA; ++i) {
            ra[i] = load_quad_coh<E, TA>(rsA, rowoff[i] + (k0 + c * 4) * (int)sizeof(TA));   // rows the tile does not have read zero
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
        const int nr = nrows - wm;   // rows of the tile among this wave's 64 (uniform in the wave)
        if (nr <= 0) {
            // nothing to multiply
        } else if (MODE == MODE_F32 && nr <= 16) {
#pragma unroll
            for (int ks = 0; ks < BK; ks += 16) {
                const f32x4_t a0 = *reinterpret_cast<const f32x4_t*>(reinterpret_cast<const float*>(sA) + (wm + lr) * STRIDE + ks + lk * 4);
                f32x4_t b[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    b[j] = *reinterpret_cast<const f32x4_t*>(reinterpret_cast<const float*>(sB) + (wn + j * 16 + lr) * STRIDE + ks + lk * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[0][j] = mfma_f32_16x16x4(a0[e], b[j][e], acc[0][j]);
            }
        } else if (MODE == MODE_BF16) {
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
    __amdgpu_buffer_rsrc_t rsC = __builtin_amdgcn_make_buffer_rsrc(w.C, 0, w.M * N * 4, 0x00020000);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int crow[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int g = rowmap[wm + i * 16 + lk * 4 + e];
            crow[e] = g >= 0 ? g * N * 4 : PIPE_NO_ROW;   // rows the tile does not have are dropped (buffer bounds)
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = col0 + wn + j * 16 + lr;
            if (n >= N) continue;
            const float bv = w.bias ? w.bias[n] : 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][e] + bv), rsC, crow[e] + n * 4, 0, 17);
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
// COHERENT (a worker's tile): the tile's rows are rowmap[0 .. 127] (LDS; -1: none), A is being written by other
// XCDs during this launch and C is read by them (loads and stores that bypass the non-coherent caches).
// Otherwise (a launch of its own): the rows [row0, row_end).
// nrows: the tile's rows are its first nrows (a worker's tile of a group with few pieces holds a handful): the waves
// whose 64 rows hold none of them neither read operands from LDS nor multiply (they still load and synchronise).
template <bool COHERENT>
__device__ __forceinline__ void pipe_gemm_tile_dma(const PipeWork& w, const int* rowmap, int row0, int row_end, int nrows, int col0,
                                                   unsigned char* smem) {
    constexpr int BK = 64;
    constexpr int AUX = COHERENT ? 17 : 0;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave >> 2) * 64, wn = (wave & 3) * 64;
    const int lr = lane & 15, lk = lane >> 4;
    const int K = w.K, N = w.N, nk = (K + BK - 1) / BK, k_tail = K % BK;
    const int ncols = min(N - col0, PIPE_BN);
    __amdgpu_buffer_rsrc_t rsA = COHERENT
        ? __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(static_cast<const bf16_t*>(w.A)), 0, w.M * K * 2, 0x00020000)
        : __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(static_cast<const bf16_t*>(w.A)) + (size_t)row0 * K, 0,
                                            (row_end - row0) * K * 2, 0x00020000);
    __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(static_cast<const bf16_t*>(w.B)) + (size_t)col0 * K, 0, ncols * K * 2, 0x00020000);
    // source offsets of this lane in the 2 (A) + 4 (B) load instructions of this wave per K-tile
    int voffA[2], voffB[4];
    const int row_in = lane >> 3, pos = lane & 7;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int row = (wave * 2 + j) * 8 + row_in;
        int src = row * K * 2;
        if (COHERENT) {
            const int g = rowmap[row];
            src = g >= 0 ? g * K * 2 : PIPE_NO_ROW;
        }
        voffA[j] = src + ((pos ^ ((row >> 1) & 7)) << 4);
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
        if (COHERENT && nrows <= wm) continue;   // (uniform in the wave)
        if (COHERENT && nrows - wm <= 16) {
            // at most 16 rows (the tiles of a group with one or two pieces): only the first of the four 16-row tiles
            // (the workers' K is a whole number of K-tiles: no tail to clear)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const u16x8_t a0 = *reinterpret_cast<const u16x8_t*>(st + arow[0] + (((ks * 4 + lk) ^ asw[0]) << 4));
                u16x8_t b[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    b[j] = *reinterpret_cast<const u16x8_t*>(st + brow[j] + (((ks * 4 + lk) ^ bsw[j]) << 4));
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[0][j] = mfma_bf16_16x16x32(a0, b[j], acc[0][j]);
            }
            continue;
        }
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
    __amdgpu_buffer_rsrc_t rsC = COHERENT ? __builtin_amdgcn_make_buffer_rsrc(w.C, 0, w.M * N * 4, 0x00020000)
                                          : __builtin_amdgcn_make_buffer_rsrc(w.C + (size_t)row0 * N, 0, (row_end - row0) * N * 4, 0x00020000);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int crow[4];   // rows the tile does not have are dropped (buffer bounds)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int lrow = wm + i * 16 + lk * 4 + e;
            crow[e] = lrow * N * 4;
            if (COHERENT) {
                const int g = rowmap[lrow];
                crow[e] = g >= 0 ? g * N * 4 : PIPE_NO_ROW;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = col0 + wn + j * 16 + lr;
            if (n >= N) continue;
            const float bv = w.bias ? w.bias[n] : 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][e] + bv), rsC, crow[e] + n * 4, 0, AUX);
        }
    }
}

// The same tiles as a launch of its own: C[M, N] = A[M, K] B[N, K]^T + bias, bf16 operands (the input projection
// of the first layer).  One workgroup per tile; consecutive workgroups (dealt round-robin to the XCDs) take the
// column tiles of one row tile, so that a row tile of A is fetched from memory by one round of workgroups.
__global__ __launch_bounds__(REC_THREADS) void lstm_proj_dma_kernel(PipeWork w, int M, int tiles_n) {
    extern __shared__ __attribute__((aligned(16))) unsigned char proj_smem[];
    const int rt = blockIdx.x / tiles_n, ct = blockIdx.x % tiles_n;
    pipe_gemm_tile_dma<false>(w, nullptr, rt * PIPE_BM, min(M, (rt + 1) * PIPE_BM), PIPE_BM, ct * PIPE_BN, proj_smem);
}

// One group's view of the hand-over words, from the plan.
__device__ __forceinline__ PipeLink pipe_link_of(const int* plan, int* sync, int M, int tiles_n, int g) {
    PipeLink pl;
    pl.progress = sync + g;
    pl.done = sync + 16 + g * pipe_done_stride(M);
    pl.rp = plan + PLAN_HDR + (size_t)g * ((size_t)M + 1);
    pl.ct = plan[PLAN_CT + g];
    pl.tiles_n = tiles_n;
    pl.T = plan[PLAN_T + g];
    return pl;
}
__device__ __forceinline__ PieceSet pipe_pieces_of(const int* plan, int g) {
    const int lo = plan[PLAN_KB + g];
    return PieceSet{lo, 1, plan[PLAN_KB + g + 1] - lo, g};
}

// Worker loop.  A worker serves one group's queue until it is empty, then the next group's (it starts with the
// group `home`).  The items of a queue are the tiles of the group's chunks in the order the consumer needs the
// chunks (DESCEND: last chunk first); item -> (chunk, row tile, column tile) is found by walking the chunks,
// which a worker only ever does forwards because a queue hands out increasing items.
// half: which of the two worker XCDs this is.  Each takes one half of the column tiles (a queue per group and half), so
// that the slab of the weights it streams again and again is half as large (4 MB at H = 1024: the size of its L2):
// counters show 0.8 instead of 1.4 GB fetched per forward launch and 1.1 instead of 1.5 GB per backward launch of the
// largest configuration, at the same launch times (the re-reads were served by the memory-side cache before).
template <int MODE, bool DESCEND>
__device__ __forceinline__ void pipe_worker(const PipeWork& w, int tiles_n, int home, int half, unsigned char* smem) {
    const int tn_lo = (tiles_n + 1) / 2;
    const int my_tn = half == 0 ? tn_lo : tiles_n - tn_lo, col_first = half == 0 ? 0 : tn_lo;
    if (my_tn == 0) return;   // (a single column tile: the other XCD's)
    __shared__ int s_item[4];    // chunk, local tile, ok (0: leave, 1: tile, 2: queue empty)
    __shared__ int s_rp[PIPE_CT_MAX + 1], s_to[PIPE_CT_MAX];
    __shared__ int s_rowmap[PIPE_BM];
    const int tid = threadIdx.x;
#ifdef VER_REC_PROF
    long long* wst = w.prof_all + 96 + home * 4;   // per home group: tiles, time in tiles, time waiting for producers, time in the queue (100 MHz)
    long long wt = 0;
#endif
    for (int visit = 0; visit < PIPE_GROUPS; ++visit) {
        const int g = (home + visit) % PIPE_GROUPS;
        const PipeLink pl = pipe_link_of(w.plan, w.sync, w.M, tiles_n, g);
        const int lo = w.plan[PLAN_KB + g];
        int* queue = w.sync + 8 + g + PIPE_GROUPS * half;
        const int n_chunks = (pl.T + pl.ct - 1) / pl.ct;
        int cur = 0, prefix = 0;     // thread 0's cursor: chunks [0, cur) in queue order hold items [0, prefix)
        for (;;) {
            if (tid == 0) {
#ifdef VER_REC_PROF
                wt = wall_clock64();
#endif
                int ok = 2, c = 0, local = 0;
                if (cur < n_chunks) {
                    const int item = __hip_atomic_fetch_add(queue, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    while (cur < n_chunks) {
                        c = DESCEND ? n_chunks - 1 - cur : cur;
                        const int tiles = pipe_chunk_tiles(pl, c) / tiles_n * my_tn;   // this half's tiles of the chunk
                        if (item < prefix + tiles) { local = item - prefix; ok = 1; break; }
                        prefix += tiles;
                        ++cur;
                    }
                }
#ifdef VER_REC_PROF
                { const long long now = wall_clock64(); atomicAdd((unsigned long long*)&wst[3], (unsigned long long)(now - wt)); wt = now; }
#endif
                if (ok == 1) {
                    // the group's producer must have completed the chunk's timesteps
                    const int t_lo = c * pl.ct, t_hi = min(t_lo + pl.ct, pl.T);
                    const int need = DESCEND ? pl.T - t_lo : t_hi;
                    long long spins = 0;
                    while (ld_agent(pl.progress) < need) {
                        ++spins;
                        if ((spins & 255) == 0 && (spins > REC_SPIN_LIMIT || ld_agent(w.err) != 0)) {
                            st_agent(w.err, 1);
                            ok = 0;
                            break;
                        }
                    }
                }
                s_item[0] = c; s_item[1] = local; s_item[2] = ok;
#ifdef VER_REC_PROF
                { const long long now = wall_clock64(); atomicAdd((unsigned long long*)&wst[2], (unsigned long long)(now - wt)); wt = now; }
#endif
            }
            bar_lds();
            const int c = s_item[0], local = s_item[1], ok = s_item[2];
            if (ok == 0) return;
            if (ok == 2) { bar_lds(); break; }   // this queue is empty: on to the next group
            // the rows of the tile: the group's rows of the chunk's timesteps, in time order, PIPE_BM at a time
            const int t0 = c * pl.ct, nt = min(pl.ct, pl.T - t0);
            const int rt = local / my_tn, ctile = col_first + local % my_tn;
            if (tid <= nt) s_rp[tid] = pl.rp[t0 + tid];
            if (tid < nt) s_to[tid] = w.t_off[t0 + tid];
            bar_lds();                      // (s_item may be rewritten from here on)
            if (tid < PIPE_BM) {
                const int slot = s_rp[0] + rt * PIPE_BM + tid;
                int row = -1;
                if (slot < s_rp[nt]) {
                    int i = 0;
                    while (s_rp[i + 1] <= slot) ++i;   // ends: s_rp[nt] > slot
                    row = s_to[i] + lo + (slot - s_rp[i]);
                }
                s_rowmap[tid] = row;
            }
            bar_lds();
            if constexpr (MODE == MODE_BF16)
                pipe_gemm_tile_dma<true>(w, s_rowmap, 0, 0, min(PIPE_BM, s_rp[nt] - s_rp[0] - rt * PIPE_BM), ctile * PIPE_BN, smem);
            else
                pipe_gemm_tile<MODE, typename LdsElem<MODE>::type>(w, s_rowmap, min(PIPE_BM, s_rp[nt] - s_rp[0] - rt * PIPE_BM), ctile * PIPE_BN, smem);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            bar_lds();
            if (tid == 0) __hip_atomic_fetch_add(&pl.done[c], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#ifdef VER_REC_PROF
            if (tid == 0) {
                atomicAdd((unsigned long long*)&wst[1], (unsigned long long)(wall_clock64() - wt));
                atomicAdd((unsigned long long*)&wst[0], 1ull);
            }
#endif
        }
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

// The kernels below run one of three roles per workgroup, each with its own set of arguments.  Taken by value, all
// of them are loaded into scalar registers at the top of the kernel and stay there (or rather in spill lanes, from
// where the time loops fetch them again and again); read in place from the kernel-argument segment (the struct is
// the kernel's only parameter, so it sits at its start), a role loads what it uses where it uses it.
template <typename A>
__device__ __forceinline__ const A& pipe_args_in_place(const A&) {
    return *(const A*)__builtin_amdgcn_kernarg_segment_ptr();   // (from the constant address space: only a C-style cast does that)
}

struct PipeFwdArgs {
    RecFwdArgs l0, l1;   // producer (layer 0) and consumer (layer 1)
    PipeWork work;
    int tiles_n;         // column tiles per row tile of the workers' GEMM
};
// Which group's queue a worker serves first: group 0's chunks are short and its consumer must never wait long,
// the last group has the most rows.
__device__ __forceinline__ int pipe_worker_home(int xcc, int rank) {
    const int wid = (xcc - 2 * PIPE_GROUPS) * REC_MAX_GROUP + rank;
    const int k = wid & 7;
    return k < 3 ? 0 : (k < 5 ? 1 : 2);
}
template <int MODE, int TPW, int KS, int NBW, bool STATIC>
__global__ __launch_bounds__(REC_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void lstm_pipe_fwd_kernel(PipeFwdArgs p_by_value) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const PipeFwdArgs& p = pipe_args_in_place<PipeFwdArgs>(p_by_value);
    int xcc;
    const int rank = xcc_ticket(p.l0.ticket, xcc);
    const int g = xcc < PIPE_GROUPS ? xcc : xcc - PIPE_GROUPS;
#ifdef VER_REC_PROF
    const bool stamp = threadIdx.x == 0 && rank == 0 && xcc < PIPE_XCDS;   // when every XCD's first workgroup starts and ends
    long long* tl = p.l0.prof + 64 + xcc * 2;
    if (stamp) tl[0] = wall_clock64();
#endif
    if (xcc < 2 * PIPE_GROUPS) {
        const PipeLink link = pipe_link_of(p.work.plan, p.work.sync, p.work.M, p.tiles_n, g);
        const PieceSet ps = pipe_pieces_of(p.work.plan, g);
        if (xcc < PIPE_GROUPS) {
            if (rank < p.l0.G)
                rec_fwd_body<MODE, TPW, KS, NBW, STATIC, PIPE_PRODUCER>(p.l0, rank, ps, link.T, p.l0.flags + xcc * REC_MAX_GROUP, link, smem);
        } else {
            if (rank < p.l1.G)
                rec_fwd_body<MODE, TPW, KS, NBW, STATIC, PIPE_CONSUMER>(p.l1, rank, ps, link.T, p.l1.flags + xcc * REC_MAX_GROUP, link, smem);
        }
    } else if (xcc < PIPE_XCDS && rank < REC_MAX_GROUP) {
        pipe_worker<MODE, false>(p.work, p.tiles_n, pipe_worker_home(xcc, rank), xcc - 2 * PIPE_GROUPS, smem);
    }
#ifdef VER_REC_PROF
    if (stamp) tl[1] = wall_clock64();
#endif
}

struct PipeBwdArgs {
    RecBwdArgs l1, l0;   // producer (layer 1) and consumer (layer 0)
    PipeWork work;
    int tiles_n;
};
template <int MODE, int MT, int KS, int NI>
__global__ __launch_bounds__(REC_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void lstm_pipe_bwd_kernel(PipeBwdArgs p_by_value) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const PipeBwdArgs& p = pipe_args_in_place<PipeBwdArgs>(p_by_value);
    int xcc;
    const int rank = xcc_ticket(p.l1.ticket, xcc);
    const int g = xcc < PIPE_GROUPS ? xcc : xcc - PIPE_GROUPS;
#ifdef VER_REC_PROF
    const bool stamp = threadIdx.x == 0 && rank == 0 && xcc < PIPE_XCDS;
    long long* tl = p.l1.prof - 16 + 64 + xcc * 2;
    if (stamp) tl[0] = wall_clock64();
#endif
    if (xcc < 2 * PIPE_GROUPS) {
        const PipeLink link = pipe_link_of(p.work.plan, p.work.sync, p.work.M, p.tiles_n, g);
        const PieceSet ps = pipe_pieces_of(p.work.plan, g);
        if (xcc < PIPE_GROUPS) {
            if (rank < p.l1.G)
                rec_bwd_body<MODE, MT, KS, NI, PIPE_PRODUCER>(p.l1, rank, ps, link.T, p.l1.flags + xcc * REC_MAX_GROUP, link, smem);
        } else {
            if (rank < p.l0.G)
                rec_bwd_body<MODE, MT, KS, NI, PIPE_CONSUMER>(p.l0, rank, ps, link.T, p.l0.flags + xcc * REC_MAX_GROUP, link, smem);
        }
    } else if (xcc < PIPE_XCDS && rank < REC_MAX_GROUP) {
        pipe_worker<MODE, true>(p.work, p.tiles_n, pipe_worker_home(xcc, rank), xcc - 2 * PIPE_GROUPS, smem);
    }
#ifdef VER_REC_PROF
    if (stamp) tl[1] = wall_clock64();
#endif
}

}  // namespace ver
