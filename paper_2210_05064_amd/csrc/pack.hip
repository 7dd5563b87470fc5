// ver_pack_minibatch: VER minibatch creation and the packed-sequence layout.
//
// Paper: section 2.2 "Learning mini-batch creation" and "Batching computation
// for learning" (figure 2B/2C).  The exact rule (sequence discovery, keyed
// random order, cut into equal step counts with splitting, longest-first
// order) is stated with the entry point's declaration.
//
// Two kernels per call:
//   pack_index_kernel  one workgroup of 1024 threads builds every integer
//                      output.  All of it is O(S) byte reads plus work on the
//                      K sequences / n_seq pieces, far below a microsecond of
//                      HBM time, so one CU with LDS-staged prefix sums and
//                      wave ballots beats a multi-launch device-wide version.
//   pack_gather_kernel a workgroup per 4 or 8 packed rows: resolves their flat steps
//                      (one search in t_off per workgroup) and copies the rows'
//                      fields with 16-byte accesses.  This is the HBM-bound part:
//                      2*4*D bytes per row (6*D with bf16 output) + small fields.
#include "common.h"

namespace ver {
namespace {

constexpr int IDX_THREADS = 1024;
constexpr int IDX_WAVES = IDX_THREADS / VER_WAVE;

struct PackWs {
    uint8_t* flags;       // [S] bit0 sequence start, bit1 episode start
    int32_t* sf;          // [S] first step of sequence id
    int32_t* sl;          // [S] length of sequence id
    uint32_t* skey;       // [S] sort key of sequence id
    int32_t* order;       // [S] sequence id at random-order position r
    int32_t* sstart;      // [S+1] stream position where position r starts
    int32_t* pf;          // [M] pieces in stream order: first step
    int32_t* plen;        // [M] length
    uint8_t* peps;        // [M] episode start
};

// Inclusive scan over the workgroup; returns this thread's inclusive value and
// the workgroup total through *total.  s_w needs IDX_WAVES + 1 ints.
__device__ __forceinline__ int block_scan_incl(int v, int* s_w, int* total) {
    const int lane = threadIdx.x & (VER_WAVE - 1), wave = threadIdx.x / VER_WAVE;
#pragma unroll
    for (int d = 1; d < VER_WAVE; d <<= 1) {
        int up = __shfl_up(v, d, VER_WAVE);
        if (lane >= d) v += up;
    }
    __syncthreads();  // protect s_w from the previous use
    if (lane == VER_WAVE - 1) s_w[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int w = 0; w < IDX_WAVES; ++w) {
            int t = s_w[w];
            s_w[w] = run;
            run += t;
        }
        s_w[IDX_WAVES] = run;
    }
    __syncthreads();
    *total = s_w[IDX_WAVES];
    return v + s_w[wave];
}

constexpr int IDX_SL_CACHE = 4096;   // sorted piece lengths kept in LDS for the per-timestep counts

// One minibatch's part of an index launch: workgroup i of the launch builds the integer outputs of job i.  The
// minibatches of an update are independent of each other (and of the weights), so all of them can be indexed by
// one launch, one workgroup (one CU) each.
constexpr int PACK_MAX_JOBS = 16;
struct PackJob {
    const uint32_t* seq_key;
    int b;
    PackWs ws;
    int32_t* info;
    int32_t* seq_first;
    int32_t* seq_len;
    uint8_t* seq_eps;
    int32_t* batch_sizes;
    int32_t* t_off;
};
struct PackJobs {
    PackJob j[PACK_MAX_JOBS];
};

__global__ __launch_bounds__(IDX_THREADS) void pack_index_kernel(
    const uint8_t* __restrict__ dones, const int32_t* __restrict__ env_off,
    const uint8_t* __restrict__ env_started_episode, int N, int S, int B, PackJobs jobs) {
    const PackJob& job = jobs.j[blockIdx.x];
    const uint32_t* __restrict__ seq_key = job.seq_key;
    const int b = job.b;
    const PackWs ws = job.ws;
    int32_t* __restrict__ info = job.info;
    int32_t* __restrict__ seq_first = job.seq_first;
    int32_t* __restrict__ seq_len = job.seq_len;
    uint8_t* __restrict__ seq_eps = job.seq_eps;
    int32_t* __restrict__ batch_sizes = job.batch_sizes;
    int32_t* __restrict__ t_off = job.t_off;
    __shared__ int s_w[IDX_WAVES + 1];
    __shared__ int s_cnt[IDX_WAVES + 1];
    __shared__ uint32_t s_key[IDX_THREADS];
    __shared__ int s_len[IDX_THREADS];
    __shared__ int s_misc[4];
    const int tid = threadIdx.x;
    const int lane = tid & (VER_WAVE - 1), wave = tid / VER_WAVE;
    const int M = S / B;
    const int lo = b * M, hi = lo + M;

    // 1. start flags: the step after an episode end ...
    for (int k = tid; k < S; k += IDX_THREADS) ws.flags[k] = (k > 0 && dones[k - 1]) ? 3 : 0;
    __syncthreads();
    // ... and the first step of every non-empty stretch (whose episode flag comes from the caller)
    for (int i = tid; i < N; i += IDX_THREADS) {
        const int k = env_off[i];
        if (env_off[i + 1] > k)
            ws.flags[k] = 1 | ((env_started_episode && env_started_episode[i]) ? 2 : 0);
    }
    __syncthreads();

    // 2. compaction: each wave owns a contiguous chunk of steps; count with ballots, then place.
    const int chunk = ((S + IDX_WAVES - 1) / IDX_WAVES + VER_WAVE - 1) / VER_WAVE * VER_WAVE;
    const int c_lo = min(S, wave * chunk), c_hi = min(S, c_lo + chunk);
    int cnt = 0;
    for (int k0 = c_lo; k0 < c_hi; k0 += 8 * VER_WAVE) {   // 8 loads in flight per lane
        unsigned char f[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + u * VER_WAVE + lane;
            f[u] = k < c_hi ? ws.flags[k] : 0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) cnt += __popcll(__ballot((f[u] & 1) != 0));
    }
    if (lane == 0) s_cnt[wave] = cnt;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int w = 0; w < IDX_WAVES; ++w) {
            int t = s_cnt[w];
            s_cnt[w] = run;
            run += t;
        }
        s_cnt[IDX_WAVES] = run;
    }
    __syncthreads();
    const int K = s_cnt[IDX_WAVES];
    int base = s_cnt[wave];
    for (int k0 = c_lo; k0 < c_hi; k0 += 8 * VER_WAVE) {
        unsigned char f[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + u * VER_WAVE + lane;
            f[u] = k < c_hi ? ws.flags[k] : 0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + u * VER_WAVE + lane;
            const bool st = (f[u] & 1) != 0;
            const unsigned long long mask = __ballot(st);
            if (st) {
                const int id = base + __popcll(mask & ((1ull << lane) - 1ull));
                ws.sf[id] = k;
                ws.skey[id] = seq_key[k];
            }
            base += __popcll(mask);
        }
    }
    __syncthreads();
    for (int s = tid; s < K; s += IDX_THREADS) ws.sl[s] = ((s + 1 < K) ? ws.sf[s + 1] : S) - ws.sf[s];

    // 3. random order: rank of (key, id) by counting, keys tiled through LDS.
    for (int s0 = 0; s0 < K; s0 += IDX_THREADS) {
        const int s = s0 + tid;
        const uint32_t my = (s < K) ? ws.skey[s] : 0u;
        int rank = 0;
        for (int q0 = 0; q0 < K; q0 += IDX_THREADS) {
            __syncthreads();
            if (q0 + tid < K) s_key[tid] = ws.skey[q0 + tid];
            __syncthreads();
            const int n = min(IDX_THREADS, K - q0);
            if (s < K)
                for (int q = 0; q < n; ++q) {
                    const uint32_t other = s_key[q];
                    rank += (other < my || (other == my && q0 + q < s)) ? 1 : 0;
                }
        }
        if (s < K) ws.order[rank] = s;
    }
    __syncthreads();

    // 4. stream positions: exclusive prefix sum of the lengths in random order, staged in LDS.
    int run = 0;
    for (int r0 = 0; r0 < K; r0 += IDX_THREADS) {
        const int r = r0 + tid;
        const int len = (r < K) ? ws.sl[ws.order[r]] : 0;
        int total;
        const int incl = block_scan_incl(len, s_w, &total);
        if (r < K) ws.sstart[r] = run + incl - len;
        run += total;
    }
    if (tid == 0) ws.sstart[K] = run;  // == S
    __syncthreads();

    // 5. pieces of minibatch b, in stream order.
    int before = 0, inside = 0;  // sequences ending at or before lo; sequences overlapping [lo, hi)
    for (int r = tid; r < K; r += IDX_THREADS) {
        const int st = ws.sstart[r], en = ws.sstart[r + 1];
        before += (en <= lo) ? 1 : 0;
        inside += (st < hi && en > lo) ? 1 : 0;
    }
    int r_lo, n_seq;
    block_scan_incl(before, s_w, &r_lo);
    block_scan_incl(inside, s_w, &n_seq);
    for (int j = tid; j < n_seq; j += IDX_THREADS) {
        const int r = r_lo + j;
        const int s = ws.order[r];
        const int st = ws.sstart[r], en = ws.sstart[r + 1];
        const int c0 = max(st, lo), c1 = min(en, hi);
        ws.pf[j] = ws.sf[s] + (c0 - st);
        ws.plen[j] = c1 - c0;
        ws.peps[j] = (c0 == st) ? ((ws.flags[ws.sf[s]] >> 1) & 1) : 0;
    }
    __syncthreads();

    // 6. longest first, ties in stream order: rank by counting, lengths tiled through LDS.
    for (int j0 = 0; j0 < n_seq; j0 += IDX_THREADS) {
        const int j = j0 + tid;
        const int my = (j < n_seq) ? ws.plen[j] : 0;
        int rank = 0;
        for (int q0 = 0; q0 < n_seq; q0 += IDX_THREADS) {
            __syncthreads();
            if (q0 + tid < n_seq) s_len[tid] = ws.plen[q0 + tid];
            __syncthreads();
            const int n = min(IDX_THREADS, n_seq - q0);
            if (j < n_seq)
                for (int q = 0; q < n; ++q) {
                    const int other = s_len[q];
                    rank += (other > my || (other == my && q0 + q < j)) ? 1 : 0;
                }
        }
        if (j < n_seq) {
            seq_first[rank] = ws.pf[j];
            seq_len[rank] = my;
            seq_eps[rank] = ws.peps[j];
        }
    }
    __syncthreads();
    const int t_max = n_seq > 0 ? seq_len[0] : 0;

    // 7. rows per timestep and their offsets.  Only the first t_max timesteps have rows: they are counted by a
    // binary search over the sorted lengths (kept in LDS as far as they fit) and scanned; the rest is filled in.
    __shared__ int s_sl[IDX_SL_CACHE];
    for (int j = tid; j < min(n_seq, IDX_SL_CACHE); j += IDX_THREADS) s_sl[j] = seq_len[j];
    __syncthreads();
    run = 0;
    int t_done = 0;
    for (int t0 = 0; t0 < t_max; t0 += IDX_THREADS) {
        const int t = t0 + tid;
        int bs = 0;
        if (t < t_max) {
            // pieces are sorted by length descending: count those with length > t
            int a = 0, z = n_seq;  // invariant: seq_len[a-1] > t (or a == 0), seq_len[z] <= t (or z == n_seq)
            while (a < z) {
                const int mid = (a + z) >> 1;
                const int len = mid < IDX_SL_CACHE ? s_sl[mid] : seq_len[mid];
                if (len > t) a = mid + 1; else z = mid;
            }
            bs = a;
        }
        int total;
        const int incl = block_scan_incl(bs, s_w, &total);
        if (t < M) batch_sizes[t] = bs;
        if (t <= M) t_off[t] = run + incl - bs;
        run += total;
        t_done = t0 + IDX_THREADS;
    }
    for (int t = t_done + tid; t <= M; t += IDX_THREADS) {   // run == M here (or 0 when the minibatch is empty)
        if (t < M) batch_sizes[t] = 0;
        t_off[t] = run;
    }
    if (tid == 0) {
        info[0] = n_seq;
        info[1] = t_max;
        info[2] = K;
        info[3] = 0;
    }
    (void)s_misc;
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f) {
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

constexpr int GATHER_THREADS = 256;
constexpr int GATHER_WAVES = GATHER_THREADS / VER_WAVE;

struct GatherArgs {
    const int32_t* info;
    const int32_t* seq_first;
    const uint8_t* seq_eps;
    const int32_t* t_off;
    int32_t* gather_idx;
    int M, S;
    const float* obs; int D; void* obs_packed; int obs_bf16;
    const uint8_t* actions; int act_bytes; uint8_t* actions_packed;
    const float* logp_old; const float* adv; const float* ret; const float* is_weight;
    float* logp_old_packed; float* adv_packed; float* ret_packed; float* is_weight_packed;
    const float* rnn_h; const float* rnn_c; int n_layers, H, seq_cap;
    float* h0; float* c0;
    bool state_vec4;   // H and the four state pointers allow 16-byte accesses
};

// One wave copies (or zeroes) a row of n floats.  The few rows of timestep 0 carry every layer's h and c (16 KB at
// two layers of 1024 units), far more than any other row: with 16-byte accesses and four loads in flight they no
// longer are the tail the whole launch waits for.
__device__ __forceinline__ void copy_state_row(float* __restrict__ dst, const float* __restrict__ src, int n, int lane,
                                               bool zero, bool vec4) {
    if (vec4) {
        const f32x4* s4 = reinterpret_cast<const f32x4*>(src);
        f32x4* d4 = reinterpret_cast<f32x4*>(dst);
        const int n4 = n / 4;
        for (int i0 = lane; i0 < n4; i0 += 4 * VER_WAVE) {
            f32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * VER_WAVE;
                v[u] = (zero || i >= n4) ? f32x4{0.f, 0.f, 0.f, 0.f} : s4[i];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * VER_WAVE;
                if (i < n4) d4[i] = v[u];
            }
        }
    } else {
        for (int i = lane; i < n; i += VER_WAVE) dst[i] = zero ? 0.f : src[i];
    }
}

// Packed rows per workgroup: 8 (two per wave) when a launch moves gigabytes (measured on 2^18 rows: 4 -> 57 %, 8 -> 61 %,
// 16 -> 59 %, 32 -> 57 % of the HBM peak), 4 (one per wave) for minibatches of the paper's sizes, where the launch is a
// matter of latency and more, shorter workgroups finish sooner (8192 rows: 22 us against 29).
constexpr int GATHER_ROWS_BIG = 8, GATHER_ROWS_SMALL = 4, GATHER_BIG_FROM = 1 << 16;

// Copies the observation rows A and (unless inB is null) B, n4 16-byte chunks each, with the loads of both rows
// in flight before the first store (a row is read once, from memory).  BF16: converts to bf16 on the way.
template <bool BF16>
__device__ __forceinline__ void copy_obs_pair(const f32x4* __restrict__ inA, const f32x4* __restrict__ inB,
                                              void* __restrict__ outA, void* __restrict__ outB, int n4, int lane) {
    for (int c0 = 0; c0 < n4; c0 += 4 * VER_WAVE) {
        f32x4 va[4], vb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (c0 + u * VER_WAVE >= n4) break;   // (uniform: whole chunk groups beyond the row are skipped)
            const int i = c0 + u * VER_WAVE + lane;
            // (ordinary loads: non-temporal ones measured 2 % slower here, non-temporal stores 1 % slower)
            va[u] = inA[i < n4 ? i : c0];
            if (inB) vb[u] = inB[i < n4 ? i : c0];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (c0 + u * VER_WAVE >= n4) break;
            const int i = c0 + u * VER_WAVE + lane;
            if (i >= n4) continue;
            if (BF16) {
                u16x4 o;
                o.x = f32_to_bf16_rne(va[u].x); o.y = f32_to_bf16_rne(va[u].y);
                o.z = f32_to_bf16_rne(va[u].z); o.w = f32_to_bf16_rne(va[u].w);
                static_cast<u16x4*>(outA)[i] = o;
                if (inB) {
                    o.x = f32_to_bf16_rne(vb[u].x); o.y = f32_to_bf16_rne(vb[u].y);
                    o.z = f32_to_bf16_rne(vb[u].z); o.w = f32_to_bf16_rne(vb[u].w);
                    static_cast<u16x4*>(outB)[i] = o;
                }
            } else {
                static_cast<f32x4*>(outA)[i] = va[u];
                if (inB) static_cast<f32x4*>(outB)[i] = vb[u];
            }
        }
    }
}

// A workgroup gathers GATHER_ROWS (4 or 8) consecutive packed rows.  Wave 0 places them: a 64-ary search in t_off for the
// timestep of the first row (every lane probes one of 64 evenly spaced offsets of the current range and a ballot
// counts how many are <= p: 3 dependent loads for 8192 timesteps), then ONE load of the next offsets, from which
// every row's timestep follows by counting (a timestep holds at least one row, so n rows span at most n
// timesteps), then one load of the piece's first step.  After that all four waves copy rows, two rows and up to
// eight 16-byte loads per lane in flight at a time, and the small per-row fields go lane-parallel over the rows.
template <int GATHER_ROWS>
__global__ __launch_bounds__(GATHER_THREADS) void pack_gather_kernel(GatherArgs g) {
    __shared__ int s_src[GATHER_ROWS], s_t[GATHER_ROWS], s_j[GATHER_ROWS];
    const int tid = threadIdx.x, lane = tid & (VER_WAVE - 1), wave = tid / VER_WAVE;
    const int p0 = blockIdx.x * GATHER_ROWS;
    const int nrows = min(GATHER_ROWS, g.M - p0);
    if (nrows <= 0) return;
    const int n_seq = g.info[0], t_max = g.info[1];
    if (wave == 0) {
        int a = 0, z = t_max;  // invariant: t_off[a] <= p0 < t_off[z]
        while (z - a > 1) {
            const int step = (z - a + VER_WAVE - 1) / VER_WAVE;
            const int idx = a + lane * step;
            const bool le = idx < z && g.t_off[idx] <= p0;      // true for a prefix of the lanes (lane 0 always)
            const int cnt = max(1, (int)__popcll(__ballot(le)));
            a += (cnt - 1) * step;
            z = min(z, a + step);
        }
        // lane l: t_off[a + l] for l = 0 .. GATHER_ROWS (t_off[t_max] = M lies above every row)
        const int o = g.t_off[min(a + min(lane, GATHER_ROWS), t_max)];
        const int p = p0 + min(lane, nrows - 1);
        int cnt = 0;
#pragma unroll
        for (int i = 1; i <= GATHER_ROWS; ++i) cnt += (__shfl(o, i, VER_WAVE) <= p) ? 1 : 0;
        cnt = min(cnt, GATHER_ROWS - 1);   // (holds for well-formed offsets; keeps the shuffle below in range otherwise)
        const int t = a + cnt;
        const int j = p - __shfl(o, cnt, VER_WAVE);
        if (lane < nrows) {
            const int src = g.seq_first[j] + t;
            s_src[lane] = src; s_t[lane] = t; s_j[lane] = j;
            g.gather_idx[p] = src;
        }
    }
    __syncthreads();

    if (g.obs && g.obs_packed) {
        if ((g.D & 3) == 0) {
            const int n4 = g.D / 4;
            const size_t out_row = (size_t)g.D * (g.obs_bf16 ? 2 : 4);
            for (int r = wave; r < nrows; r += 2 * GATHER_WAVES) {
                const int rb = r + GATHER_WAVES;
                const f32x4* inA = reinterpret_cast<const f32x4*>(g.obs + (size_t)s_src[r] * g.D);
                const f32x4* inB = rb < nrows ? reinterpret_cast<const f32x4*>(g.obs + (size_t)s_src[rb] * g.D) : nullptr;
                char* outA = static_cast<char*>(g.obs_packed) + (size_t)(p0 + r) * out_row;
                char* outB = static_cast<char*>(g.obs_packed) + (size_t)(p0 + rb) * out_row;
                if (g.obs_bf16) copy_obs_pair<true>(inA, inB, outA, outB, n4, lane);
                else copy_obs_pair<false>(inA, inB, outA, outB, n4, lane);
            }
        } else {
            for (int r = wave; r < nrows; r += GATHER_WAVES) {
                const float* in = g.obs + (size_t)s_src[r] * g.D;
                const size_t po = (size_t)(p0 + r) * g.D;
                for (int i = lane; i < g.D; i += VER_WAVE) {
                    if (g.obs_bf16) static_cast<unsigned short*>(g.obs_packed)[po + i] = f32_to_bf16_rne(in[i]);
                    else static_cast<float*>(g.obs_packed)[po + i] = in[i];
                }
            }
        }
    }
    if (g.actions && g.actions_packed) {
        if ((g.act_bytes & 3) == 0) {
            const int aw = g.act_bytes / 4;
            for (int i = tid; i < nrows * aw; i += GATHER_THREADS) {
                const int r = i / aw, c = i - r * aw;
                reinterpret_cast<int32_t*>(g.actions_packed + (size_t)(p0 + r) * g.act_bytes)[c] =
                    reinterpret_cast<const int32_t*>(g.actions + (size_t)s_src[r] * g.act_bytes)[c];
            }
        } else {
            for (int i = tid; i < nrows * g.act_bytes; i += GATHER_THREADS) {
                const int r = i / g.act_bytes, c = i - r * g.act_bytes;
                g.actions_packed[(size_t)(p0 + r) * g.act_bytes + c] = g.actions[(size_t)s_src[r] * g.act_bytes + c];
            }
        }
    }
    // the per-row scalars: field f of row r in thread f * GATHER_ROWS + r
    for (int i = tid; i < 4 * nrows; i += GATHER_THREADS) {
        const int f = i / nrows, r = i - f * nrows;
        const int src = s_src[r], p = p0 + r;
        if (f == 0 && g.logp_old && g.logp_old_packed) g.logp_old_packed[p] = g.logp_old[src];
        if (f == 1 && g.adv && g.adv_packed) g.adv_packed[p] = g.adv[src];
        if (f == 2 && g.ret && g.ret_packed) g.ret_packed[p] = g.ret[src];
        if (f == 3 && g.is_weight && g.is_weight_packed) g.is_weight_packed[p] = g.is_weight[src];
    }
    // rows of timestep 0 are the pieces' first steps: fetch their initial recurrent state
    for (int r = wave; r < nrows; r += GATHER_WAVES) {
        const int j = s_j[r], src = s_src[r];
        if (s_t[r] != 0 || j >= n_seq || j >= g.seq_cap) continue;
        const bool zero = g.seq_eps[j] != 0;
        for (int l = 0; l < g.n_layers; ++l) {
            const size_t in_off = ((size_t)l * g.S + src) * g.H, out_off = ((size_t)l * g.seq_cap + j) * g.H;
            if (g.rnn_h && g.h0) copy_state_row(g.h0 + out_off, g.rnn_h + in_off, g.H, lane, zero, g.state_vec4);
            if (g.rnn_c && g.c0) copy_state_row(g.c0 + out_off, g.rnn_c + in_off, g.H, lane, zero, g.state_vec4);
        }
    }
}

inline size_t pack_ws_layout(int S, int M, void* base, PackWs* ws) {
    Carver cv(base);
    uint8_t* flags = cv.take<uint8_t>((size_t)S);
    int32_t* sf = cv.take<int32_t>((size_t)S);
    int32_t* sl = cv.take<int32_t>((size_t)S);
    uint32_t* skey = cv.take<uint32_t>((size_t)S);
    int32_t* order = cv.take<int32_t>((size_t)S);
    int32_t* sstart = cv.take<int32_t>((size_t)S + 1);
    int32_t* pf = cv.take<int32_t>((size_t)M);
    int32_t* plen = cv.take<int32_t>((size_t)M);
    uint8_t* peps = cv.take<uint8_t>((size_t)M);
    if (ws) *ws = PackWs{flags, sf, sl, skey, order, sstart, pf, plen, peps};
    return cv.used;
}

// Truncated importance weight of every step (paper section 4 "Training"; appendix hyper-parameter table:
// importance sampling on, maximum 1.0): w = min(max_is, (S/N) / L_i) for the steps of environment i.
// A workgroup writes IS_TILE consecutive steps: two wave-wide searches find the environments of its first and
// last step, the offsets in between are copied to LDS, and every thread then places its 4 consecutive steps
// there (a binary search for the first, a walk over the stretch boundaries for the rest; empty stretches are
// stepped over).  4 bytes written per step, 16 per store.
constexpr int IS_THREADS = 256;
constexpr int IS_ITEMS = 4;
constexpr int IS_TILE = 4096;
constexpr int IS_WIN = IS_TILE + 2;   // offsets kept in LDS (more only with many empty environments: then memory is searched)

// off[0 .. n_env]: offsets of the tile's environments (off[0] <= first step, off[n_env] > last step).
// wtab (may be null): the weight of environment i of the tile, when the caller has computed them once per
// environment; without it a lane divides whenever it enters a stretch (a double division is ~40 instructions, and a
// wave executes it in every unrolled position in which any of its lanes crosses a boundary).
template <typename OffPtr>
__device__ __forceinline__ void is_weight_tile(OffPtr off, const float* wtab, int n_env, int k_lo, int S, double share, float max_is,
                                               float* __restrict__ weight) {
    for (int r = 0; r < IS_TILE / (IS_THREADS * IS_ITEMS); ++r) {
        const int k0 = k_lo + (r * IS_THREADS + (int)threadIdx.x) * IS_ITEMS;
        if (k0 >= S) return;
        // The environment of the wave's first step by a 64-ary search of the whole wave (every lane probes one offset,
        // a ballot counts: one or two rounds instead of a binary search of a dozen dependent reads per lane), then
        // every lane walks on from there to its own first step (the 256 steps of a wave span a few environments).
        const int lane = threadIdx.x & (VER_WAVE - 1);
        const int k_wave = k0 - lane * IS_ITEMS;
        int lo = 0, len = n_env;   // off[lo] <= k_wave, the answer is in [lo, lo + len)
        while (len > 1) {
            const int step = (len + VER_WAVE - 1) / VER_WAVE, idx = lo + lane * step;
            const unsigned long long below = __ballot(idx < lo + len && off[idx] <= k_wave);   // a prefix of the lanes, lane 0 among them
            const int c = __popcll(below) - 1;
            len = min(step, len - c * step);
            lo += c * step;
        }
        int env = lo;
        while (off[env + 1] <= k0) ++env;   // (off[n_env] lies beyond the tile's last step)
        int end = off[env + 1];
        float w = wtab ? wtab[env] : fminf(max_is, (float)(share / (double)(end - off[env])));
        float out[IS_ITEMS];
#pragma unroll
        for (int i = 0; i < IS_ITEMS; ++i) {
            const int k = k0 + i;
            if (k < S && k >= end) {
                int begin;
                do {
                    begin = end;
                    end = off[++env + 1];
                } while (k >= end);
                w = wtab ? wtab[env] : fminf(max_is, (float)(share / (double)(end - begin)));
            }
            out[i] = w;
        }
        if (k0 + IS_ITEMS <= S) {
            *reinterpret_cast<float4*>(weight + k0) = make_float4(out[0], out[1], out[2], out[3]);
        } else {
            for (int i = 0; k0 + i < S; ++i) weight[k0 + i] = out[i];
        }
    }
}

__global__ __launch_bounds__(IS_THREADS) void is_weight_kernel(const int32_t* __restrict__ env_off, int N, int S,
                                                               double share, float max_is,
                                                               float* __restrict__ weight) {
    __shared__ int s_off[IS_WIN];
    __shared__ int s_env[2];
    const int k_lo = blockIdx.x * IS_TILE, k_hi = min(S, k_lo + IS_TILE) - 1;
    const int wave = threadIdx.x / VER_WAVE;
    if (wave < 2) {
        const int e = segment_of_wave(env_off, N, wave == 0 ? k_lo : k_hi);
        if ((threadIdx.x & (VER_WAVE - 1)) == 0) s_env[wave] = e;
    }
    __syncthreads();
    const int e0 = s_env[0], n_env = s_env[1] - e0 + 1;
    if (n_env + 1 <= IS_WIN) {
        for (int i = threadIdx.x; i <= n_env; i += IS_THREADS) s_off[i] = env_off[e0 + i];
        __syncthreads();
        is_weight_tile(static_cast<const int*>(s_off), static_cast<const float*>(nullptr), n_env, k_lo, S, share, max_is, weight);
    } else {
        is_weight_tile(env_off + e0, static_cast<const float*>(nullptr), n_env, k_lo, S, share, max_is, weight);
    }
}

// Large buffers (from IS_MARK_FROM steps on) take two launches, because the two searches above are four dependent
// rounds of loads each, and with every CU full of workgroups that wait for them the kernel runs at the pace of those
// rounds, not of its stores.  First launch: one thread per environment writes its index into the output array at the
// first step of every tile that begins inside its stretch (every tile start lies in exactly one non-empty stretch;
// a stretch that spans many tiles is handed to the whole wave).  Second launch: a tile reads its first environment
// from its own first output element (which only this tile overwrites, afterwards), loads the 256 offsets that follow
// in one round and fills in its steps; a tile with more environments than that, or whose mark is not a valid index
// (malformed offsets), searches as above.
constexpr int IS_MARK_FROM = 1 << 20;
constexpr int IS_MARK_WAVE_FROM = 8;   // tiles from which a stretch is marked by the whole wave
__global__ __launch_bounds__(256) void is_weight_mark_kernel(const int32_t* __restrict__ env_off, int N, int S,
                                                             int* __restrict__ mark) {
    const int e = blockIdx.x * 256 + threadIdx.x, lane = threadIdx.x & (VER_WAVE - 1);
    int lo = 0, hi = 0;
    if (e < N) { lo = env_off[e]; hi = min(env_off[e + 1], S); }
    lo = max(lo, 0);
    // tiles t with lo <= t * IS_TILE < hi
    int t0 = (lo + IS_TILE - 1) / IS_TILE, t1 = hi > lo ? (hi - 1) / IS_TILE : t0 - 1;   // [t0, t1]
    const bool wide = t1 - t0 + 1 >= IS_MARK_WAVE_FROM;
    if (!wide)
        for (int t = t0; t <= t1; ++t) mark[(size_t)t * IS_TILE] = e;
    unsigned long long todo = __ballot(wide);
    while (todo) {
        const int src = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        const int a = __shfl(t0, src, VER_WAVE), b = __shfl(t1, src, VER_WAVE), who = __shfl(e, src, VER_WAVE);
        for (int t = a + lane; t <= b; t += VER_WAVE) mark[(size_t)t * IS_TILE] = who;
    }
}

__global__ __launch_bounds__(IS_THREADS) void is_weight_fill_kernel(const int32_t* __restrict__ env_off, int N, int S,
                                                                    double share, float max_is,
                                                                    float* __restrict__ weight) {
    __shared__ int s_off[IS_THREADS];
    __shared__ float s_w[IS_THREADS];
    __shared__ int s_env[2];
    const int k_lo = blockIdx.x * IS_TILE, k_hi = min(S, k_lo + IS_TILE) - 1;
    const int wave = threadIdx.x / VER_WAVE;
    int e0 = reinterpret_cast<const int*>(weight)[k_lo];   // left by is_weight_mark_kernel
    // the offsets that follow, one per thread (beyond off[N] = S: that one again)
    const bool valid = e0 >= 0 && e0 < N;
    if (!valid) e0 = 0;
    const int mine = env_off[min(e0 + (int)threadIdx.x, N)];
    s_off[threadIdx.x] = mine;
    __syncthreads();   // (also: every thread has read the mark before any thread overwrites it)
    // The tile is covered when the first offset is not beyond its first step and the last one is beyond its last
    // step; its environments then end at the first offset beyond k_hi, found by counting (every wave counts for
    // itself and gets the same number).  Whatever the offsets hold, the walk then stays inside s_off[0 .. n_env].
    constexpr int last = IS_THREADS - 1;
    int n_env = 0;
    if (valid && s_off[0] <= k_lo && s_off[last] > k_hi) {
        int cnt = 0;
        for (int i = threadIdx.x & (VER_WAVE - 1); i <= last; i += VER_WAVE) cnt += s_off[i] <= k_hi ? 1 : 0;
#pragma unroll
        for (int d = VER_WAVE / 2; d > 0; d >>= 1) cnt += __shfl_xor(cnt, d, VER_WAVE);
        n_env = cnt;
    }
    if (n_env > 0 && n_env <= last && s_off[n_env] > k_hi) {
        // one division per environment of the tile (an empty one divides by zero: its weight belongs to no step)
        if ((int)threadIdx.x < n_env) s_w[threadIdx.x] = fminf(max_is, (float)(share / (double)(s_off[threadIdx.x + 1] - mine)));
        __syncthreads();
        is_weight_tile(static_cast<const int*>(s_off), static_cast<const float*>(s_w), n_env, k_lo, S, share, max_is, weight);
        return;
    }
    // not covered by 256 offsets (or no valid mark): search as the single-launch kernel does, offsets read in place
    if (wave < 2) {
        const int e = segment_of_wave(env_off, N, wave == 0 ? k_lo : k_hi);
        if ((threadIdx.x & (VER_WAVE - 1)) == 0) s_env[wave] = e;
    }
    __syncthreads();
    e0 = s_env[0];
    is_weight_tile(env_off + e0, static_cast<const float*>(nullptr), s_env[1] - e0 + 1, k_lo, S, share, max_is, weight);
}

}  // namespace
}  // namespace ver

extern "C" int ver_is_weight(const int32_t* env_off, int32_t N, int32_t S, float max_is, float* weight,
                             void* stream) {
    if (N <= 0 || S < 0 || !(max_is > 0.f)) return VER_EINVAL;
    if (S == 0) return VER_OK;
    if (!env_off || !weight || (reinterpret_cast<uintptr_t>(weight) & 15)) return VER_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int per_block = ver::IS_TILE;
    ver::ProfScope prof(VER_PROF_IS_WEIGHT, s);
    if (S >= ver::IS_MARK_FROM) {
        hipLaunchKernelGGL(ver::is_weight_mark_kernel, dim3((N + 255) / 256), dim3(256), 0, s, env_off, N, S,
                           reinterpret_cast<int*>(weight));
        hipLaunchKernelGGL(ver::is_weight_fill_kernel, dim3((S + per_block - 1) / per_block), dim3(ver::IS_THREADS), 0, s,
                           env_off, N, S, (double)S / (double)N, max_is, weight);
    } else {
        hipLaunchKernelGGL(ver::is_weight_kernel, dim3((S + per_block - 1) / per_block), dim3(ver::IS_THREADS), 0, s,
                           env_off, N, S, (double)S / (double)N, max_is, weight);
    }
    return ver::launch_status();
}

extern "C" size_t ver_pack_workspace_bytes(int32_t N, int32_t S, int32_t B) {
    if (N < 0 || S <= 0 || B <= 0) return 0;
    return ver::pack_ws_layout(S, S / B, nullptr, nullptr);
}

namespace ver {
namespace {
// Host checks of the arguments the index part reads, and the job they describe.
int pack_job_of(const ver_pack_args* a, PackJob* job) {
    if (!a) return VER_EINVAL;
    if (a->N <= 0 || a->S <= 0 || a->B <= 0 || a->b < 0 || a->b >= a->B || a->S % a->B != 0) return VER_EINVAL;
    if (!a->dones || !a->env_off || !a->seq_key || !a->info || !a->seq_first || !a->seq_len ||
        !a->seq_is_ep_start || !a->batch_sizes || !a->t_off)
        return VER_EINVAL;
    if (!a->workspace || a->workspace_bytes < ver_pack_workspace_bytes(a->N, a->S, a->B)) return VER_EWORKSPACE;
    job->seq_key = a->seq_key;
    job->b = a->b;
    pack_ws_layout(a->S, a->S / a->B, a->workspace, &job->ws);
    job->info = a->info; job->seq_first = a->seq_first; job->seq_len = a->seq_len; job->seq_eps = a->seq_is_ep_start;
    job->batch_sizes = a->batch_sizes; job->t_off = a->t_off;
    return VER_OK;
}
}  // namespace
}  // namespace ver

extern "C" int ver_pack_index_batch(const ver_pack_args* args, int32_t n, void* stream) {
    if (n < 0 || (n > 0 && !args)) return VER_EINVAL;
    if (n == 0) return VER_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // check everything before anything is launched
    for (int i = 0; i < n; ++i) {
        ver::PackJob job;
        const int st = ver::pack_job_of(&args[i], &job);
        if (st != VER_OK) return st;
        const ver_pack_args& a = args[i];
        const ver_pack_args& f = args[0];
        if (a.dones != f.dones || a.env_off != f.env_off || a.env_started_episode != f.env_started_episode || a.N != f.N ||
            a.S != f.S || a.B != f.B)
            return VER_EINVAL;   // one rollout, one minibatch count per call
        for (int k = 0; k < i; ++k)
            if (args[k].workspace == a.workspace || args[k].info == a.info) return VER_EINVAL;   // outputs must not be shared
    }
    ver::ProfScope prof(VER_PROF_PACK_INDEX, s);
    for (int i0 = 0; i0 < n; i0 += ver::PACK_MAX_JOBS) {
        const int cnt = n - i0 < ver::PACK_MAX_JOBS ? n - i0 : ver::PACK_MAX_JOBS;
        ver::PackJobs jobs = {};
        for (int i = 0; i < cnt; ++i) (void)ver::pack_job_of(&args[i0 + i], &jobs.j[i]);
        hipLaunchKernelGGL(ver::pack_index_kernel, dim3(cnt), dim3(ver::IDX_THREADS), 0, s, args[0].dones, args[0].env_off,
                           args[0].env_started_episode, args[0].N, args[0].S, args[0].B, jobs);
    }
    return ver::launch_status();
}

extern "C" int ver_pack_minibatch(const ver_pack_args* a, void* stream) {
    ver::PackJobs jobs = {};
    {
        const int st = ver::pack_job_of(a, &jobs.j[0]);
        if (st != VER_OK) return st;
    }
    if (!a->gather_idx) return VER_EINVAL;
    if (a->obs && a->obs_packed && a->D <= 0) return VER_EINVAL;
    if (a->actions && a->actions_packed && a->act_bytes <= 0) return VER_EINVAL;
    const bool states = (a->rnn_h && a->h0) || (a->rnn_c && a->c0);
    if (states && (a->n_layers <= 0 || a->H <= 0 || a->seq_cap <= 0)) return VER_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int M = a->S / a->B;
    if (!a->index_ready) {
    ver::ProfScope prof(VER_PROF_PACK_INDEX, s);
    hipLaunchKernelGGL(ver::pack_index_kernel, dim3(1), dim3(ver::IDX_THREADS), 0, s, a->dones, a->env_off,
                       a->env_started_episode, a->N, a->S, a->B, jobs);
    }
    if (hipGetLastError() != hipSuccess) return VER_EHIP;
    ver::GatherArgs g;
    g.info = a->info; g.seq_first = a->seq_first; g.seq_eps = a->seq_is_ep_start; g.t_off = a->t_off;
    g.gather_idx = a->gather_idx; g.M = M; g.S = a->S;
    g.obs = a->obs; g.D = a->D; g.obs_packed = a->obs_packed; g.obs_bf16 = a->obs_packed_bf16;
    g.actions = static_cast<const uint8_t*>(a->actions); g.act_bytes = a->act_bytes;
    g.actions_packed = static_cast<uint8_t*>(a->actions_packed);
    g.logp_old = a->logp_old; g.adv = a->adv; g.ret = a->ret;
    g.logp_old_packed = a->logp_old_packed; g.adv_packed = a->adv_packed; g.ret_packed = a->ret_packed;
    g.is_weight = a->is_weight; g.is_weight_packed = a->is_weight_packed;
    g.rnn_h = a->rnn_h; g.rnn_c = a->rnn_c; g.n_layers = states ? a->n_layers : 0; g.H = a->H;
    g.seq_cap = a->seq_cap; g.h0 = a->h0; g.c0 = a->c0;
    g.state_vec4 = a->H % 4 == 0 && ((reinterpret_cast<uintptr_t>(a->rnn_h) | reinterpret_cast<uintptr_t>(a->rnn_c) |
                                      reinterpret_cast<uintptr_t>(a->h0) | reinterpret_cast<uintptr_t>(a->c0)) & 15) == 0;
    ver::ProfScope prof(VER_PROF_PACK_GATHER, s);
    if (M >= ver::GATHER_BIG_FROM)
        hipLaunchKernelGGL(ver::pack_gather_kernel<ver::GATHER_ROWS_BIG>, dim3((M + ver::GATHER_ROWS_BIG - 1) / ver::GATHER_ROWS_BIG),
                           dim3(ver::GATHER_THREADS), 0, s, g);
    else
        hipLaunchKernelGGL(ver::pack_gather_kernel<ver::GATHER_ROWS_SMALL>, dim3((M + ver::GATHER_ROWS_SMALL - 1) / ver::GATHER_ROWS_SMALL),
                           dim3(ver::GATHER_THREADS), 0, s, g);
    return ver::launch_status();
}
