// ver_ingest: from the linear collection buffer (steps in arrival order, each
// tagged with its environment) to the environment-major ragged buffer the
// learning phase works on.
//
// Paper: section 2.2 "Batching computation for learning" (experience is written
// into a linear buffer in GPU memory during collection) and section 2.1
// (inference workers store steps as they arrive, so environments interleave and
// each contributes a different number of steps).
//
// Bucketing by environment with arrival order kept inside a bucket is a STABLE
// sort of the slots by environment id.  It is done as a least-significant-digit
// radix sort with digits of up to 10 bits (one pass up to 511 environments, two
// up to about a million): per pass a histogram per tile of 2048 slots, one
// exclusive scan over (digit, tile), and a scatter in which every wave ranks
// its own contiguous run of slots with wave ballots (the lanes that hold the
// same digit find each other in `bits` ballots; the lowest of them advances the
// wave's running count in LDS), so the order of equal digits is the arrival
// order by construction: no atomics decide a position, the result is
// bit-reproducible.  The offsets env_off come from the sorted ids: the thread
// at a boundary writes the offsets of every environment that starts there
// (empty ones included).  Ids outside [0, N) are filed in an extra bucket N
// behind all environments and counted, so bad input cannot write out of bounds.
//
// Traffic per pass: ids and slots read twice and written once (20 B/slot); the
// gather of a per-step field into the new order reads and writes it once.
// Buffers of 2^20 slots and more use larger tiles that leave through LDS in
// sorted order and carry the step counters along (+8 B/slot and pass), which
// keeps the stores contiguous and spares the last kernel a random gather.
#include "common.h"

namespace ver {
namespace {

constexpr int ING_THREADS = 256;
constexpr int ING_WAVES = ING_THREADS / VER_WAVE;
constexpr int ING_ITEMS = 8;                          // slots per lane
constexpr int ING_WAVE_RUN = ING_ITEMS * VER_WAVE;    // contiguous slots ranked by one wave
constexpr int ING_TILE = ING_THREADS * ING_ITEMS;     // slots per workgroup
constexpr int ING_MAX_BITS = 10;
constexpr int ING_MAX_BINS = 1 << ING_MAX_BITS;
constexpr int ING_SCAN_THREADS = 1024;
constexpr int ING_MAX_S = 1 << 24;   // slots per call
constexpr int ING_SCAN_CHUNK = 4096;            // counters per workgroup of the two-level scan
constexpr int ING_SCAN_DIRECT = 4 * ING_SCAN_CHUNK;   // up to here one workgroup scans all counters by itself

// Sort key of arrival slot a in the first pass: the environment id, or N for an id outside [0, N).
__device__ __forceinline__ int key_of_env(int e, int N) { return (unsigned)e < (unsigned)N ? e : N; }

__device__ __forceinline__ int load_key(const int32_t* __restrict__ keys, int a, int N, bool first) {
    const int k = keys[a];
    return first ? key_of_env(k, N) : k;
}

// hist[d * tiles + tile] = number of slots of the tile whose digit is d.
template <int ITEMS>
__global__ __launch_bounds__(ING_THREADS) void ingest_hist_kernel(const int32_t* __restrict__ keys, int S, int N, int first,
                                                                  int shift, int bits, int tiles, int32_t* __restrict__ hist) {
    __shared__ int cnt[ING_MAX_BINS];
    const int bins = 1 << bits, tile = blockIdx.x;
    for (int d = threadIdx.x; d < bins; d += ING_THREADS) cnt[d] = 0;
    __syncthreads();
    const int base = tile * (ING_THREADS * ITEMS);
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int a = base + it * ING_THREADS + threadIdx.x;
        if (a < S) atomicAdd(&cnt[(load_key(keys, a, N, first) >> shift) & (bins - 1)], 1);
    }
    __syncthreads();
    for (int d = threadIdx.x; d < bins; d += ING_THREADS) hist[(size_t)d * tiles + tile] = cnt[d];
}

// In-place exclusive prefix sum over n counters, one workgroup.
__global__ __launch_bounds__(ING_SCAN_THREADS) void ingest_scan_kernel(int32_t* __restrict__ hist, int n) {
    __shared__ int part[ING_SCAN_THREADS];
    const int per = (n + ING_SCAN_THREADS - 1) / ING_SCAN_THREADS;
    const int lo = min(n, (int)threadIdx.x * per), hi = min(n, lo + per);
    int s = 0;
    for (int i = lo; i < hi; ++i) s += hist[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int d = 1; d < ING_SCAN_THREADS; d <<= 1) {   // inclusive scan of the per-thread sums
        const int v = (int)threadIdx.x >= d ? part[threadIdx.x - d] : 0;
        __syncthreads();
        part[threadIdx.x] += v;
        __syncthreads();
    }
    int run = part[threadIdx.x] - s;
    for (int i = lo; i < hi; ++i) {
        const int c = hist[i];
        hist[i] = run;
        run += c;
    }
}

// Two-level scan for many counters: every workgroup scans its own chunk of ING_SCAN_CHUNK counters in place
// (exclusive) and leaves the chunk's total in sums[chunk]; ingest_scan_kernel then scans the totals, and the
// scatter adds sums[i / ING_SCAN_CHUNK] to counter i when it reads it.
__global__ __launch_bounds__(ING_THREADS) void ingest_scan_chunks_kernel(int32_t* __restrict__ hist, int n,
                                                                         int32_t* __restrict__ sums) {
    constexpr int PER = ING_SCAN_CHUNK / ING_THREADS;
    __shared__ int wsum[ING_WAVES];
    const int lane = threadIdx.x & (VER_WAVE - 1), wave = threadIdx.x / VER_WAVE;
    const int lo = blockIdx.x * ING_SCAN_CHUNK + threadIdx.x * PER;
    int c[PER], s = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        c[i] = lo + i < n ? hist[lo + i] : 0;
        s += c[i];
    }
    int incl = s;
#pragma unroll
    for (int d = 1; d < VER_WAVE; d <<= 1) {
        const int up = __shfl_up(incl, d, VER_WAVE);
        if (lane >= d) incl += up;
    }
    if (lane == VER_WAVE - 1) wsum[wave] = incl;
    __syncthreads();
    int run = incl - s;
    for (int w = 0; w < wave; ++w) run += wsum[w];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        if (lo + i < n) hist[lo + i] = run;
        run += c[i];
    }
    if (threadIdx.x == ING_THREADS - 1) sums[blockIdx.x] = run;
}

// Stable scatter of one tile.  Wave w ranks the contiguous slots [tile*TILE + w*WAVE_RUN, +WAVE_RUN) in rounds of
// 64; wcnt[w][d] is the number of slots with digit d the wave has seen so far.
__global__ __launch_bounds__(ING_THREADS) void ingest_scatter_kernel(
    const int32_t* __restrict__ keys, const int32_t* __restrict__ vals, int S, int N, int first, int shift, int bits, int tiles,
    const int32_t* __restrict__ gbase, const int32_t* __restrict__ sums, int32_t* __restrict__ keys_out,
    int32_t* __restrict__ vals_out) {
    __shared__ int wcnt[ING_WAVES][ING_MAX_BINS];
    const int bins = 1 << bits, tile = blockIdx.x;
    const int lane = threadIdx.x & (VER_WAVE - 1), wave = threadIdx.x / VER_WAVE;
    for (int d = threadIdx.x; d < ING_WAVES * bins; d += ING_THREADS) wcnt[d / bins][d % bins] = 0;
    __syncthreads();
    volatile int* mine = wcnt[wave];
    const int run0 = tile * ING_TILE + wave * ING_WAVE_RUN;
    const unsigned long long lanes_below = (1ull << lane) - 1ull;
    int key[ING_ITEMS], val[ING_ITEMS], rank[ING_ITEMS];
#pragma unroll
    for (int it = 0; it < ING_ITEMS; ++it) {
        const int a = run0 + it * VER_WAVE + lane;
        const bool live = a < S;
        key[it] = live ? load_key(keys, a, N, first) : 0;
        val[it] = live ? (first ? a : vals[a]) : 0;
        const int d = (key[it] >> shift) & (bins - 1);
        // lanes of this round that hold the same digit
        unsigned long long peers = __ballot(live);
        for (int b = 0; b < bits; ++b) {
            const bool bit = (d >> b) & 1;
            const unsigned long long with = __ballot(live && bit);
            peers &= bit ? with : ~with;
        }
        int seen = 0;
        if (live) seen = mine[d];
        rank[it] = seen + __popcll(peers & lanes_below);
        if (live && (peers & lanes_below) == 0ull) mine[d] = seen + __popcll(peers);   // lowest peer advances the count
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    // wcnt[w][d] <- first output position of the wave's slots with digit d
    for (int d = threadIdx.x; d < bins; d += ING_THREADS) {
        const size_t at = (size_t)d * tiles + tile;
        int pos = gbase[at] + (sums ? sums[at / ING_SCAN_CHUNK] : 0);
        for (int w = 0; w < ING_WAVES; ++w) {
            const int c = wcnt[w][d];
            wcnt[w][d] = pos;
            pos += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < ING_ITEMS; ++it) {
        const int a = run0 + it * VER_WAVE + lane;
        if (a < S) {
            const int pos = wcnt[wave][(key[it] >> shift) & (bins - 1)] + rank[it];
            keys_out[pos] = key[it];
            vals_out[pos] = val[it];
        }
    }
}

// The same scatter for large buffers: tiles of ING_BIG_ITEMS slots per lane, and the tile leaves through LDS in
// sorted order.  Written straight from the lanes that ranked them, the slots of one digit go out as single
// 4-byte stores from different lanes at different times: one L2 request each and partly filled sectors towards
// memory (measured: 5.5 times the algorithmic traffic).  Here every slot is first put at its place inside the
// sorted tile in LDS; consecutive threads then write consecutive sorted slots, so a digit's slots of this tile
// (a run of S / (tiles * bins) on average) leave as contiguous stores.
constexpr int ING_BIG_ITEMS = 16;
constexpr int ING_BIG_TILE = ING_THREADS * ING_BIG_ITEMS;
constexpr int ING_BIG_FROM = 1 << 20;   // slots from which the large-buffer kernels are used

__global__ __launch_bounds__(ING_THREADS) void ingest_scatter_sorted_kernel(
    const int32_t* __restrict__ keys, const int32_t* __restrict__ vals, int S, int N, int first, int shift, int bits, int tiles,
    const int32_t* __restrict__ gbase, const int32_t* __restrict__ sums, int32_t* __restrict__ keys_out,
    int32_t* __restrict__ vals_out, const int32_t* __restrict__ t_in, int32_t* __restrict__ t_out) {
    extern __shared__ int ing_smem[];
    const int bins = 1 << bits, tile = blockIdx.x;
    int* wcnt = ing_smem;                       // [ING_WAVES][bins] slots of digit d seen by wave w, later: before wave w
    int* lstart = wcnt + ING_WAVES * bins;      // [bins] first place of digit d inside the sorted tile
    int* gpos = lstart + bins;                  // [bins] output position of the tile's sorted slot j with digit d, minus j
    int* s_key = gpos + bins;                   // [ING_BIG_TILE] the tile in sorted order
    int* s_val = s_key + ING_BIG_TILE;
    __shared__ int s_wsum[ING_WAVES];
    const int lane = threadIdx.x & (VER_WAVE - 1), wave = threadIdx.x / VER_WAVE;
    for (int d = threadIdx.x; d < ING_WAVES * bins; d += ING_THREADS) wcnt[d] = 0;
    __syncthreads();
    volatile int* mine = wcnt + wave * bins;
    const int run0 = tile * ING_BIG_TILE + wave * (ING_BIG_ITEMS * VER_WAVE);
    const unsigned long long lanes_below = (1ull << lane) - 1ull;
    int key[ING_BIG_ITEMS], val[ING_BIG_ITEMS], rank[ING_BIG_ITEMS];
#pragma unroll
    for (int it = 0; it < ING_BIG_ITEMS; ++it) {
        const int a = run0 + it * VER_WAVE + lane;
        const bool live = a < S;
        key[it] = live ? load_key(keys, a, N, first) : 0;
        val[it] = live ? (first ? a : vals[a]) : 0;
        const int d = (key[it] >> shift) & (bins - 1);
        unsigned long long peers = __ballot(live);
        for (int b = 0; b < bits; ++b) {
            const bool bit = (d >> b) & 1;
            const unsigned long long with = __ballot(live && bit);
            peers &= bit ? with : ~with;
        }
        int seen = 0;
        if (live) seen = mine[d];
        rank[it] = seen + __popcll(peers & lanes_below);
        if (live && (peers & lanes_below) == 0ull) mine[d] = seen + __popcll(peers);   // lowest peer advances the count
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    // per digit: slots in the tile, and how many of them the waves before each wave hold
    for (int d = threadIdx.x; d < bins; d += ING_THREADS) {
        int before = 0;
        for (int w = 0; w < ING_WAVES; ++w) {
            const int c = wcnt[w * bins + d];
            wcnt[w * bins + d] = before;
            before += c;
        }
        lstart[d] = before;
    }
    __syncthreads();
    // exclusive prefix sum of lstart over the digits (bins <= 4 per thread)
    {
        const int per = (bins + ING_THREADS - 1) / ING_THREADS;
        const int lo = min(bins, (int)threadIdx.x * per), hi = min(bins, lo + per);
        int sum = 0;
        for (int d = lo; d < hi; ++d) sum += lstart[d];
        int incl = sum;
#pragma unroll
        for (int dd = 1; dd < VER_WAVE; dd <<= 1) {
            const int up = __shfl_up(incl, dd, VER_WAVE);
            if (lane >= dd) incl += up;
        }
        if (lane == VER_WAVE - 1) s_wsum[wave] = incl;
        __syncthreads();
        int run = incl - sum;
        for (int w = 0; w < wave; ++w) run += s_wsum[w];
        for (int d = lo; d < hi; ++d) {
            const int c = lstart[d];
            lstart[d] = run;
            const size_t at = (size_t)d * tiles + tile;
            gpos[d] = gbase[at] + (sums ? sums[at / ING_SCAN_CHUNK] : 0) - run;
            run += c;
        }
    }
    __syncthreads();
    // the step counters travel with the slots (t_in: in arrival order in the first pass, else as the pass before
    // left them), so that the last kernel finds them next to each other instead of gathering them at random
    int cnt_t[ING_BIG_ITEMS];
    if (t_in) {
#pragma unroll
        for (int it = 0; it < ING_BIG_ITEMS; ++it) {
            const int a = run0 + it * VER_WAVE + lane;
            cnt_t[it] = a < S ? t_in[a] : 0;
        }
    }
#pragma unroll
    for (int it = 0; it < ING_BIG_ITEMS; ++it) {
        const int a = run0 + it * VER_WAVE + lane;
        if (a < S) {
            const int d = (key[it] >> shift) & (bins - 1);
            const int at = lstart[d] + wcnt[wave * bins + d] + rank[it];
            rank[it] = at;   // place inside the sorted tile
            s_key[at] = key[it];
            s_val[at] = val[it];
        }
    }
    __syncthreads();
    const int n_tile = min(ING_BIG_TILE, S - tile * ING_BIG_TILE);
    for (int j = threadIdx.x; j < n_tile; j += ING_THREADS) {
        const int k = s_key[j];
        const int pos = gpos[(k >> shift) & (bins - 1)] + j;
        keys_out[pos] = k;
        vals_out[pos] = s_val[j];
        s_val[j] = pos;   // kept for the counters
    }
    if (t_in) {
        __syncthreads();
#pragma unroll
        for (int it = 0; it < ING_BIG_ITEMS; ++it)
            if (run0 + it * VER_WAVE + lane < S) s_key[rank[it]] = cnt_t[it];
        __syncthreads();
        for (int j = threadIdx.x; j < n_tile; j += ING_THREADS) t_out[s_val[j]] = s_key[j];
    }
}

// Offsets from the sorted keys, count of ids outside [0, N), check of the per-environment step counters.
__global__ __launch_bounds__(ING_THREADS) void ingest_finish_kernel(const int32_t* __restrict__ keys,
                                                                    const int32_t* __restrict__ order,
                                                                    const int32_t* __restrict__ arr_t,
                                                                    const int32_t* __restrict__ t_sorted, int S, int N,
                                                                    int32_t* __restrict__ env_off, int32_t* __restrict__ info) {
    const int k = blockIdx.x * ING_THREADS + threadIdx.x;
    // the step counter of flat step k (from the sorted copy the large-buffer passes leave, else gathered: a random
    // access), handed to the next lane
    const int lane = threadIdx.x & (VER_WAVE - 1);
    int t_here = 0;
    if (arr_t && k < S) t_here = t_sorted ? t_sorted[k] : arr_t[order[k]];
    int t_prev = __shfl_up(t_here, 1, VER_WAVE);
    if (k >= S) return;
    if (arr_t && lane == 0 && k > 0) t_prev = t_sorted ? t_sorted[k - 1] : arr_t[order[k - 1]];
    const int key = keys[k], prev = k > 0 ? keys[k - 1] : -1;
    // k is the first flat step whose key is >= e for every e in (prev, key]
    for (int e = prev + 1; e <= key; ++e) env_off[e] = k;
    if (k == S - 1)
        for (int e = key + 1; e <= N; ++e) env_off[e] = S;
    if (key == N && prev != N) info[1] = S - k;            // slots with an id outside [0, N)
    if (arr_t && key == prev && key < N && t_here != t_prev + 1) atomicAdd(&info[0], 1);
}

__global__ __launch_bounds__(ING_THREADS) void ingest_dense_kernel(int T, int N, int32_t* __restrict__ env_off,
                                                                   int32_t* __restrict__ order) {
    const long long k = (long long)blockIdx.x * ING_THREADS + threadIdx.x;
    if (k <= N) env_off[k] = (int)(k * T);
    if (k < (long long)T * N) {
        const int i = (int)(k / T), t = (int)(k % T);
        order[k] = t * N + i;
    }
}

// dst row k = src row order[k]; rows of `units` elements of type U.
template <typename U>
__global__ __launch_bounds__(ING_THREADS) void ingest_gather_kernel(const int32_t* __restrict__ order, long long total,
                                                                    int units, const U* __restrict__ src, U* __restrict__ dst) {
    const long long stride = (long long)gridDim.x * ING_THREADS;
    for (long long i = (long long)blockIdx.x * ING_THREADS + threadIdx.x; i < total; i += stride) {
        const long long k = i / units;
        const int c = (int)(i - k * units);
        dst[i] = src[(long long)order[k] * units + c];
    }
}

// Several fields in one launch: a field takes the blocks [block_first[f], block_first[f + 1]) and moves its rows in
// units of 16, 4 or 1 bytes (what its addresses and row size allow), exactly as a launch of its own would.
struct GatherBatch {
    const void* src[VER_INGEST_MAX_FIELDS];
    void* dst[VER_INGEST_MAX_FIELDS];
    int units[VER_INGEST_MAX_FIELDS];     // units per row
    int unit[VER_INGEST_MAX_FIELDS];      // bytes per unit
    int block_first[VER_INGEST_MAX_FIELDS + 1];
    int n;
};
template <typename U>
__device__ __forceinline__ void gather_field(const int32_t* __restrict__ order, long long total, int units, const void* src, void* dst,
                                             int block, int blocks) {
    const U* __restrict__ s = static_cast<const U*>(src);
    U* __restrict__ d = static_cast<U*>(dst);
    const long long stride = (long long)blocks * ING_THREADS;
    for (long long i = (long long)block * ING_THREADS + threadIdx.x; i < total; i += stride) {
        const long long k = i / units;
        const int c = (int)(i - k * units);
        d[i] = s[(long long)order[k] * units + c];
    }
}
__global__ __launch_bounds__(ING_THREADS) void ingest_gather_batch_kernel(const int32_t* __restrict__ order, int S, GatherBatch g) {
    int f = 0;
#pragma unroll
    for (int i = 1; i < VER_INGEST_MAX_FIELDS; ++i)
        if (i < g.n && (int)blockIdx.x >= g.block_first[i]) f = i;
    // (uniform selects: constant indices only, so that the arguments are read in place)
    const void* src = g.src[0]; void* dst = g.dst[0];
    int units = g.units[0], unit = g.unit[0], b0 = g.block_first[0], b1 = g.block_first[1];
#pragma unroll
    for (int i = 1; i < VER_INGEST_MAX_FIELDS; ++i)
        if (f == i) { src = g.src[i]; dst = g.dst[i]; units = g.units[i]; unit = g.unit[i]; b0 = g.block_first[i]; b1 = g.block_first[i + 1]; }
    const long long total = (long long)S * units;
    if (unit == 16) gather_field<int4>(order, total, units, src, dst, blockIdx.x - b0, b1 - b0);
    else if (unit == 4) gather_field<int32_t>(order, total, units, src, dst, blockIdx.x - b0, b1 - b0);
    else gather_field<uint8_t>(order, total, units, src, dst, blockIdx.x - b0, b1 - b0);
}

inline int bits_for(int n) {   // bits needed to write the value n
    int b = 1;
    while ((n >> b) != 0) ++b;
    return b;
}

struct IngestPlan {
    int tiles, passes, bits[4];
    bool big;   // large-buffer kernels (tiles of ING_BIG_TILE slots)
    size_t hist_words, sum_words;
};

inline IngestPlan ingest_plan(int N, int S) {
    IngestPlan p;
    p.big = S >= ING_BIG_FROM;
    const int tile = p.big ? ING_BIG_TILE : ING_TILE;
    p.tiles = (S + tile - 1) / tile;
    const int total = bits_for(N);                       // keys run from 0 to N (N = the bucket of bad ids)
    p.passes = (total + ING_MAX_BITS - 1) / ING_MAX_BITS;
    int left = total;
    for (int i = 0; i < p.passes; ++i) {
        p.bits[i] = (left + (p.passes - i) - 1) / (p.passes - i);
        left -= p.bits[i];
    }
    p.hist_words = (size_t)ING_MAX_BINS * (size_t)(p.tiles > 0 ? p.tiles : 1);
    p.sum_words = p.hist_words / ING_SCAN_CHUNK + 1;
    return p;
}

}  // namespace
}  // namespace ver

extern "C" size_t ver_ingest_workspace_bytes(int32_t N, int32_t S) {
    if (N <= 0 || S < 0 || S > ver::ING_MAX_S) return 0;
    const ver::IngestPlan p = ver::ingest_plan(N, S);
    const size_t per = ver::align_up((size_t)(S > 0 ? S : 1) * 4, 256);
    return (p.big ? 5 : 3) * per + ver::align_up(p.hist_words * 4, 256) + ver::align_up(p.sum_words * 4, 256);
}

extern "C" int ver_ingest(const int32_t* arr_env, const int32_t* arr_t, int32_t N, int32_t S, int32_t* env_off,
                          int32_t* order, int32_t* info, void* workspace, size_t workspace_bytes, void* stream) {
    using namespace ver;
    if (N <= 0 || S < 0 || !env_off || !info) return VER_EINVAL;
    if (S > ING_MAX_S) return VER_EUNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ProfScope prof(VER_PROF_INGEST, s);
    fill_words(info, 4, 0, s);
    if (S == 0) {
        fill_words(env_off, (size_t)N + 1, 0, s);
        return launch_status();
    }
    if (!arr_env || !order) return VER_EINVAL;
    if (!workspace || workspace_bytes < ver_ingest_workspace_bytes(N, S)) return VER_EWORKSPACE;
    const IngestPlan p = ingest_plan(N, S);
    Carver cv(workspace);
    int32_t* key_buf[2] = {cv.take<int32_t>(S), cv.take<int32_t>(S)};
    int32_t* val_tmp = cv.take<int32_t>(S);
    int32_t* hist = cv.take<int32_t>(p.hist_words);
    int32_t* sums = cv.take<int32_t>(p.sum_words);
    int32_t* t_buf[2] = {nullptr, nullptr};
    if (p.big && arr_t) { t_buf[0] = cv.take<int32_t>(S); t_buf[1] = cv.take<int32_t>(S); }
    const int32_t* t_in = arr_t;
    // slots ping-pong between `order` and val_tmp so that the last pass writes `order`
    const int32_t* keys_in = arr_env;
    const int32_t* vals_in = nullptr;
    int shift = 0;
    for (int pass = 0; pass < p.passes; ++pass) {
        const int first = pass == 0, bits = p.bits[pass];
        int32_t* keys_out = key_buf[pass & 1];
        int32_t* vals_out = ((p.passes - 1 - pass) & 1) ? val_tmp : order;
        if (p.big)
            hipLaunchKernelGGL(ingest_hist_kernel<ING_BIG_ITEMS>, dim3(p.tiles), dim3(ING_THREADS), 0, s, keys_in, S, N, first,
                               shift, bits, p.tiles, hist);
        else
            hipLaunchKernelGGL(ingest_hist_kernel<ING_ITEMS>, dim3(p.tiles), dim3(ING_THREADS), 0, s, keys_in, S, N, first,
                               shift, bits, p.tiles, hist);
        const int counters = (1 << bits) * p.tiles;
        const bool two_level = counters > ING_SCAN_DIRECT;
        if (two_level) {
            const int chunks = (counters + ING_SCAN_CHUNK - 1) / ING_SCAN_CHUNK;
            hipLaunchKernelGGL(ingest_scan_chunks_kernel, dim3(chunks), dim3(ING_THREADS), 0, s, hist, counters, sums);
            hipLaunchKernelGGL(ingest_scan_kernel, dim3(1), dim3(ING_SCAN_THREADS), 0, s, sums, chunks);
        } else {
            hipLaunchKernelGGL(ingest_scan_kernel, dim3(1), dim3(ING_SCAN_THREADS), 0, s, hist, counters);
        }
        const int32_t* sums_in = two_level ? sums : (const int32_t*)nullptr;
        if (p.big) {
            const size_t lds = ((size_t)(ING_WAVES + 2) * (1 << bits) + 2 * ING_BIG_TILE) * sizeof(int);   // <= 56 KB
            hipLaunchKernelGGL(ingest_scatter_sorted_kernel, dim3(p.tiles), dim3(ING_THREADS), lds, s, keys_in, vals_in, S, N,
                               first, shift, bits, p.tiles, hist, sums_in, keys_out, vals_out, arr_t ? t_in : nullptr,
                               t_buf[pass & 1]);
            t_in = t_buf[pass & 1];
        } else {
            hipLaunchKernelGGL(ingest_scatter_kernel, dim3(p.tiles), dim3(ING_THREADS), 0, s, keys_in, vals_in, S, N, first,
                               shift, bits, p.tiles, hist, sums_in, keys_out, vals_out);
        }
        keys_in = keys_out;
        vals_in = vals_out;
        shift += bits;
    }
    hipLaunchKernelGGL(ingest_finish_kernel, dim3((S + ING_THREADS - 1) / ING_THREADS), dim3(ING_THREADS), 0, s, keys_in,
                       order, arr_t, (p.big && arr_t) ? t_in : (const int32_t*)nullptr, S, N, env_off, info);
    return launch_status();
}

extern "C" int ver_ingest_dense(int32_t T, int32_t N, int32_t* env_off, int32_t* order, void* stream) {
    using namespace ver;
    if (N <= 0 || T < 0 || !env_off || (long long)T * N > ING_MAX_S) return VER_EINVAL;
    if (T > 0 && !order) return VER_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const long long n = (long long)T * N > N + 1 ? (long long)T * N : N + 1;
    ProfScope prof(VER_PROF_INGEST, s);
    hipLaunchKernelGGL(ingest_dense_kernel, dim3((unsigned)((n + ING_THREADS - 1) / ING_THREADS)), dim3(ING_THREADS), 0, s,
                       T, N, env_off, order);
    return launch_status();
}

extern "C" int ver_ingest_gather(const int32_t* order, int32_t S, const void* src, int32_t row_bytes, void* dst,
                                 void* stream) {
    using namespace ver;
    if (S < 0 || row_bytes <= 0) return VER_EINVAL;
    if (S == 0) return VER_OK;
    if (!order || !src || !dst || src == dst) return VER_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uintptr_t both = reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst) | (uintptr_t)row_bytes;
    const int unit = (both & 15) == 0 ? 16 : (both & 3) == 0 ? 4 : 1;
    const int units = row_bytes / unit;
    const long long total = (long long)S * units;
    long long blocks = (total + ING_THREADS - 1) / ING_THREADS;
    if (blocks > 65536) blocks = 65536;
    ProfScope prof(VER_PROF_INGEST, s);
    if (unit == 16)
        hipLaunchKernelGGL(ingest_gather_kernel<int4>, dim3((unsigned)blocks), dim3(ING_THREADS), 0, s, order, total, units,
                           static_cast<const int4*>(src), static_cast<int4*>(dst));
    else if (unit == 4)
        hipLaunchKernelGGL(ingest_gather_kernel<int32_t>, dim3((unsigned)blocks), dim3(ING_THREADS), 0, s, order, total,
                           units, static_cast<const int32_t*>(src), static_cast<int32_t*>(dst));
    else
        hipLaunchKernelGGL(ingest_gather_kernel<uint8_t>, dim3((unsigned)blocks), dim3(ING_THREADS), 0, s, order, total,
                           units, static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst));
    return launch_status();
}

extern "C" int ver_ingest_gather_batch(const int32_t* order, int32_t S, int32_t n_fields, const void* const* src,
                                       const int32_t* row_bytes, void* const* dst, void* stream) {
    using namespace ver;
    if (S < 0 || n_fields < 0 || n_fields > VER_INGEST_MAX_FIELDS) return VER_EINVAL;
    if (S == 0 || n_fields == 0) return VER_OK;
    if (!order || !src || !row_bytes || !dst) return VER_EINVAL;
    GatherBatch g{};
    g.n = n_fields;
    int blocks = 0;
    for (int f = 0; f < n_fields; ++f) {
        if (!src[f] || !dst[f] || src[f] == dst[f] || row_bytes[f] <= 0) return VER_EINVAL;
        const uintptr_t both = reinterpret_cast<uintptr_t>(src[f]) | reinterpret_cast<uintptr_t>(dst[f]) | (uintptr_t)row_bytes[f];
        const int unit = (both & 15) == 0 ? 16 : (both & 3) == 0 ? 4 : 1;
        g.src[f] = src[f]; g.dst[f] = dst[f]; g.unit[f] = unit; g.units[f] = row_bytes[f] / unit;
        const long long total = (long long)S * g.units[f];
        long long b = (total + ING_THREADS - 1) / ING_THREADS;
        if (b > 65536) b = 65536;
        g.block_first[f] = blocks;
        blocks += (int)b;
    }
    g.block_first[n_fields] = blocks;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ProfScope prof(VER_PROF_INGEST, s);
    hipLaunchKernelGGL(ingest_gather_batch_kernel, dim3((unsigned)blocks), dim3(ING_THREADS), 0, s, order, S, g);
    return launch_status();
}
