// ver_lstm_fwd / ver_lstm_bwd: multi-layer LSTM actor-critic over a packed
// minibatch and back-propagation through time.
//
// Paper: section 4 "Architecture" (embedding + state vector -> 2-layer LSTM ->
// action distribution and value), sequences for BPTT from section 2.2.
//
// Per layer the work splits into what has no time dependence and what has:
//   time-batched (one MFMA GEMM over all M rows):  W_ih x_t + b  (forward),
//       dx = W_ih^T dz, dW_ih = dz^T x, dW_hh = dz^T h_{t-1}     (backward)
//   sequential (persistent kernels, W_hh resident in registers): h_{t-1} W_hh^T + gates
//       (forward), dz_t and W_hh dz_t (backward) - see lstm_rec.h.
// Internally the 4H gate rows are interleaved (row = unit*4 + gate); user-facing
// weights and gradients keep the gate-major order i,f,g,o of the declaration.
#include <cstring>
#include <mutex>

#include "lstm_pipe.h"

namespace ver {
namespace {

// ---------------------------------------------------------------- weight preparation
// dst[q][d] = W[(q%4)*H + q/4][d] and dstT[d][q]; q = unit*4 + gate.  A block moves a 64 x 64 tile through LDS so
// that the reads of W and both writes are contiguous along their fastest index.
// Four converted elements as one store (8 bytes bf16, 16 bytes fp32).
__device__ __forceinline__ void st4(float* p, float a, float b, float c, float d) { *reinterpret_cast<f32x4_t*>(p) = f32x4_t{a, b, c, d}; }
__device__ __forceinline__ void st4(bf16_t* p, float a, float b, float c, float d) {
    u16x4_t v;
    v.x = to_bf16(a); v.y = to_bf16(b); v.z = to_bf16(c); v.w = to_bf16(d);
    *reinterpret_cast<u16x4_t*>(p) = v;
}
// A thread moves 4 adjacent elements at a time (16-byte loads, 8- or 16-byte stores; cols is a multiple of 4):
// 16 lanes cover a tile row in either direction.
// All matrices and bias vectors of a call in one launch (blockIdx.z: the job; a launch per matrix took ~10 us each,
// most of it ramp and tail).
constexpr int PREP_MAX_JOBS = 24;   // 2 matrices + 1 bias per layer, 8 layers
struct PrepJob {
    const float* W;      // matrix [4H, cols] gate-major, or b_ih when cols == 0
    const float* b_hh;   // (bias jobs)
    void* dst; void* dstT;
    int cols;            // 0: bias job
};
struct PrepArgs { PrepJob job[PREP_MAX_JOBS]; };
template <typename E>
__global__ __launch_bounds__(256) void prep_weights_kernel(PrepArgs a, int H) {
    __shared__ float tile[64][65];
    const PrepJob& jb = a.job[blockIdx.z];   // (uniform index into the kernel arguments: scalar loads)
    const int cols = jb.cols;
    if (cols == 0) {   // bias: dst[q] = b_ih + b_hh, gate rows interleaved
        const int q = (blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x;
        if (q < 4 * H) {
            const int src = (q & 3) * H + (q >> 2);
            static_cast<float*>(jb.dst)[q] = jb.W[src] + jb.b_hh[src];
        }
        return;
    }
    const int q0 = blockIdx.y * 64, d0 = blockIdx.x * 64;
    if (d0 >= cols) return;
    const float* __restrict__ W = jb.W;
    E* __restrict__ dst = static_cast<E*>(jb.dst);
    E* __restrict__ dstT = static_cast<E*>(jb.dstT);
    const int c4 = (threadIdx.x & 15) * 4, r0 = threadIdx.x >> 4;
#pragma unroll
    for (int r = r0; r < 64; r += 16) {
        const int q = q0 + r, d = d0 + c4;   // 4H is a multiple of 64: q is always a valid row
        f32x4_t v = {0.f, 0.f, 0.f, 0.f};
        if (d < cols) {
            v = *reinterpret_cast<const f32x4_t*>(W + ((size_t)(q & 3) * H + (q >> 2)) * cols + d);
            st4(dst + (size_t)q * cols + d, v[0], v[1], v[2], v[3]);
        }
        tile[r][c4] = v[0]; tile[r][c4 + 1] = v[1]; tile[r][c4 + 2] = v[2]; tile[r][c4 + 3] = v[3];
    }
    __syncthreads();
#pragma unroll
    for (int r = r0; r < 64; r += 16) {
        const int d = d0 + r, q = q0 + c4;
        if (d < cols) st4(dstT + (size_t)d * 4 * H + q, tile[c4][r], tile[c4 + 1][r], tile[c4 + 2][r], tile[c4 + 3][r]);
    }
}

// ---------------------------------------------------------------- heads
__device__ __forceinline__ float wave_sum_all(float v) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, VER_WAVE);
    return v;
}

// head_out[p][a] = W_a[a] . h[p] + b_a[a];  value[p] = w_v . h[p] + b_v: a skinny fp32 GEMM (at most 64 columns)
// bound by reading h once.  One workgroup per 16 rows, fp32 MFMA 16x16x4 with the heads (action outputs, then the
// value) on the N dimension, 16 at a time; its four waves take a quarter of the contraction each (H is a multiple
// of 64) and the partial tiles are added in LDS in a fixed order: four times as many waves in flight as with one
// wave per block, which is what a latency-bound streaming read needs.
__global__ __launch_bounds__(256) void heads_fwd_kernel(const float* __restrict__ h, int M, int H, int A,
                                                        const float* __restrict__ W_a, const float* __restrict__ b_a,
                                                        const float* __restrict__ w_v, const float* __restrict__ b_v,
                                                        float* __restrict__ head_out, float* __restrict__ value) {
    __shared__ f32x4_t s_part[3][64];
    const int lane = threadIdx.x & 63, lr = lane & 15, lk = lane >> 4, wave = threadIdx.x >> 6;
    const int p0 = blockIdx.x * 16;
    const bool row_ok = p0 + lr < M;
    const int kq = H / 4;   // this wave's share of the contraction: [wave * kq, (wave + 1) * kq)
    const float* hrow = h + (size_t)(row_ok ? p0 + lr : p0) * H + wave * kq + lk * 4;
    for (int ht = 0; ht * 16 <= A; ++ht) {
        const int hd = ht * 16 + lr;   // this lane's head as B operand
        const float* wrow = (hd < A ? W_a + (size_t)hd * H : w_v) + wave * kq + lk * 4;
        const bool head_ok = hd <= A;
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
        for (int k0 = 0; k0 < kq; k0 += 16) {
            f32x4_t av = *reinterpret_cast<const f32x4_t*>(hrow + k0);
            f32x4_t wv = *reinterpret_cast<const f32x4_t*>(wrow + k0);
            if (!row_ok) av = f32x4_t{0.f, 0.f, 0.f, 0.f};
            if (!head_ok) wv = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < 4; ++e) acc = mfma_f32_16x16x4(av[e], wv[e], acc);
        }
        __syncthreads();   // s_part may still be read from the previous head tile
        if (wave > 0) s_part[wave - 1][lane] = acc;
        __syncthreads();
        if (wave > 0) continue;
#pragma unroll
        for (int w = 0; w < 3; ++w) {
            const f32x4_t o = s_part[w][lane];
            acc[0] += o[0]; acc[1] += o[1]; acc[2] += o[2]; acc[3] += o[3];
        }
        // element r of the lane: row lk*4 + r, head ht*16 + lr
        if (head_ok) {
            const float bias = hd < A ? b_a[hd] : b_v[0];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int p = p0 + lk * 4 + r;
                if (p >= M) continue;
                if (hd < A) head_out[(size_t)p * A + hd] = acc[r] + bias;
                else value[p] = acc[r] + bias;
            }
        }
    }
}

// dh[p][j] = sum_a d_u[p][a] W_a[a][j] + d_v[p] w_v[j].  A thread owns 4 adjacent columns (16-byte stores; H is a
// multiple of 64) for a block of HB_ROWS rows, so a head weight is read once per block instead of once per row
// (the loss gradients are wave-uniform scalars).  Bound by writing dh once.
constexpr int HB_ROWS = 8;
__global__ __launch_bounds__(256) void heads_bwd_dh_kernel(const float* __restrict__ d_u, const float* __restrict__ d_v,
                                                           int M, int H, int A, const float* __restrict__ W_a,
                                                           const float* __restrict__ w_v, float* __restrict__ dh,
                                                           int32_t* __restrict__ clear, int n_clear) {
    __shared__ float s_g[HB_ROWS][64];   // the block's loss gradients: heads 0..A-1, then the value head
    const int j = (blockIdx.x * 256 + threadIdx.x) * 4;
    const int p0 = blockIdx.y * HB_ROWS;
    // (first kernel of the backward pass: it also clears the synchronisation words of the two-layer launch that
    // follows, which saves a launch of its own)
    if (blockIdx.x == 0)
        for (int i = blockIdx.y * 256 + threadIdx.x; i < n_clear; i += gridDim.y * 256) clear[i] = 0;
    for (int i = threadIdx.x; i < HB_ROWS * 64; i += 256) {
        const int r = i >> 6, a = i & 63, p = p0 + r;
        s_g[r][a] = (p < M) ? (a < A ? d_u[(size_t)p * A + a] : (a == A ? d_v[p] : 0.f)) : 0.f;
    }
    __syncthreads();
    if (j >= H) return;
    f32x4_t s[HB_ROWS];
    const f32x4_t wv = *reinterpret_cast<const f32x4_t*>(w_v + j);
#pragma unroll
    for (int r = 0; r < HB_ROWS; ++r) {
        const float g = s_g[r][A];
        s[r] = f32x4_t{g * wv[0], g * wv[1], g * wv[2], g * wv[3]};
    }
    for (int a = 0; a < A; ++a) {
        const f32x4_t w = *reinterpret_cast<const f32x4_t*>(W_a + (size_t)a * H + j);
#pragma unroll
        for (int r = 0; r < HB_ROWS; ++r) {
            const float g = s_g[r][a];   // same address in every lane: a broadcast read
            s[r][0] += g * w[0]; s[r][1] += g * w[1]; s[r][2] += g * w[2]; s[r][3] += g * w[3];
        }
    }
#pragma unroll
    for (int r = 0; r < HB_ROWS; ++r)
        if (p0 + r < M) *reinterpret_cast<f32x4_t*>(dh + (size_t)(p0 + r) * H + j) = s[r];
}

// Partial sums over a block of rows: part[rb][a][j] = sum_{p in block rb} du(p,a) * h[p][j], a = 0..A (A = value head).
// A thread owns 4 adjacent columns (16-byte loads of h; H is a multiple of 64) and reads h once per 8 heads, four
// rows in flight; the loss gradients are wave-uniform scalars.  Bound by reading h once.
constexpr int HW_ROWS = 32;  // rows per row block
__global__ __launch_bounds__(256) void heads_wgrad_partial_kernel(const float* __restrict__ d_u,
                                                                  const float* __restrict__ d_v,
                                                                  const float* __restrict__ h, int M, int H, int A,
                                                                  float* __restrict__ part, float* __restrict__ part_b) {
    __shared__ float s_g[HW_ROWS][64];   // the block's loss gradients: heads 0..A-1, then the value head, then zeros
    const int j = (blockIdx.x * 256 + threadIdx.x) * 4;
    const int rb = blockIdx.y;
    const int p_lo = rb * HW_ROWS, p_hi = min(M, p_lo + HW_ROWS);
    for (int i = threadIdx.x; i < HW_ROWS * 64; i += 256) {
        const int r = i >> 6, a = i & 63, p = p_lo + r;
        s_g[r][a] = (p < p_hi) ? (a < A ? d_u[(size_t)p * A + a] : (a == A ? d_v[p] : 0.f)) : 0.f;
    }
    __syncthreads();
    // bias gradients: the block's sum of every head's loss gradient (first column block only), rows in order
    if (blockIdx.x == 0 && (int)threadIdx.x <= A) {
        float sb = 0.f;
        for (int r = 0; r < HW_ROWS; ++r) sb += s_g[r][threadIdx.x];
        part_b[(size_t)rb * 64 + threadIdx.x] = sb;
    }
    if (j >= H) return;
    // 16 heads per pass over the block's rows (one pass for every policy of the paper: 4 or 11 outputs + the value)
    for (int a0 = 0; a0 <= A; a0 += 16) {
        f32x4_t acc[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int p = p_lo; p < p_hi; p += 4) {
            f32x4_t hv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                hv[u] = (p + u < p_hi) ? *reinterpret_cast<const f32x4_t*>(h + (size_t)(p + u) * H + j) : f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (p + u >= p_hi) continue;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float g = s_g[p + u - p_lo][a0 + e];   // same address in every lane: a broadcast read
                    acc[e][0] += g * hv[u][0]; acc[e][1] += g * hv[u][1]; acc[e][2] += g * hv[u][2]; acc[e][3] += g * hv[u][3];
                }
            }
        }
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (a0 + e <= A) *reinterpret_cast<f32x4_t*>(part + ((size_t)rb * (A + 1) + a0 + e) * H + j) = acc[e];
    }
}
// One workgroup adds the row blocks' partial sums for 64 columns of one head: its four waves take a quarter of the
// row blocks each (in index order, 8 loads in flight), and the four shares are added in wave order.
constexpr int HF_COLS = 64;
__global__ __launch_bounds__(256) void heads_wgrad_final_kernel(const float* __restrict__ part, const float* __restrict__ part_b, int n_rb,
                                                                int H, int A, float* __restrict__ dW_a, float* __restrict__ dw_v,
                                                                float* __restrict__ db_a, float* __restrict__ db_v) {
    __shared__ float red[256];
    const int lane = threadIdx.x & 63, share = threadIdx.x >> 6;
    const int j = blockIdx.x * HF_COLS + lane;
    const int a = blockIdx.y;
    if (blockIdx.x == 0) {
        float sb = 0.f;
        for (int rb = threadIdx.x; rb < n_rb; rb += 256) sb += part_b[(size_t)rb * 64 + a];
        red[threadIdx.x] = sb;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            if (a < A) db_a[a] = red[0]; else db_v[0] = red[0];
        }
        __syncthreads();
    }
    const int per = (n_rb + 3) / 4, rb_end = min(n_rb, (share + 1) * per);
    float s = 0.f;
    int rb = share * per;
    if (j < H) {
        for (; rb + 8 <= rb_end; rb += 8) {   // 8 loads in flight, added in index order
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = part[((size_t)(rb + u) * (A + 1) + a) * H + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; rb < rb_end; ++rb) s += part[((size_t)rb * (A + 1) + a) * H + j];
    }
    red[threadIdx.x] = s;
    __syncthreads();
    if (share == 0 && j < H) {
        s = ((red[lane] + red[64 + lane]) + red[128 + lane]) + red[192 + lane];
        if (a < A) dW_a[(size_t)a * H + j] = s; else dw_v[j] = s;
    }
}

// out[perm(c)] (and out2) = sum over the n_rb rows of part[n_rb][cols], in row order (deterministic);
// unperm_h > 0 maps interleaved column c to (c%4)*H + c/4.
// blockIdx.y = 1: the second set (the other layer of a two-layer launch), whose partial sums follow at part_stride.
__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ part, int n_rb, int cols,
                                                           int unperm_h, float* __restrict__ out,
                                                           float* __restrict__ out2, size_t part_stride,
                                                           float* __restrict__ out_b, float* __restrict__ out2_b) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= cols) return;
    if (blockIdx.y == 1) { part += part_stride; out = out_b; out2 = out2_b; }
    float s = 0.f;
    int rb = 0;
    for (; rb + 8 <= n_rb; rb += 8) {   // 8 loads in flight, added in index order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = part[(size_t)(rb + u) * cols + c];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; rb < n_rb; ++rb) s += part[(size_t)rb * cols + c];
    const int dst = unperm_h > 0 ? (c & 3) * unperm_h + (c >> 2) : c;
    out[dst] = s;
    if (out2) out2[dst] = s;
}

// ---------------------------------------------------------------- workspace
constexpr int REC_FLAG_WORDS = 8 * REC_MAX_GROUP + 64;   // flags[group][32], then one ticket per group

struct LayerWs {
    void* wih;    // [4H, D_l]  operand type, interleaved rows
    void* wihT;   // [D_l, 4H]
    void* whh;    // [4H, H]
    void* whhT;   // [H, 4H]
    float* bias;  // [4H]
    float* gates; // [M, 4H]
    float* c;     // [M, H]
    float* hout;  // [M, H]
    void* hprev;  // [M, H] operand type
    void* hcopy;  // [M, H] operand type: h_t, for the workers of a two-layer launch
};
struct LstmWs {
    int* err;          // word 0 of the workspace
    int* flags;        // [REC_FLAG_WORDS]: per-workgroup flags of a recurrent launch, then its ticket counters
    long long* prof;   // [128] phase counters of the recurrent kernels (forward 0..15, backward 16..31; +32: consumer layer), timeline, workers
    LayerWs layer[8];
    void* dz[2];       // [M, 4H] operand type; the second one only when two layers share a launch
    int* pipe;         // hand-over words of a two-layer launch: progress[8], queues at [8], done[][] from [16]
    int pipe_words;
    int* plan[2];      // which pieces every group of a two-layer launch runs, and its chunks (lstm_pipe.h): forward, backward
    float* plan_scratch;
    float* dh[2];      // [M, H] ping-pong: gradient arriving at a layer's h
    float* dh_state;   // [M, H]
    float* dc_state;   // [M, H]
    float* part;       // partial sums of the two-stage reductions
    float* part_b;     // [row blocks][64]: the heads' bias gradients per row block
    float* gemm_part;  // partial tiles of GEMMs whose contraction is split over workgroups
    float* db_part;    // [2][8][4H]: per layer of a launch and group, the sum of the gate gradients over the group's rows
    size_t bytes;
};

inline size_t part_floats(const ver_lstm_cfg& c, int M) {
    const size_t rb_heads = (size_t)(M + HW_ROWS - 1) / HW_ROWS;
    return rb_heads * (c.act_dim + 1) * c.hidden;   // the row-block partial sums of the heads' weight gradient
}

// Largest split-K scratch any GEMM of the forward or backward pass asks for.
inline size_t gemm_part_max(const ver_lstm_cfg& c, int M) {
    const int bk = c.compute ? GemmGeom<MODE_BF16>::BK : GemmGeom<MODE_F32>::BK;
    const int H = c.hidden;
    size_t m = 0;
    for (int l = 0; l < c.n_layers; ++l) {
        const int D = l == 0 ? c.input_dim : H;
        const size_t v[4] = {gemm_part_floats(M, 4 * H, D, bk), gemm_part_floats(M, D, 4 * H, bk),
                             gemm_part_floats(4 * H, D, M, bk), gemm_part_floats(4 * H, H, M, bk)};
        for (size_t x : v) m = x > m ? x : m;
    }
    return m;
}

inline void lstm_ws_layout(const ver_lstm_cfg& c, int M, void* base, LstmWs* ws) {
    const size_t es = c.compute ? 2 : 4;
    const size_t H = c.hidden, Mz = (size_t)M;
    Carver cv(base);
    int* head = cv.take<int>(64);
    ws->err = head;
    ws->flags = cv.take<int>(REC_FLAG_WORDS);
    ws->prof = cv.take<long long>(128);
    // the hand-over words sit right behind, so that one fill clears everything a launch needs cleared
    ws->pipe_words = pipe_sync_words(M);
    ws->pipe = cv.take<int>(ws->pipe_words);
    ws->plan[0] = cv.take<int>(plan_words(M));
    ws->plan[1] = cv.take<int>(plan_words(M));
    ws->plan_scratch = cv.take<float>(plan_scratch_floats(M));
    for (int l = 0; l < c.n_layers; ++l) {
        const size_t D = l == 0 ? c.input_dim : H;
        LayerWs& L = ws->layer[l];
        L.wih = cv.take<char>(4 * H * D * es);
        L.wihT = cv.take<char>(4 * H * D * es);
        L.whh = cv.take<char>(4 * H * H * es);
        L.whhT = cv.take<char>(4 * H * H * es);
        L.bias = cv.take<float>(4 * H);
        L.gates = cv.take<float>(Mz * 4 * H);
        L.c = cv.take<float>(Mz * H);
        L.hout = cv.take<float>(Mz * H);
        L.hprev = cv.take<char>(Mz * H * es);
        L.hcopy = (c.n_layers == 2 && l == 0) ? cv.take<char>(Mz * H * es) : nullptr;
    }
    ws->dz[0] = cv.take<char>(Mz * 4 * H * es);
    ws->dz[1] = c.n_layers == 2 ? cv.take<char>(Mz * 4 * H * es) : ws->dz[0];
    ws->dh[0] = cv.take<float>(Mz * H);
    ws->dh[1] = cv.take<float>(Mz * H);
    ws->dh_state = cv.take<float>(2 * Mz * H);
    ws->dc_state = cv.take<float>(2 * Mz * H);
    ws->part = cv.take<float>(part_floats(c, M));
    ws->part_b = cv.take<float>((size_t)(M + HW_ROWS - 1) / HW_ROWS * 64);
    ws->gemm_part = cv.take<float>(gemm_part_max(c, M));
    ws->db_part = cv.take<float>((size_t)2 * REC_GROUPS * 4 * H);
    ws->bytes = cv.used;
}

inline int check_cfg(const ver_lstm_cfg* c, int M) {
    if (!c || M <= 0) return VER_EINVAL;
    if (c->compute != 0 && c->compute != 1) return VER_EINVAL;
    if (c->layer_by_layer != 0 && c->layer_by_layer != 1) return VER_EINVAL;
    if (c->x_bf16 && !c->compute) return VER_EINVAL;
    if (c->n_layers < 1 || c->n_layers > 8 || c->act_dim < 1 || c->act_dim > 63) return VER_EUNSUPPORTED;
    if (c->hidden < 64 || c->hidden % 64 != 0 || c->input_dim < 4 || c->input_dim % 4 != 0) return VER_EUNSUPPORTED;
    // a wave keeps its [16, H] share of W_hh in 128 registers; a 16-row tile of dz ([16, 4H]) must fit in LDS
    if (c->hidden > (c->compute ? 1024 : 512)) return VER_EUNSUPPORTED;
    // the time-loop kernels address the rows of an activation array with 32-bit byte offsets
    if ((long long)M * 16 * c->hidden >= (1LL << 31)) return VER_EUNSUPPORTED;
    return VER_OK;
}

// How many 16-row tiles of exchanged rows fit in a CU's 160 KB of LDS next to the reduction buffer.
inline int rec_tiles(size_t tile_bytes, size_t red_bytes_per_tile) {
    int n = (int)((160 * 1024) / (tile_bytes + red_bytes_per_tile));
    return n < 1 ? 1 : (n > REC_NTC ? REC_NTC : n);
}

template <typename K>
inline bool set_lds(K kernel, size_t bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes) == hipSuccess;
}

// C[M, N] = A[M, K] B[N, K]^T (+ bias), all three row-major, A and B bf16: the LDS-direct 128 x 256 tiles, one
// workgroup per tile.  False if the shape does not fit the kernel's 32-bit byte offsets (the caller then uses
// the general GEMM).
inline bool launch_proj_dma(const void* A, const void* B, float* C, const float* bias, int M, int N, int K, hipStream_t s) {
    if ((size_t)M * K * 2 >= 0x7fffffff || (size_t)N * K * 2 >= 0x7fffffff || (size_t)M * N * 4 >= 0x7fffffff) return false;
    if (!set_lds(lstm_proj_dma_kernel, (size_t)PIPE_STAGES * PIPE_STAGE_BYTES)) return false;
    PipeWork pw{};
    pw.A = A; pw.B = B; pw.C = C; pw.bias = bias; pw.K = K; pw.N = N; pw.M = M;
    const int tiles_n = (N + PIPE_BN - 1) / PIPE_BN, tiles_m = (M + PIPE_BM - 1) / PIPE_BM;
    hipLaunchKernelGGL(lstm_proj_dma_kernel, dim3(tiles_m * tiles_n), dim3(REC_THREADS), (size_t)PIPE_STAGES * PIPE_STAGE_BYTES, s,
                       pw, M, tiles_n);
    return true;
}

// The persistent time-loop kernels are written for the whole of one MI355X: a grid of one workgroup per CU that
// must be co-resident, grouped by the XCD it runs on (8 XCDs of 32 CUs).  On any other device (another
// architecture, a partition of the chip with fewer CUs) their groups would be incomplete and the bounded waits
// would give up, so the entry points refuse to launch there.  Looked up once per device.
inline int device_fits_time_loops() {
    static std::mutex lock;
    static signed char known[64];   // 0 unknown, 1 fits, -1 does not
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return VER_EHIP;
    if (dev < 0 || dev >= 64) return VER_EUNSUPPORTED;
    std::lock_guard<std::mutex> hold(lock);
    if (known[dev] == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return VER_EHIP;
        const bool ok = prop.multiProcessorCount == REC_GRID && std::strncmp(prop.gcnArchName, "gfx950", 6) == 0;
        known[dev] = ok ? 1 : -1;
    }
    return known[dev] > 0 ? VER_OK : VER_EUNSUPPORTED;
}

// LDS of a worker of a two-layer launch: one 128 x BK and one 256 x BK operand tile.
template <int MODE>
inline size_t pipe_worker_lds() {
    if (MODE == MODE_BF16) return (size_t)PIPE_STAGES * PIPE_STAGE_BYTES;
    return (size_t)(PIPE_BM + PIPE_BN) * GemmGeom<MODE>::LDS_STRIDE * sizeof(typename LdsElem<MODE>::type);
}
// Before the forward two-layer launch: one small kernel zeroes the flags, ticket counters, hand-over words and the
// sticky time-out word at the start of the workspace, and writes the plans of both launches of the minibatch (the
// backward call runs on the packing of the forward call whose activations it finds in the workspace).  Before the
// backward launch only the words are cleared.
inline void pipe_prepare_fwd(LstmWs& ws, int M, const int32_t* info, const int32_t* batch_sizes, hipStream_t s) {
    int* last = ws.pipe + ws.pipe_words;
    hipLaunchKernelGGL(lstm_pipe_plan_kernel, dim3(1), dim3(PLAN_THREADS), 0, s, info, batch_sizes, M, ws.plan[0], ws.plan[1],
                       ws.plan_scratch, ws.err, (int)(last - ws.err), PLAN_COST_FWD, PLAN_COST_BWD);
}
inline void pipe_work(const LstmWs& ws, int dir, int M, const int32_t* t_off, PipeWork* pw) {
    pw->M = M;
    pw->t_off = t_off;
    pw->plan = ws.plan[dir];
    pw->sync = ws.pipe;
    pw->err = ws.err;
    pw->prof_all = ws.prof;
}

template <int MODE>
int run_fwd(const ver_lstm_cfg& c, const void* x, int M, const int32_t* info, const int32_t* batch_sizes,
            const int32_t* t_off, const float* h0, const float* c0, int seq_cap, const float* const* w,
            float* head_out, float* value, LstmWs& ws, hipStream_t s) {
    typedef typename RecGeom<MODE>::E E;
    const int H = c.hidden, A = c.act_dim;
    const bool pipelined = c.n_layers == 2 && !c.layer_by_layer;   // both time loops in one launch
    if (!pipelined) fill_words(ws.err, 1, 0, s);

    // 8 waves = row groups x shares of the contraction (TPW tiles of 16 gate rows per wave): a workgroup owns
    // 8 tiles (32 units) when 32 workgroups need all of H/32 units each, else 4 tiles (16 units)
    const bool wide = H / 16 > REC_MAX_GROUP;
    // Shares of the contraction: with 8 tiles per workgroup two (a wave then reads 16 operand blocks per piece tile
    // and the cell update adds two partial sums; measured 2.7 % faster than four shares, which read less from LDS but
    // reduce more: the group that bounds a launch has one or two alive pieces, whose reads are broadcasts; one share,
    // without any reduction, is 9 % slower), with 4 tiles four (two was measured 0.4 % slower on H = 512).
    const bool quarter = MODE == MODE_F32 || (!wide && H % 128 == 0);   // a quarter of H is a whole number of operand blocks
    const int ks = quarter ? 4 : 2;
    const int mt = wide ? 8 : 4;
    const size_t tile = (size_t)16 * (H + RecGeom<MODE>::PAD) * sizeof(E);
    const size_t red_per_tile = (size_t)ks * mt * 64 * 16 + (size_t)16 * 4 * mt * sizeof(E);   // partial sums + new h
    const int ntc = rec_tiles(tile, red_per_tile);
    size_t lds = ntc * (tile + red_per_tile);
    if (pipelined && pipe_worker_lds<MODE>() > lds) lds = pipe_worker_lds<MODE>();
    const int nb = (H / ks) / RecGeom<MODE>::KBLK;

    // operand-type copies of every layer's weights (and their transposes) and the summed biases: one launch
    auto prep_all = [&]() {
        ProfScope prof(VER_PROF_LSTM_PREP, s);
        PrepArgs pa{};
        int n = 0, max_cols = H;
        for (int l = 0; l < c.n_layers; ++l) {
            const int D = l == 0 ? c.input_dim : H;
            LayerWs& L = ws.layer[l];
            max_cols = D > max_cols ? D : max_cols;
            pa.job[n++] = PrepJob{w[4 * l], nullptr, L.wih, L.wihT, D};
            pa.job[n++] = PrepJob{w[4 * l + 1], nullptr, L.whh, L.whhT, H};
            pa.job[n++] = PrepJob{w[4 * l + 2], w[4 * l + 3], L.bias, nullptr, 0};
        }
        hipLaunchKernelGGL(prep_weights_kernel<E>, dim3((max_cols + 63) / 64, 4 * H / 64, n), dim3(256), 0, s, pa, H);
    };
    // time-batched input projection: gates[M, 4H] = x W_ih^T + (b_ih + b_hh), interleaved columns
    auto project = [&](int l) {
        const int D = l == 0 ? c.input_dim : H;
        LayerWs& L = ws.layer[l];
        ProfScope prof(VER_PROF_LSTM_GEMM_FWD, s);
        if (l == 0) {
            if constexpr (MODE == MODE_BF16) {
                // bf16 rows on both sides: the LDS-direct tiles of the two-layer launch, as a launch of their own
                if (c.x_bf16 && launch_proj_dma(x, L.wih, L.gates, L.bias, M, 4 * H, D, s)) return;
            }
            if (c.x_bf16)
                gemm_launch<MODE, bf16_t, E, false>(static_cast<const bf16_t*>(x), D, static_cast<const E*>(L.wih), D,
                                                    L.gates, 4 * H, M, 4 * H, D, L.bias, 0, ws.gemm_part, true, s);
            else
                gemm_launch<MODE, float, E, false>(static_cast<const float*>(x), D, static_cast<const E*>(L.wih), D,
                                                   L.gates, 4 * H, M, 4 * H, D, L.bias, 0, ws.gemm_part, true, s);
        } else {
            gemm_launch<MODE, float, E, false>(ws.layer[l - 1].hout, H, static_cast<const E*>(L.wih), H, L.gates,
                                               4 * H, M, 4 * H, H, L.bias, 0, ws.gemm_part, true, s);
        }
    };
    auto rec_args = [&](int l) {
        LayerWs& L = ws.layer[l];
        RecFwdArgs ra;
        ra.info = info; ra.batch_sizes = batch_sizes; ra.t_off = t_off;
        ra.gates = L.gates; ra.c = L.c; ra.hout = L.hout; ra.hprev = L.hprev; ra.hcopy = L.hcopy; ra.whh = L.whh;
        ra.h0 = h0 ? h0 + (size_t)l * seq_cap * H : nullptr;
        ra.c0 = c0 ? c0 + (size_t)l * seq_cap * H : nullptr;
        ra.H = H; ra.seq_cap = seq_cap; ra.M = M; ra.flags = ws.flags; ra.ticket = ws.flags + 8 * REC_MAX_GROUP;
        ra.err = ws.err; ra.prof = ws.prof + (pipelined && l == 1 ? 32 : 0); ra.prof_all = ws.prof;
        ra.G = H / (4 * mt); ra.ntc = ntc;
        return ra;
    };
    bool ok = true;
#define VER_FWD_LAUNCH(KERNEL, ARGS, TPW_, KS_, NBW_, ST_) do { ok = set_lds(KERNEL<MODE, TPW_, KS_, NBW_, ST_>, lds); \
        if (ok) hipLaunchKernelGGL((KERNEL<MODE, TPW_, KS_, NBW_, ST_>), dim3(REC_GRID), dim3(REC_THREADS), lds, s, ARGS); } while (0)
#define VER_FWD_DISPATCH(KERNEL, ARGS) do { \
        if constexpr (MODE == MODE_BF16) { \
            if (wide) { \
                if (!quarter && nb == 16) VER_FWD_LAUNCH(KERNEL, ARGS, 2, 2, 16, true); \
                else VER_FWD_LAUNCH(KERNEL, ARGS, 2, 2, 16, false); \
            } else { \
                if (!quarter && nb == 8) VER_FWD_LAUNCH(KERNEL, ARGS, 1, 2, 8, true); \
                else if (!quarter) VER_FWD_LAUNCH(KERNEL, ARGS, 1, 2, 8, false); \
                else if (nb == 4) VER_FWD_LAUNCH(KERNEL, ARGS, 2, 4, 4, true); \
                else VER_FWD_LAUNCH(KERNEL, ARGS, 2, 4, 4, false); \
            } \
        } else { \
            if (nb == 8) VER_FWD_LAUNCH(KERNEL, ARGS, 2, 4, 8, true); \
            else VER_FWD_LAUNCH(KERNEL, ARGS, 2, 4, 8, false); \
        } } while (0)

    prep_all();
    if (pipelined) {
        project(0);
        pipe_prepare_fwd(ws, M, info, batch_sizes, s);
        PipeFwdArgs pa;
        pa.l0 = rec_args(0);
        pa.l1 = rec_args(1);
        pa.work.A = ws.layer[0].hcopy; pa.work.B = ws.layer[1].wih; pa.work.C = ws.layer[1].gates;
        pa.work.bias = ws.layer[1].bias; pa.work.K = H; pa.work.N = 4 * H;
        pipe_work(ws, 0, M, t_off, &pa.work);
        pa.tiles_n = (4 * H + PIPE_BN - 1) / PIPE_BN;
        ProfScope prof(VER_PROF_LSTM_REC_FWD, s);
        VER_FWD_DISPATCH(lstm_pipe_fwd_kernel, pa);
        if (!ok) return VER_EHIP;
    } else {
        for (int l = 0; l < c.n_layers; ++l) {
            project(l);
            fill_words(ws.flags, REC_FLAG_WORDS, 0, s);
            RecFwdArgs ra = rec_args(l);
            ProfScope prof(VER_PROF_LSTM_REC_FWD, s);
            VER_FWD_DISPATCH(lstm_rec_fwd_kernel, ra);
            if (!ok) return VER_EHIP;
        }
    }
#undef VER_FWD_DISPATCH
#undef VER_FWD_LAUNCH
    ProfScope prof(VER_PROF_HEADS_FWD, s);
    hipLaunchKernelGGL(heads_fwd_kernel, dim3((M + 15) / 16), dim3(256), 0, s, ws.layer[c.n_layers - 1].hout, M, H, A,
                       w[4 * c.n_layers], w[4 * c.n_layers + 1], w[4 * c.n_layers + 2], w[4 * c.n_layers + 3],
                       head_out, value);
    return launch_status();
}

template <int MODE>
int run_bwd(const ver_lstm_cfg& c, const void* x, int M, const int32_t* info, const int32_t* batch_sizes,
            const int32_t* t_off, const float* c0, int seq_cap, const float* const* w, const float* d_u,
            const float* d_v, float* const* gw, float* d_x, LstmWs& ws, hipStream_t s) {
    typedef typename RecGeom<MODE>::E E;
    const int H = c.hidden, A = c.act_dim, nl = c.n_layers;
    const float* h_top = ws.layer[nl - 1].hout;
    const bool pipelined = nl == 2 && !c.layer_by_layer;   // both time loops in one launch
    // heads
    {
    ProfScope prof(VER_PROF_HEADS_BWD, s);
    hipLaunchKernelGGL(heads_bwd_dh_kernel, dim3((H / 4 + 255) / 256, (M + HB_ROWS - 1) / HB_ROWS), dim3(256), 0, s, d_u, d_v, M, H, A, w[4 * nl],
                       w[4 * nl + 2], ws.dh[0], pipelined ? ws.flags : nullptr, pipelined ? (int)(ws.pipe + ws.pipe_words - ws.flags) : 0);
    const int rb_h = (M + HW_ROWS - 1) / HW_ROWS;
    hipLaunchKernelGGL(heads_wgrad_partial_kernel, dim3((H / 4 + 255) / 256, rb_h), dim3(256), 0, s, d_u, d_v, h_top, M, H,
                       A, ws.part, ws.part_b);
    hipLaunchKernelGGL(heads_wgrad_final_kernel, dim3((H + HF_COLS - 1) / HF_COLS, A + 1), dim3(256), 0, s, ws.part, ws.part_b, rb_h, H, A,
                       gw[4 * nl], gw[4 * nl + 2], gw[4 * nl + 1], gw[4 * nl + 3]);
    }

    // one wave per (16 units, share of the 4H contraction): 2 tiles x 4 when H/16 > 32 workgroups, else 1 x 8
    const bool wide = H / 16 > REC_MAX_GROUP;
    const int mt = wide ? 2 : 1, ks = wide ? 4 : 8;
    const size_t tile = (size_t)16 * (4 * H + RecGeom<MODE>::PAD) * sizeof(E);
    const size_t red_per_tile = (size_t)ks * mt * 64 * 16 + (size_t)16 * 16 * mt * sizeof(float);   // partial sums + carried dh
    const int ntc = rec_tiles(tile, red_per_tile);
    size_t lds = ntc * (tile + red_per_tile);
    if (pipelined && pipe_worker_lds<MODE>() > lds) lds = pipe_worker_lds<MODE>();
    const int ni = (4 * H / ks) / RecGeom<MODE>::KBLK;

    // ws.dh[l == nl-1 ? 0 : 1 ...]: gradient arriving at layer l's h; dz_of(l): its gate gradients
    auto dz_of = [&](int l) { return pipelined ? ws.dz[l] : ws.dz[0]; };
    auto rec_args = [&](int l, const float* dh_above) {
        LayerWs& L = ws.layer[l];
        RecBwdArgs ra;
        ra.info = info; ra.batch_sizes = batch_sizes; ra.t_off = t_off;
        ra.gates = L.gates; ra.c = L.c; ra.c0 = c0 ? c0 + (size_t)l * seq_cap * H : nullptr;
        ra.dh_above = dh_above; ra.dz = dz_of(l); ra.whhT = L.whhT;
        // the two layers of a shared launch carry their state in separate halves of the scratch
        ra.dh_state = ws.dh_state + (pipelined ? (size_t)l * M * H : 0);
        ra.dc_state = ws.dc_state + (pipelined ? (size_t)l * M * H : 0);
        ra.db_part = ws.db_part + (pipelined ? (size_t)l * REC_GROUPS * 4 * H : 0);
        ra.H = H; ra.seq_cap = seq_cap; ra.flags = ws.flags; ra.ticket = ws.flags + 8 * REC_MAX_GROUP;
        ra.err = ws.err; ra.prof = ws.prof + 16 + (pipelined && l == 0 ? 32 : 0); ra.prof_all = ws.prof;
        ra.G = H / (16 * mt); ra.ntc = ntc;
        return ra;
    };
    bool ok = true;
#define VER_BWD_LAUNCH(KERNEL, ARGS, MT_, KS_, N_) do { ok = set_lds(KERNEL<MODE, MT_, KS_, N_>, lds); \
        if (ok) hipLaunchKernelGGL((KERNEL<MODE, MT_, KS_, N_>), dim3(REC_GRID), dim3(REC_THREADS), lds, s, ARGS); } while (0)
#define VER_BWD_DISPATCH(KERNEL, ARGS) do { \
        if (wide) { \
            if (ni == 32) VER_BWD_LAUNCH(KERNEL, ARGS, 2, 4, 32); else VER_BWD_LAUNCH(KERNEL, ARGS, 2, 4, 0); \
        } else { \
            if (ni == 16) VER_BWD_LAUNCH(KERNEL, ARGS, 1, 8, 16); \
            else if (ni == 8) VER_BWD_LAUNCH(KERNEL, ARGS, 1, 8, 8); \
            else if (ni == 4) VER_BWD_LAUNCH(KERNEL, ARGS, 1, 8, 4); \
            else VER_BWD_LAUNCH(KERNEL, ARGS, 1, 8, 0); \
        } } while (0)
    // everything of layer l that is not the time loop: dx (optional), dW_ih, dW_hh, db
    TnGroup dw_group;
    auto layer_grads = [&](int l, float* dx, bool flush_dw) {
        const int D = l == 0 ? c.input_dim : H;
        LayerWs& L = ws.layer[l];
        const E* dz = static_cast<const E*>(dz_of(l));
        // gradient w.r.t. the layer input: dx[M, D] = dz[M, 4H] . W_ih[4H, D]
        if (dx) {
            ProfScope prof(VER_PROF_LSTM_GEMM_DX, s);
            bool done = false;
            if constexpr (MODE == MODE_BF16) done = launch_proj_dma(dz, L.wihT, dx, nullptr, M, D, 4 * H, s);
            if (!done)
                gemm_launch<MODE, E, E, false>(dz, 4 * H, static_cast<const E*>(L.wihT), 4 * H, dx, D, M, D, 4 * H,
                                               nullptr, 0, ws.gemm_part, true, s);
        }
        // dW_ih[4H, D] = dz^T x ; dW_hh[4H, H] = dz^T h_{t-1}; stored gate-major.  Contractions whose operands are both
        // bf16 join the grouped launch (dw_group) when they fit it; the others are launched on the spot.
        {
        ProfScope prof(VER_PROF_LSTM_GEMM_DW, s);
        auto grouped = [&](const void* B, int ldb, float* C, int Nc) {
            if constexpr (MODE == MODE_BF16)
                return dw_group.add(reinterpret_cast<const bf16_t*>(dz), 4 * H, static_cast<const bf16_t*>(B), ldb, C, Nc, 4 * H, Nc, M, H);
            return false;
        };
        if (l > 0 && pipelined && ws.layer[l - 1].hcopy) {   // the layer below left its h in operand type
            if (!grouped(ws.layer[l - 1].hcopy, H, gw[4 * l], D))
                gemm_launch<MODE, E, E, true>(dz, 4 * H, static_cast<const E*>(ws.layer[l - 1].hcopy), H, gw[4 * l], D, 4 * H, D, M,
                                              nullptr, H, ws.gemm_part, true, s);
        } else if (l > 0)
            gemm_launch<MODE, E, float, true>(dz, 4 * H, ws.layer[l - 1].hout, H, gw[4 * l], D, 4 * H, D, M, nullptr, H, ws.gemm_part, true, s);
        else if (c.x_bf16) {
            if (!grouped(x, D, gw[4 * l], D))
                gemm_launch<MODE, E, bf16_t, true>(dz, 4 * H, static_cast<const bf16_t*>(x), D, gw[4 * l], D, 4 * H, D, M,
                                                   nullptr, H, ws.gemm_part, true, s);
        } else
            gemm_launch<MODE, E, float, true>(dz, 4 * H, static_cast<const float*>(x), D, gw[4 * l], D, 4 * H, D, M,
                                              nullptr, H, ws.gemm_part, true, s);
        if (!grouped(L.hprev, H, gw[4 * l + 1], H))
            gemm_launch<MODE, E, E, true>(dz, 4 * H, static_cast<const E*>(L.hprev), H, gw[4 * l + 1], H, 4 * H, H, M,
                                          nullptr, H, ws.gemm_part, true, s);
        if (flush_dw) dw_group.launch(s);
        }
        // db_ih = db_hh = column sums of dz: the time loop left one partial sum per group (two-layer launch: both
        // layers' sums in one launch, after the second call)
        if (!pipelined || l == 0) {
        ProfScope prof(VER_PROF_LSTM_DBIAS, s);
        const size_t stride = (size_t)REC_GROUPS * 4 * H;
        if (pipelined)
            hipLaunchKernelGGL(colsum_final_kernel, dim3((4 * H + 255) / 256, 2), dim3(256), 0, s, ws.db_part, PIPE_GROUPS, 4 * H, H,
                               gw[2], gw[3], stride, gw[6], gw[7]);
        else
            hipLaunchKernelGGL(colsum_final_kernel, dim3((4 * H + 255) / 256, 1), dim3(256), 0, s, ws.db_part, REC_GROUPS, 4 * H, H,
                               gw[4 * l + 2], gw[4 * l + 3], stride, static_cast<float*>(nullptr), static_cast<float*>(nullptr));
        }
    };

    if (pipelined) {
        PipeBwdArgs pa;   // (the launch's synchronisation words were cleared by heads_bwd_dh_kernel)
        pa.l1 = rec_args(1, ws.dh[0]);
        pa.l0 = rec_args(0, ws.dh[1]);
        pa.work.A = ws.dz[1]; pa.work.B = ws.layer[1].wihT; pa.work.C = ws.dh[1]; pa.work.bias = nullptr;
        pa.work.K = 4 * H; pa.work.N = H;
        pipe_work(ws, 1, M, t_off, &pa.work);
        pa.tiles_n = (H + PIPE_BN - 1) / PIPE_BN;
        {
        ProfScope prof(VER_PROF_LSTM_REC_BWD, s);
        VER_BWD_DISPATCH(lstm_pipe_bwd_kernel, pa);
        if (!ok) return VER_EHIP;
        }
        layer_grads(1, nullptr, false);   // the weight gradients of both layers leave in one grouped launch
        layer_grads(0, d_x, true);
    } else {
        int cur = 0;  // ws.dh[cur] holds the gradient arriving at the current layer's h
        for (int l = nl - 1; l >= 0; --l) {
            fill_words(ws.flags, REC_FLAG_WORDS, 0, s);
            RecBwdArgs ra = rec_args(l, ws.dh[cur]);
            {
            ProfScope prof(VER_PROF_LSTM_REC_BWD, s);
            VER_BWD_DISPATCH(lstm_rec_bwd_kernel, ra);
            if (!ok) return VER_EHIP;
            }
            layer_grads(l, l > 0 ? ws.dh[cur ^ 1] : d_x, true);
            cur ^= 1;
        }
    }
#undef VER_BWD_DISPATCH
#undef VER_BWD_LAUNCH
    return launch_status();
}

}  // namespace
}  // namespace ver

extern "C" size_t ver_lstm_workspace_bytes(const ver_lstm_cfg* cfg, int32_t M) {
    if (ver::check_cfg(cfg, M) != VER_OK) return 0;
    ver::LstmWs ws;
    ver::lstm_ws_layout(*cfg, M, nullptr, &ws);
    return ws.bytes;
}

extern "C" int ver_lstm_fwd(const ver_lstm_cfg* cfg, const void* x_packed, int32_t M, const int32_t* info,
                            const int32_t* batch_sizes, const int32_t* t_off, const float* h0, const float* c0,
                            int32_t seq_cap, const float* const* weights, float* head_out, float* value,
                            void* workspace, size_t workspace_bytes, void* stream) {
    const int st = ver::check_cfg(cfg, M);
    if (st != VER_OK) return st;
    if (!x_packed || !info || !batch_sizes || !t_off || !weights || !head_out || !value) return VER_EINVAL;
    if ((h0 || c0) && seq_cap <= 0) return VER_EINVAL;
    for (int i = 0; i < 4 * cfg->n_layers + 4; ++i)
        if (!weights[i]) return VER_EINVAL;
    if (!workspace || workspace_bytes < ver_lstm_workspace_bytes(cfg, M)) return VER_EWORKSPACE;
    const int dev_st = ver::device_fits_time_loops();
    if (dev_st != VER_OK) return dev_st;
    ver::LstmWs ws;
    ver::lstm_ws_layout(*cfg, M, workspace, &ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    return cfg->compute ? ver::run_fwd<ver::MODE_BF16>(*cfg, x_packed, M, info, batch_sizes, t_off, h0, c0, seq_cap,
                                                       weights, head_out, value, ws, s)
                        : ver::run_fwd<ver::MODE_F32>(*cfg, x_packed, M, info, batch_sizes, t_off, h0, c0, seq_cap,
                                                      weights, head_out, value, ws, s);
}

extern "C" int ver_lstm_bwd(const ver_lstm_cfg* cfg, const void* x_packed, int32_t M, const int32_t* info,
                            const int32_t* batch_sizes, const int32_t* t_off, const float* h0, const float* c0,
                            int32_t seq_cap, const float* const* weights, const float* d_head_out,
                            const float* d_value, float* const* weight_grads, float* d_x, void* workspace,
                            size_t workspace_bytes, void* stream) {
    (void)h0;  // h_{t-1} of every row, including the initial state, was saved by the forward pass
    const int st = ver::check_cfg(cfg, M);
    if (st != VER_OK) return st;
    if (!x_packed || !info || !batch_sizes || !t_off || !weights || !d_head_out || !d_value || !weight_grads)
        return VER_EINVAL;
    if (c0 && seq_cap <= 0) return VER_EINVAL;
    for (int i = 0; i < 4 * cfg->n_layers + 4; ++i)
        if (!weights[i] || !weight_grads[i]) return VER_EINVAL;
    if (!workspace || workspace_bytes < ver_lstm_workspace_bytes(cfg, M)) return VER_EWORKSPACE;
    const int dev_st = ver::device_fits_time_loops();
    if (dev_st != VER_OK) return dev_st;
    ver::LstmWs ws;
    ver::lstm_ws_layout(*cfg, M, workspace, &ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    return cfg->compute ? ver::run_bwd<ver::MODE_BF16>(*cfg, x_packed, M, info, batch_sizes, t_off, c0, seq_cap,
                                                       weights, d_head_out, d_value, weight_grads, d_x, ws, s)
                        : ver::run_bwd<ver::MODE_F32>(*cfg, x_packed, M, info, batch_sizes, t_off, c0, seq_cap,
                                                      weights, d_head_out, d_value, weight_grads, d_x, ws, s);
}
