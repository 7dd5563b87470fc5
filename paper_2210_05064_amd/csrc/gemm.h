// LDS-tiled MFMA GEMM for the time-batched contractions of the LSTM
// (input projections, input gradients, weight gradients).  gfx950 only.
//
//   C[m][n] = sum_k A(m,k) * B(n,k)  (+ bias[n])
//
// Operands are "K-major" (A(m,k) = A[m*lda + k]: the contraction index is
// contiguous) or, with TRANS, "K-minor" (A(m,k) = A[k*lda + m]: used for the
// weight gradients, where the contraction runs over the packed rows).  Either
// way a 128x128 tile of C is built by 4 waves (2x2, 64x64 each) from K-tiles
// staged in LDS as [row][k] so that every MFMA operand is one aligned 16-byte
// LDS read.  K-minor tiles are transposed in registers (4x4 blocks) on the way
// into LDS.  The global loads of K-tile i+1 are issued before the MFMAs of tile
// i (register double buffering), and the contraction can be split over
// gridDim.z with the partial tiles summed in index order by a second kernel, so
// that small outputs still fill the chip; both keep the result deterministic.
//   MODE_BF16: operands rounded to bf16 on the way into LDS (or already bf16),
//              v_mfma_f32_16x16x32_bf16, fp32 accumulate.
//   MODE_F32 : fp32 operands, v_mfma_f32_16x16x4_f32.
#pragma once
#include "common.h"

namespace ver {

typedef unsigned short bf16_t;  // storage type of a bf16 value
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned short u16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16_t to_bf16(float f) {  // round to nearest even
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float from_bf16(bf16_t h) { return __uint_as_float(((unsigned int)h) << 16); }

__device__ __forceinline__ f32x4_t mfma_bf16_16x16x32(u16x8_t a, u16x8_t b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                   c, 0, 0, 0);
}
__device__ __forceinline__ f32x4_t mfma_f32_16x16x4(float a, float b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

enum { MODE_F32 = 0, MODE_BF16 = 1 };

template <int MODE> struct LdsElem;
template <> struct LdsElem<MODE_F32> { typedef float type; };
template <> struct LdsElem<MODE_BF16> { typedef bf16_t type; };

template <typename TO> __device__ __forceinline__ TO cvt_elem(float v);
template <> __device__ __forceinline__ float cvt_elem<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t cvt_elem<bf16_t>(float v) { return to_bf16(v); }
template <typename TO> __device__ __forceinline__ TO cvt_elem(bf16_t v);
template <> __device__ __forceinline__ float cvt_elem<float>(bf16_t v) { return from_bf16(v); }
template <> __device__ __forceinline__ bf16_t cvt_elem<bf16_t>(bf16_t v) { return v; }

// 4 consecutive elements (aligned to 4 elements) of a source row, converted to the LDS element type.
template <typename E> struct Quad { E v[4]; };
template <typename E, typename T> __device__ __forceinline__ Quad<E> load_quad(const T* p);
template <> __device__ __forceinline__ Quad<float> load_quad<float, float>(const float* p) {
    const f32x4_t t = *reinterpret_cast<const f32x4_t*>(p);
    return Quad<float>{{t[0], t[1], t[2], t[3]}};
}
template <> __device__ __forceinline__ Quad<bf16_t> load_quad<bf16_t, float>(const float* p) {
    const f32x4_t t = *reinterpret_cast<const f32x4_t*>(p);
    return Quad<bf16_t>{{to_bf16(t[0]), to_bf16(t[1]), to_bf16(t[2]), to_bf16(t[3])}};
}
template <> __device__ __forceinline__ Quad<bf16_t> load_quad<bf16_t, bf16_t>(const bf16_t* p) {
    const u16x4_t t = *reinterpret_cast<const u16x4_t*>(p);
    return Quad<bf16_t>{{t[0], t[1], t[2], t[3]}};
}
template <> __device__ __forceinline__ Quad<float> load_quad<float, bf16_t>(const bf16_t* p) {
    const u16x4_t t = *reinterpret_cast<const u16x4_t*>(p);
    return Quad<float>{{from_bf16(t[0]), from_bf16(t[1]), from_bf16(t[2]), from_bf16(t[3])}};
}
template <typename E> __device__ __forceinline__ Quad<E> zero_quad() {
    Quad<E> q;
    q.v[0] = q.v[1] = q.v[2] = q.v[3] = E(0);
    return q;
}
// One aligned store of 4 consecutive LDS elements (8 bytes bf16, 16 bytes fp32).
__device__ __forceinline__ void store_quad(bf16_t* dst, const Quad<bf16_t>& q) {
    u16x4_t t;
    t[0] = q.v[0]; t[1] = q.v[1]; t[2] = q.v[2]; t[3] = q.v[3];
    *reinterpret_cast<u16x4_t*>(dst) = t;
}
__device__ __forceinline__ void store_quad(float* dst, const Quad<float>& q) {
    *reinterpret_cast<f32x4_t*>(dst) = f32x4_t{q.v[0], q.v[1], q.v[2], q.v[3]};
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;

constexpr int GEMM_BM = 128, GEMM_BN = 128, GEMM_THREADS = 256;

// Which tile a workgroup computes.  Workgroups are dealt to the 8 XCDs round-robin in launch order and every
// XCD has its own 4 MB L2, so the workgroups of one XCD are given a band of row tiles (with all its column tiles
// and K-splits), and inside the band the ~64 workgroups that are resident at a time form an 8 x 8 block of
// tiles: the operand tiles they share are then fetched from HBM once per block instead of once per workgroup.
// bx: column tile, by: row tile, bz: K-split.
__device__ __forceinline__ void gemm_tile_of_block(int& bx, int& by, int& bz) {
    const int gx = gridDim.x, gy = gridDim.y, gz = gridDim.z;
    const int id = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
    if (gy % 8 != 0) {   // no even bands: launch order as it is
        bx = blockIdx.x; by = blockIdx.y; bz = blockIdx.z;
        return;
    }
    const int R = gy / 8;                       // row tiles of a band
    const int xcd = id % 8, slot = id / 8;      // slot: 0 .. R*gx*gz - 1 in launch order on this XCD
    bz = slot / (R * gx);
    const int rem = slot - bz * (R * gx);
    const int Rb = R % 8 == 0 ? 8 : R, Cb = gx % 8 == 0 ? 8 : gx;   // block of tiles that is resident together
    const int blk = rem / (Rb * Cb), in = rem - blk * (Rb * Cb);
    const int blocks_x = gx / Cb;
    by = xcd * R + (blk / blocks_x) * Rb + in / Cb;
    bx = (blk % blocks_x) * Cb + in % Cb;
}

template <int MODE> struct GemmGeom;
template <> struct GemmGeom<MODE_BF16> { static constexpr int BK = 64, LDS_STRIDE = 72; };
template <> struct GemmGeom<MODE_F32> { static constexpr int BK = 32, LDS_STRIDE = 36; };

// One operand tile (128 rows x BK) on its way from global memory to LDS, held in registers as
// QUADS 4-element groups per thread.
template <int MODE> struct TileRegs {
    typedef typename LdsElem<MODE>::type E;
    static constexpr int QUADS = 128 * GemmGeom<MODE>::BK / 4 / GEMM_THREADS;
    Quad<E> q[QUADS];
};

// K-major source: quad c (of BK/4) of row r; 16-byte (fp32) or 8-byte (bf16) coalesced loads.
// K-minor source: each thread owns 4(k) x 4(rows) blocks, loaded as 4 row-quads and transposed.
template <int MODE, typename T, bool TRANS>
__device__ __forceinline__ void tile_load(const T* __restrict__ src, int ld, int row0, int n_rows, int k0, int k_end,
                                          TileRegs<MODE>& regs) {
    typedef typename LdsElem<MODE>::type E;
    constexpr int BK = GemmGeom<MODE>::BK, QUADS = TileRegs<MODE>::QUADS;
    const int tid = threadIdx.x;
    if (!TRANS) {
        constexpr int CPR = BK / 4;                      // quads per row
        constexpr int RPP = GEMM_THREADS / CPR;          // rows per pass
        const int c = tid % CPR, r = tid / CPR;
#pragma unroll
        for (int i = 0; i < QUADS; ++i) {
            const int gr = row0 + r + i * RPP, gk = k0 + c * 4;
            regs.q[i] = (gr < n_rows && gk < k_end) ? load_quad<E, T>(src + (size_t)gr * ld + gk) : zero_quad<E>();
        }
    } else {
        constexpr int MB = 128 / 4;                      // 4-row blocks across the tile
        constexpr int KPP = GEMM_THREADS / MB;           // 4-k blocks per pass
        const int mb = tid % MB, kb = tid / MB;
#pragma unroll
        for (int i = 0; i < QUADS / 4; ++i) {
            const int gk = k0 + (kb + i * KPP) * 4, gr = row0 + mb * 4;
            Quad<E> in[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                in[j] = (gk + j < k_end && gr < n_rows) ? load_quad<E, T>(src + (size_t)(gk + j) * ld + gr) : zero_quad<E>();
#pragma unroll
            for (int m = 0; m < 4; ++m)                  // row gr+m gets k = gk .. gk+3
#pragma unroll
                for (int j = 0; j < 4; ++j) regs.q[i * 4 + m].v[j] = in[j].v[m];
        }
    }
}

template <int MODE, bool TRANS>
__device__ __forceinline__ void tile_store(const TileRegs<MODE>& regs, typename LdsElem<MODE>::type* __restrict__ lds) {
    constexpr int BK = GemmGeom<MODE>::BK, STRIDE = GemmGeom<MODE>::LDS_STRIDE, QUADS = TileRegs<MODE>::QUADS;
    const int tid = threadIdx.x;
    if (!TRANS) {
        constexpr int CPR = BK / 4, RPP = GEMM_THREADS / CPR;
        const int c = tid % CPR, r = tid / CPR;
#pragma unroll
        for (int i = 0; i < QUADS; ++i) store_quad(lds + (r + i * RPP) * STRIDE + c * 4, regs.q[i]);
    } else {
        constexpr int MB = 128 / 4, KPP = GEMM_THREADS / MB;
        const int mb = tid % MB, kb = tid / MB;
#pragma unroll
        for (int i = 0; i < QUADS / 4; ++i)
#pragma unroll
            for (int m = 0; m < 4; ++m)
                store_quad(lds + (mb * 4 + m) * STRIDE + (kb + i * KPP) * 4, regs.q[i * 4 + m]);
    }
}

// unperm_h > 0: output row m is stored at row (m % 4) * unperm_h + m / 4 (gate-interleaved -> gate-major).
// gridDim.z > 1: block z contracts k in [z*k_chunk, (z+1)*k_chunk) and writes its partial tile to
// C + z*split_stride without bias and without the row permutation (gemm_reduce_kernel applies both).
template <int MODE, typename TA, typename TB, bool TRANS>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(
    const TA* __restrict__ A, int lda, const TB* __restrict__ B, int ldb, float* __restrict__ C, int ldc,
    int Mr, int Nc, int K, const float* __restrict__ bias, int unperm_h, int k_chunk, size_t split_stride) {
    typedef typename LdsElem<MODE>::type E;
    constexpr int BK = GemmGeom<MODE>::BK, STRIDE = GemmGeom<MODE>::LDS_STRIDE;
    __shared__ __attribute__((aligned(16))) E sA[GEMM_BM * STRIDE];
    __shared__ __attribute__((aligned(16))) E sB[GEMM_BN * STRIDE];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    int bx, by, bz;
    gemm_tile_of_block(bx, by, bz);
    const int m0 = by * GEMM_BM, n0 = bx * GEMM_BN;
    const int lr = lane & 15, lk = lane >> 4;
    const int k_begin = bz * k_chunk, k_end = min(K, k_begin + k_chunk);
    const bool split = gridDim.z > 1;
    if (split) C += (size_t)bz * split_stride;

    f32x4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    TileRegs<MODE> ra, rb;
    tile_load<MODE, TA, TRANS>(A, lda, m0, Mr, k_begin, k_end, ra);
    tile_load<MODE, TB, TRANS>(B, ldb, n0, Nc, k_begin, k_end, rb);
    for (int k0 = k_begin; k0 < k_end; k0 += BK) {
        tile_store<MODE, TRANS>(ra, sA);
        tile_store<MODE, TRANS>(rb, sB);
        __syncthreads();
        if (k0 + BK < k_end) {   // next K-tile: in flight while this one is multiplied
            tile_load<MODE, TA, TRANS>(A, lda, m0, Mr, k0 + BK, k_end, ra);
            tile_load<MODE, TB, TRANS>(B, ldb, n0, Nc, k0 + BK, k_end, rb);
        }
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
                // a lane takes 4 consecutive k of its row in one 16-byte read and feeds them to 4 MFMAs; which
                // k a lane contributes is free as long as A and B agree
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
        __syncthreads();
    }
    // C fragment: element r of lane l is row (l / 16) * 4 + r, column l % 16 of the 16x16 tile.
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + wn + j * 16 + lr;
            if (n >= Nc) continue;
            const float bv = (bias && !split) ? bias[n] : 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = m0 + wm + i * 16 + lk * 4 + r;
                if (m >= Mr) continue;
                const int out_row = (unperm_h > 0 && !split) ? (m & 3) * unperm_h + (m >> 2) : m;
                C[(size_t)out_row * ldc + n] = acc[i][j][r] + bv;
            }
        }
}

// C[perm(m)][n] = sum_z part[z][m][n] (+ bias[n]), z ascending.
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const float* __restrict__ part, int splits, size_t split_stride,
                                                          int Mr, int Nc, float* __restrict__ C, int ldc,
                                                          const float* __restrict__ bias, int unperm_h) {
    const size_t total = (size_t)Mr * Nc;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int m = (int)(i / Nc), n = (int)(i % Nc);
        float s = 0.f;
        for (int z = 0; z < splits; ++z) s += part[(size_t)z * split_stride + i];
        if (bias) s += bias[n];
        const int out_row = unperm_h > 0 ? (m & 3) * unperm_h + (m >> 2) : m;
        C[(size_t)out_row * ldc + n] = s;
    }
}

// ---- K-minor bf16 operands through LDS-direct loads --------------------------------------------------------
// C[m][n] = sum_k A[k*lda + m] * B[k*ldb + n] (weight gradients: the contraction runs over the packed rows).
// Tiles of 32 k-rows go from global memory straight into LDS, four stages deep (three tiles in flight while
// one is multiplied, one barrier per tile); the MFMA operands are read with the transposing LDS load
// (ds_read_b64_tr_b16): in every group of 16 lanes, lane i supplies the address of 4 consecutive elements of
// row k = i/4 (columns 4*(i%4)..+3 of a 16-column tile) and receives, for column i, the 4 values of rows
// 0..3 - measured layout: result[j] of lane l = element l%4 of source lane l/4 + 4j.
// An LDS row holds the 128 columns of one k as 16 chunks of 16 bytes; chunk position p of row k holds chunk
// p ^ swz(k), swz(k) = 2*(k&3) | 8*((k>>3)&1), so that the 32 lanes served together (rows k..k+3 and k+8..k+11,
// two chunks each) touch every bank once.  A load instruction fills 4 rows (lane -> row lane/16, position
// lane%16): the swizzle is applied on the global side.
constexpr int TN_BK = 32;
// WM: 16-row tiles per wave along m (wave tile 16*WM x 64, workgroup tile 32*WM x 128).  WM = 8 halves the LDS
// bytes read per MFMA (the limit of the 64 x 64 wave tile) at the price of one stage less in flight.
template <int WM> struct TnGeom {
    static constexpr int BM = 32 * WM, ROW_A = BM * 2, STAGE = TN_BK * (ROW_A + 256), STAGES = WM == 8 ? 3 : 4;
    static constexpr int NA = TN_BK * ROW_A / 1024 / 4;   // A load instructions per wave and stage
    static constexpr int LDS = STAGES * STAGE;
};
#ifndef VER_TN_TARGET_WGS
#define VER_TN_TARGET_WGS 256
#endif
constexpr int TN_TARGET_WGS = VER_TN_TARGET_WGS;
typedef short s16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int tn_swz(int k) { return ((k & 3) << 1) | (((k >> 3) & 1) << 3); }

// XTRA: the output has a few columns (x_cols <= 32) beyond its last whole column tile, [Nc - x_cols, Nc).  Instead of
// a column tile of their own they ride along with the whole tiles of the same row tile, which have the A operand
// in LDS anyway: column tile bx < 2 * WM / x_mt also multiplies the 16-row tiles bx * x_mt .. + x_mt - 1 of its rows
// with those columns (32 more columns of B per stage, two to four more MFMAs per K-tile in one wave).
constexpr int TN_X_STAGE = TN_BK * 64;   // bytes per stage: 32 k-rows of 32 columns
template <int WM, bool XTRA = false>
__device__ __forceinline__ void gemm_tn_dma_body(
    const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ B, int ldb, float* __restrict__ C, int ldc,
    int Mr, int Nc, int K, int unperm_h, int k_chunk, size_t split_stride, unsigned char* smem, int bx, int by, int bz,
    bool split, int x_cols = 0, int x_mt = 0) {
    typedef TnGeom<WM> G;
    constexpr int TN_STAGES = G::STAGES, TN_STAGE_BYTES = G::STAGE + (XTRA ? TN_X_STAGE : 0), ROW_A = G::ROW_A, NA = G::NA;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave >> 1) * 16 * WM, wn = (wave & 1) * 64;
    const int m0 = by * G::BM, n0 = bx * GEMM_BN;
    const int lr = lane & 15, lk = lane >> 4;
    const int k_begin = bz * k_chunk, k_end = min(K, k_begin + k_chunk);
    const int nk = (k_end - k_begin + TN_BK - 1) / TN_BK;
    if (split) C += (size_t)bz * split_stride;
    // rows beyond K read zero (buffer bounds); columns beyond the matrix only feed outputs that are not stored
    __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(A), 0, (int)min((size_t)K * lda * 2, (size_t)0x7fffffff), 0x00020000);
    __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(B), 0, (int)min((size_t)K * ldb * 2, (size_t)0x7fffffff), 0x00020000);
    // this lane's part of the NA + 2 load instructions of its wave per stage (an instruction fills 1 KB of LDS:
    // 1024 / ROW_A rows of A, 4 rows of B)
    int voffA[NA], voffB[2];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const int k = (wave * NA + j) * (1024 / ROW_A) + lane / (ROW_A / 16), c = (lane % (ROW_A / 16)) ^ tn_swz(k);
        voffA[j] = k * lda * 2 + m0 * 2 + c * 16;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int k = (wave * 2 + j) * 4 + (lane >> 4), c = (lane & 15) ^ tn_swz(k);
        voffB[j] = k * ldb * 2 + n0 * 2 + c * 16;
    }
    // extra columns: half an instruction per wave and stage (lanes 0..31: row wave * 8 + lane / 4, 16-byte chunk
    // lane % 4 of the row's 64 bytes); what lies beyond column Nc belongs to the next row (finite values that only
    // feed outputs which are not stored) or, at the end of the buffer, reads zero
    const bool x_here = XTRA && bx * x_mt < 2 * WM;
    const int x_n0 = Nc - x_cols;                     // first extra column
    const int x_wave = ((bx * x_mt) / WM) << 1;       // the wave whose row tiles those are (column half 0)
    const int voffX = (wave * 8 + ((lane & 31) >> 2)) * ldb * 2 + x_n0 * 2 + (lane & 3) * 16;
    auto issue = [&](int kt) {
        unsigned char* st = smem + (kt % TN_STAGES) * TN_STAGE_BYTES;
        const int k0 = k_begin + kt * TN_BK;
        // the row goes into the per-lane offset: only that one is checked against the buffer bounds
#pragma unroll
        for (int j = 0; j < NA; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (lds_ptr_t)(st + (wave * NA + j) * 1024), 16, voffA[j] + k0 * lda * 2, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 2; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (lds_ptr_t)(st + TN_BK * ROW_A + (wave * 2 + j) * 1024), 16,
                                                     voffB[j] + k0 * ldb * 2, 0, 0, 0);
        if (XTRA && lane < 32)   // (every wave issues it, so the counts of loads in flight below hold for all of them)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (lds_ptr_t)(st + G::STAGE + wave * 512), 16, voffX + k0 * ldb * 2, 0, 0, 0);
    };
    // operand read offsets: source row k = lk*8 + lr/4 (+4 for the second half), columns tile*16 + 4*(lr%4)..+3
    int offA[WM][2], offB[4][2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int k = lk * 8 + (lr >> 2) + 4 * h;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int colA = wm + i * 16 + 4 * (lr & 3);
            offA[i][h] = k * ROW_A + ((((colA * 2) >> 4) ^ tn_swz(k)) << 4) + ((colA * 2) & 8);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int colB = wn + i * 16 + 4 * (lr & 3);
            offB[i][h] = TN_BK * ROW_A + k * 256 + ((((colB * 2) >> 4) ^ tn_swz(k)) << 4) + ((colB * 2) & 8);
        }
    }
    int offAx[2][2], offBx[2][2];
    f32x4_t accx[2][2];
    if (XTRA) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int k = lk * 8 + (lr >> 2) + 4 * h;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int colA = ((bx * x_mt + i) & (2 * WM - 1)) * 16 + 4 * (lr & 3), colB = i * 16 + 4 * (lr & 3);
                offAx[i][h] = k * ROW_A + ((((colA * 2) >> 4) ^ tn_swz(k)) << 4) + ((colA * 2) & 8);
                offBx[i][h] = G::STAGE + k * 64 + colB * 2;
                accx[i][h] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            }
        }
    }
    f32x4_t acc[WM][4];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    for (int kt = 0; kt < TN_STAGES - 1 && kt < nk; ++kt) issue(kt);
    for (int kt = 0; kt < nk; ++kt) {
        // this wave's NA + 2 loads of stage kt have landed; up to STAGES - 2 younger stages may be in flight
        const int younger = min(nk - 1 - kt, TN_STAGES - 2);
        if (WM == 8) {
            if (younger >= 1 && XTRA) asm volatile("s_waitcnt vmcnt(7)" ::: "memory");
            else if (younger >= 1) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else if (XTRA) {   // 7 loads per wave and stage
            if (younger >= 2) asm volatile("s_waitcnt vmcnt(14)" ::: "memory");
            else if (younger == 1) asm volatile("s_waitcnt vmcnt(7)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else {
            if (younger >= 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            else if (younger == 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        bar_lds();   // everyone's loads of stage kt have landed, and everyone is done reading stage kt-1
        if (kt + TN_STAGES - 1 < nk) issue(kt + TN_STAGES - 1);
        const unsigned char* st = smem + (kt % TN_STAGES) * TN_STAGE_BYTES;
        u16x8_t a[WM], b[4];
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(st + offA[i][0]));
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(st + offA[i][1]));
            a[i] = u16x8_t{(bf16_t)lo[0], (bf16_t)lo[1], (bf16_t)lo[2], (bf16_t)lo[3], (bf16_t)hi[0], (bf16_t)hi[1], (bf16_t)hi[2], (bf16_t)hi[3]};
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(st + offB[j][0]));
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(st + offB[j][1]));
            b[j] = u16x8_t{(bf16_t)lo[0], (bf16_t)lo[1], (bf16_t)lo[2], (bf16_t)lo[3], (bf16_t)hi[0], (bf16_t)hi[1], (bf16_t)hi[2], (bf16_t)hi[3]};
        }
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = mfma_bf16_16x16x32(a[i], b[j], acc[i][j]);
        if (XTRA && x_here && wave == x_wave) {
            u16x8_t bxr[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(st + offBx[j][0]));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(st + offBx[j][1]));
                bxr[j] = u16x8_t{(bf16_t)lo[0], (bf16_t)lo[1], (bf16_t)lo[2], (bf16_t)lo[3], (bf16_t)hi[0], (bf16_t)hi[1], (bf16_t)hi[2], (bf16_t)hi[3]};
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                if (i >= x_mt) break;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(st + offAx[i][0]));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(st + offAx[i][1]));
                const u16x8_t ax = u16x8_t{(bf16_t)lo[0], (bf16_t)lo[1], (bf16_t)lo[2], (bf16_t)lo[3], (bf16_t)hi[0], (bf16_t)hi[1], (bf16_t)hi[2], (bf16_t)hi[3]};
#pragma unroll
                for (int j = 0; j < 2; ++j) accx[i][j] = mfma_bf16_16x16x32(ax, bxr[j], accx[i][j]);
            }
        }
    }
    if (XTRA && x_here && wave == x_wave) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (i >= x_mt) break;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = x_n0 + j * 16 + lr;
                if (n >= Nc) continue;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = m0 + (bx * x_mt + i) * 16 + lk * 4 + r;
                    if (m >= Mr) continue;
                    const int out_row = unperm_h > 0 ? (m & 3) * unperm_h + (m >> 2) : m;
                    C[(size_t)out_row * ldc + n] = accx[i][j][r];
                }
            }
        }
    }
    // C fragment: element r of lane l is row (l / 16) * 4 + r, column l % 16 of the 16x16 tile.
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + wn + j * 16 + lr;
            if (n >= Nc) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = m0 + wm + i * 16 + lk * 4 + r;
                if (m >= Mr) continue;
                const int out_row = (unperm_h > 0 && !split) ? (m & 3) * unperm_h + (m >> 2) : m;
                C[(size_t)out_row * ldc + n] = acc[i][j][r];
            }
        }
}

// (plain kernels around the template body: the transposing-load builtin only exists in the device pass)
__global__ __launch_bounds__(GEMM_THREADS) void gemm_tn_dma_kernel(
    const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ B, int ldb, float* __restrict__ C, int ldc,
    int Mr, int Nc, int K, int unperm_h, int k_chunk, size_t split_stride) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int bx, by, bz;
    gemm_tile_of_block(bx, by, bz);
    gemm_tn_dma_body<4>(A, lda, B, ldb, C, ldc, Mr, Nc, K, unperm_h, k_chunk, split_stride, smem, bx, by, bz, gridDim.z > 1);
}
__global__ __launch_bounds__(GEMM_THREADS) void gemm_tn_dma_tall_kernel(
    const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ B, int ldb, float* __restrict__ C, int ldc,
    int Mr, int Nc, int K, int unperm_h, int k_chunk, size_t split_stride) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int bx, by, bz;
    gemm_tile_of_block(bx, by, bz);
    gemm_tn_dma_body<8>(A, lda, B, ldb, C, ldc, Mr, Nc, K, unperm_h, k_chunk, split_stride, smem, bx, by, bz, gridDim.z > 1);
}

// Several such contractions in one launch (the weight gradients of a minibatch: same row count, different
// operands).  One launch of all their tiles lets two workgroups share a CU, so that one multiplies while the
// other waits at its stage barrier, and the ramps and tails of the separate launches are gone.
// The tiles are dealt to the 8 XCDs (workgroups go to them round-robin in launch order) for reuse in their L2s:
// problems with the same A operand form a set whose column tiles lie side by side; an XCD takes a band of row tiles
// of every set, a row tile's column tiles next to each other (counters: 79 % of the L2 requests hit).  Slots s and
// s + 32 of an XCD (the two workgroups that end up on one CU when 64 are resident per XCD) take neighbouring column
// tiles of one row tile: the second one finds the A rows in the CU's own cache (-4 %).
constexpr int TN_GROUP_MAX = 4;
struct TnProblem {
    const bf16_t* A; const bf16_t* B; float* C;
    int lda, ldb, ldc, Mr, Nc, K, unperm_h;
    int tiles_n;               // column tiles
    int x_cols, x_mt;          // columns beyond the last whole column tile that ride along with the whole tiles (0: none)
    int xcd_first, xcd_count;  // the XCDs that work on this problem's set
    int band;                  // row tiles per XCD
    int col_first, cols_set;   // this problem's first column tile among the cols_set of its set
    int slot_first;            // first slot of the set on its XCDs
};
struct TnGroupArgs { TnProblem p[TN_GROUP_MAX]; int n; int slots; };
template <int WM>
__device__ __forceinline__ void gemm_tn_dma_group_body(const TnGroupArgs g, unsigned char* smem) {
#if defined(__HIP_DEVICE_COMPILE__)   // (the transposing-load builtin of the tile body only exists in the device pass)
    const int xcd = blockIdx.x % 8;
    int slot = blockIdx.x / 8;
    if (g.slots % 64 == 0) slot = (slot & ~63) | ((slot & 31) << 1) | ((slot >> 5) & 1);
    int pi = -1, by = 0, bx = 0;
#pragma unroll
    for (int i = 0; i < TN_GROUP_MAX; ++i) {   // (constant indices only: the arguments are read in place)
        const int rel = slot - g.p[i].slot_first, x = xcd - g.p[i].xcd_first, cs = g.p[i].cols_set > 0 ? g.p[i].cols_set : 1;
        const int col = rel % cs - g.p[i].col_first;
        const bool mine = i < g.n && x >= 0 && x < g.p[i].xcd_count && rel >= 0 && rel < g.p[i].band * cs && col >= 0 && col < g.p[i].tiles_n;
        if (mine) { pi = i; by = x * g.p[i].band + rel / cs; bx = col; }
    }
    if (pi < 0) return;   // (uniform: an XCD whose sets have fewer tiles than another's)
    TnProblem q = g.p[0];   // uniform selects (an indexed copy of a kernel argument would live in scratch memory)
#pragma unroll
    for (int i = 1; i < TN_GROUP_MAX; ++i)
        if (pi == i) q = g.p[i];
    if (q.x_cols > 0)
        gemm_tn_dma_body<WM, true>(q.A, q.lda, q.B, q.ldb, q.C, q.ldc, q.Mr, q.Nc, q.K, q.unperm_h, q.K, 0, smem, bx, by, 0, false,
                                   q.x_cols, q.x_mt);
    else
        gemm_tn_dma_body<WM>(q.A, q.lda, q.B, q.ldb, q.C, q.ldc, q.Mr, q.Nc, q.K, q.unperm_h, q.K, 0, smem, bx, by, 0, false);
#endif
}
__global__ __launch_bounds__(GEMM_THREADS, 2) void gemm_tn_dma_group_kernel(TnGroupArgs g) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    gemm_tn_dma_group_body<4>(g, smem);
}
__global__ __launch_bounds__(GEMM_THREADS, 2) void gemm_tn_dma_group_tall_kernel(TnGroupArgs g) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    gemm_tn_dma_group_body<8>(g, smem);
}

// Whether a K-minor bf16 contraction can join a grouped launch, and the launch itself.
inline bool tn_group_fits(int lda, int ldb, int Mr, int K) {
    return lda % 2 == 0 && ldb % 2 == 0 && Mr % (GEMM_BM * 8) == 0 && (size_t)K * lda * 2 < 0x7fffffff &&
           (size_t)K * ldb * 2 < 0x7fffffff;
}
#ifndef VER_TN_TALL_FROM
#define VER_TN_TALL_FROM 448
#endif
struct TnGroup {
    TnGroupArgs a{};
    bool add(const bf16_t* A, int lda, const bf16_t* B, int ldb, float* C, int ldc, int Mr, int Nc, int K, int unperm_h) {
        if (a.n >= TN_GROUP_MAX || !tn_group_fits(lda, ldb, Mr, K)) return false;
        TnProblem& q = a.p[a.n++];
        q.A = A; q.B = B; q.C = C; q.lda = lda; q.ldb = ldb; q.ldc = ldc; q.Mr = Mr; q.Nc = Nc; q.K = K; q.unperm_h = unperm_h;
        return true;
    }
    // Tiles of `bm` rows: column tiles and extra columns of every problem, sets, XCDs and slots; returns the number
    // of workgroups (0 if some problem has no even bands of such tiles).
    int lay_out(int bm) {
        int set_first[TN_GROUP_MAX], set_n[TN_GROUP_MAX], set_cols[TN_GROUP_MAX], sets = 0;
        for (int i = 0; i < a.n; ++i) {
            TnProblem& q = a.p[i];
            if (q.Mr % (bm * 8) != 0) return 0;
            q.tiles_n = (q.Nc + GEMM_BN - 1) / GEMM_BN;
            q.x_cols = q.x_mt = 0;
            const int whole = q.Nc / GEMM_BN, rest = q.Nc % GEMM_BN, mt = bm / 16;   // mt: 16-row tiles of a workgroup tile
            if (rest > 0 && rest <= 32 && whole * 2 >= mt) {   // the last few columns ride along with the whole tiles
                q.tiles_n = whole;
                q.x_cols = rest;
                q.x_mt = whole >= mt ? 1 : 2;
            }
            // consecutive problems with the same A operand form a set
            if (sets > 0 && a.p[set_first[sets - 1]].A == q.A && a.p[set_first[sets - 1]].Mr == q.Mr) {
                q.col_first = set_cols[sets - 1];
                set_cols[sets - 1] += q.tiles_n;
                ++set_n[sets - 1];
            } else {
                q.col_first = 0;
                set_first[sets] = i; set_n[sets] = 1; set_cols[sets] = q.tiles_n;
                ++sets;
            }
        }
        // the sets one after the other in every XCD's slots (giving each of two sets four XCDs of its own halves what
        // the loads miss in L2, and measured the same)
        int slots = 0;
        for (int k = 0; k < sets; ++k) {
            const int band = a.p[set_first[k]].Mr / (bm * 8);
            for (int i = set_first[k]; i < set_first[k] + set_n[k]; ++i) {
                TnProblem& q = a.p[i];
                q.xcd_first = 0; q.xcd_count = 8; q.band = band; q.cols_set = set_cols[k];
                q.slot_first = slots;
            }
            slots += band * set_cols[k];
        }
        a.slots = slots;
        return 8 * slots;
    }
    void launch(hipStream_t s) {
        if (a.n == 0) return;
        // 256-row tiles (fewer LDS and L2 bytes per MFMA) when they fill two workgroups per CU, else 128-row tiles
        int wgs = lay_out(256);
        if (wgs >= VER_TN_TALL_FROM) {
            constexpr int lds = TnGeom<8>::LDS + TnGeom<8>::STAGES * TN_X_STAGE;
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_tn_dma_group_tall_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            hipLaunchKernelGGL(gemm_tn_dma_group_tall_kernel, dim3(wgs), dim3(GEMM_THREADS), lds, s, a);
        } else {
            wgs = lay_out(128);
            constexpr int lds = TnGeom<4>::LDS + TnGeom<4>::STAGES * TN_X_STAGE;
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_tn_dma_group_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            hipLaunchKernelGGL(gemm_tn_dma_group_kernel, dim3(wgs), dim3(GEMM_THREADS), lds, s, a);
        }
        a.n = 0;
    }
};

// How many ways to split the contraction so that the grid has a few workgroups per CU.
inline int gemm_splits(int Mr, int Nc, int K, int BK) {
    const long tiles = (long)((Mr + GEMM_BM - 1) / GEMM_BM) * ((Nc + GEMM_BN - 1) / GEMM_BN);
    int s = (int)((768 + tiles - 1) / tiles);
    const int max_s = K / (4 * BK) > 0 ? K / (4 * BK) : 1;   // at least 4 K-tiles per split
    if (s > max_s) s = max_s;
    if (s > 8) s = 8;
    return s < 1 ? 1 : s;
}
inline size_t gemm_part_floats(int Mr, int Nc, int K, int BK) {
    const int s = gemm_splits(Mr, Nc, K, BK);
    return s > 1 ? (size_t)s * Mr * Nc : 0;
}

// part: scratch of gemm_part_floats(...) floats (may be NULL when that is 0 or allow_split is false).
template <int MODE, typename TA, typename TB, bool TRANS>
inline void gemm_launch(const TA* A, int lda, const TB* B, int ldb, float* C, int ldc, int Mr, int Nc, int K,
                        const float* bias, int unperm_h, float* part, bool allow_split, hipStream_t s) {
    constexpr int BK = GemmGeom<MODE>::BK;
    const int splits = (allow_split && part) ? gemm_splits(Mr, Nc, K, BK) : 1;
    dim3 grid((Nc + GEMM_BN - 1) / GEMM_BN, (Mr + GEMM_BM - 1) / GEMM_BM, splits);
    if constexpr (TRANS && MODE == MODE_BF16 && sizeof(TA) == 2 && sizeof(TB) == 2) {
        // both operands bf16 and K-minor: the LDS-direct kernel (bias is never used with these shapes)
        if (!bias && lda % 2 == 0 && ldb % 2 == 0 && (size_t)K * lda * 2 < 0x7fffffff && (size_t)K * ldb * 2 < 0x7fffffff) {
            // Aim at one workgroup per CU, split as little as possible: measured on the weight gradients of the largest
            // configuration (4096 x 1024 outputs over 8192 rows), 256 tiles of 128 x 128 without any split (5.9 ms per
            // update) beat 128 tiles of 256 x 128 split 4 ways (6.7 ms, a quarter of it the pass that adds the partial
            // tiles) and the same 128 x 128 tiles split 2 or 3 ways (6.5, 7.1 ms); 3 or 5 stages instead of 4: 7.2, 7.5 ms.
            const bool tall = Mr % 256 == 0 && (long)(Mr / 256) * grid.x >= TN_TARGET_WGS;   // 256-row tiles when they alone fill the chip
            if (tall) grid.y = Mr / 256;
            const int tiles = grid.x * grid.y;
            int sp = (allow_split && part) ? (TN_TARGET_WGS + tiles / 2) / tiles : 1;
            const int max_sp = K / (8 * TN_BK) > 0 ? K / (8 * TN_BK) : 1;
            sp = sp < 1 ? 1 : (sp > 8 ? 8 : sp);
            if (sp > max_sp) sp = max_sp;
            if (sp > gemm_splits(Mr, Nc, K, BK)) sp = gemm_splits(Mr, Nc, K, BK);   // the scratch is sized for that many
            grid.z = sp;
            const int splits = sp;
            const int k_chunk = splits == 1 ? K : ((K + splits - 1) / splits + BK - 1) / BK * BK;
            const size_t stride = (size_t)Mr * Nc;
            if (tall) {
                (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_tn_dma_tall_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    TnGeom<8>::LDS);
                hipLaunchKernelGGL(gemm_tn_dma_tall_kernel, grid, dim3(GEMM_THREADS), TnGeom<8>::LDS, s, reinterpret_cast<const bf16_t*>(A),
                                   lda, reinterpret_cast<const bf16_t*>(B), ldb, splits == 1 ? C : part, splits == 1 ? ldc : Nc, Mr, Nc,
                                   K, unperm_h, k_chunk, stride);
            } else {
                (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_tn_dma_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    TnGeom<4>::LDS);
                hipLaunchKernelGGL(gemm_tn_dma_kernel, grid, dim3(GEMM_THREADS), TnGeom<4>::LDS, s, reinterpret_cast<const bf16_t*>(A),
                                   lda, reinterpret_cast<const bf16_t*>(B), ldb, splits == 1 ? C : part, splits == 1 ? ldc : Nc, Mr, Nc,
                                   K, unperm_h, k_chunk, stride);
            }
            if (splits > 1)
                hipLaunchKernelGGL(gemm_reduce_kernel, dim3(1024), dim3(256), 0, s, part, splits, stride, Mr, Nc, C, ldc, bias,
                                   unperm_h);
            return;
        }
    }
    if (splits == 1) {
        hipLaunchKernelGGL((gemm_kernel<MODE, TA, TB, TRANS>), grid, dim3(GEMM_THREADS), 0, s, A, lda, B, ldb, C, ldc, Mr,
                           Nc, K, bias, unperm_h, K, (size_t)0);
        return;
    }
    const int k_chunk = ((K + splits - 1) / splits + BK - 1) / BK * BK;
    const size_t stride = (size_t)Mr * Nc;
    hipLaunchKernelGGL((gemm_kernel<MODE, TA, TB, TRANS>), grid, dim3(GEMM_THREADS), 0, s, A, lda, B, ldb, part, Nc, Mr,
                       Nc, K, bias, unperm_h, k_chunk, stride);
    hipLaunchKernelGGL(gemm_reduce_kernel, dim3(1024), dim3(256), 0, s, part, splits, stride, Mr, Nc, C, ldc, bias,
                       unperm_h);
}

}  // namespace ver
