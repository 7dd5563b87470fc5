// LDS-tiled MFMA GEMM for the time-batched contractions of the LSTM
// (input projections, input gradients, weight gradients).  gfx950 only.
//
//   C[m][n] = sum_k A(m,k) * B(n,k)  (+ bias[n])
//
// Operands are "K-major" (A(m,k) = A[m*lda + k]: the contraction index is
// contiguous) or, with TRANS, "K-minor" (A(m,k) = A[k*lda + m]: used for the
// weight gradients, where the contraction runs over the packed rows).  Either
// way a 128x128 tile of C is built by 4 waves (2x2, 64x64 each) from K-tiles
// staged in LDS as [row][k] so that every MFMA operand is one aligned LDS read.
//   MODE_BF16: operands rounded to bf16 on the way into LDS (or already bf16),
//              v_mfma_f32_16x16x32_bf16, fp32 accumulate.
//   MODE_F32 : fp32 operands, v_mfma_f32_16x16x4_f32.
// Results are deterministic (no split-K, no atomics).
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

// Loads 4 consecutive elements (aligned to 4 elements) as floats or raw bf16.
template <typename T> struct Vec4;
template <> struct Vec4<float> {
    float v[4];
    __device__ __forceinline__ void load(const float* p) {
        f32x4_t t = *reinterpret_cast<const f32x4_t*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    __device__ __forceinline__ void zero() { v[0] = v[1] = v[2] = v[3] = 0.f; }
};
template <> struct Vec4<bf16_t> {
    bf16_t v[4];
    __device__ __forceinline__ void load(const bf16_t* p) {
        u16x4_t t = *reinterpret_cast<const u16x4_t*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    __device__ __forceinline__ void zero() { v[0] = v[1] = v[2] = v[3] = 0; }
};

constexpr int GEMM_BM = 128, GEMM_BN = 128, GEMM_THREADS = 256;

template <int MODE> struct GemmGeom;
template <> struct GemmGeom<MODE_BF16> { static constexpr int BK = 32, LDS_STRIDE = 40; };
template <> struct GemmGeom<MODE_F32> { static constexpr int BK = 16, LDS_STRIDE = 20; };

// Stages one operand tile (128 rows x BK) into LDS as [row][k].
template <int MODE, typename T, bool TRANS>
__device__ __forceinline__ void gemm_stage(const T* __restrict__ src, int ld, int row0, int n_rows, int k0, int K,
                                           typename LdsElem<MODE>::type* __restrict__ lds) {
    typedef typename LdsElem<MODE>::type E;
    constexpr int BK = GemmGeom<MODE>::BK, STRIDE = GemmGeom<MODE>::LDS_STRIDE;
    const int tid = threadIdx.x;
    if (!TRANS) {
        constexpr int CHUNKS = BK / 4;                   // 4-element chunks per row
        constexpr int ROWS_PER_PASS = GEMM_THREADS / CHUNKS;
        const int c = tid % CHUNKS, r = tid / CHUNKS;
#pragma unroll
        for (int pass = 0; pass < 128 / ROWS_PER_PASS; ++pass) {
            const int row = r + pass * ROWS_PER_PASS;
            const int gr = row0 + row, gk = k0 + c * 4;
            Vec4<T> v;
            if (gr < n_rows && gk < K) v.load(src + (size_t)gr * ld + gk); else v.zero();
            E* dst = lds + row * STRIDE + c * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[i] = cvt_elem<E>(v.v[i]);
        }
    } else {
        constexpr int CHUNKS = 128 / 4;                  // 4-row chunks per k
        constexpr int K_PER_PASS = GEMM_THREADS / CHUNKS;
        const int c = tid % CHUNKS, kk = tid / CHUNKS;
#pragma unroll
        for (int pass = 0; pass < BK / K_PER_PASS; ++pass) {
            const int k = kk + pass * K_PER_PASS;
            const int gk = k0 + k, gr = row0 + c * 4;
            Vec4<T> v;
            if (gk < K && gr < n_rows) v.load(src + (size_t)gk * ld + gr); else v.zero();
#pragma unroll
            for (int i = 0; i < 4; ++i) lds[(c * 4 + i) * STRIDE + k] = cvt_elem<E>(v.v[i]);
        }
    }
}

// unperm_h > 0: output row m is stored at row (m % 4) * unperm_h + m / 4 (gate-interleaved -> gate-major).
template <int MODE, typename TA, typename TB, bool TRANS>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(
    const TA* __restrict__ A, int lda, const TB* __restrict__ B, int ldb, float* __restrict__ C, int ldc,
    int Mr, int Nc, int K, const float* __restrict__ bias, int unperm_h) {
    typedef typename LdsElem<MODE>::type E;
    constexpr int BK = GemmGeom<MODE>::BK, STRIDE = GemmGeom<MODE>::LDS_STRIDE;
    __shared__ __attribute__((aligned(16))) E sA[GEMM_BM * STRIDE];
    __shared__ __attribute__((aligned(16))) E sB[GEMM_BN * STRIDE];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int m0 = blockIdx.y * GEMM_BM, n0 = blockIdx.x * GEMM_BN;
    const int lr = lane & 15, lk = lane >> 4;

    f32x4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    for (int k0 = 0; k0 < K; k0 += BK) {
        __syncthreads();
        gemm_stage<MODE, TA, TRANS>(A, lda, m0, Mr, k0, K, sA);
        gemm_stage<MODE, TB, TRANS>(B, ldb, n0, Nc, k0, K, sB);
        __syncthreads();
        if (MODE == MODE_BF16) {
            u16x8_t a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                a[i] = *reinterpret_cast<const u16x8_t*>(reinterpret_cast<const bf16_t*>(sA) + (wm + i * 16 + lr) * STRIDE + lk * 8);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                b[j] = *reinterpret_cast<const u16x8_t*>(reinterpret_cast<const bf16_t*>(sB) + (wn + j * 16 + lr) * STRIDE + lk * 8);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = mfma_bf16_16x16x32(a[i], b[j], acc[i][j]);
        } else {
#pragma unroll
            for (int ks = 0; ks < BK; ks += 4) {
                float a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = reinterpret_cast<const float*>(sA)[(wm + i * 16 + lr) * STRIDE + ks + lk];
#pragma unroll
                for (int j = 0; j < 4; ++j) b[j] = reinterpret_cast<const float*>(sB)[(wn + j * 16 + lr) * STRIDE + ks + lk];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = mfma_f32_16x16x4(a[i], b[j], acc[i][j]);
            }
        }
    }
    // C fragment: element r of lane l is row (l / 16) * 4 + r, column l % 16 of the 16x16 tile.
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + wn + j * 16 + lr;
            if (n >= Nc) continue;
            const float bv = bias ? bias[n] : 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = m0 + wm + i * 16 + lk * 4 + r;
                if (m >= Mr) continue;
                const int out_row = unperm_h > 0 ? (m & 3) * unperm_h + (m >> 2) : m;
                C[(size_t)out_row * ldc + n] = acc[i][j][r] + bv;
            }
        }
}

template <int MODE, typename TA, typename TB, bool TRANS>
inline void gemm_launch(const TA* A, int lda, const TB* B, int ldb, float* C, int ldc, int Mr, int Nc, int K,
                        const float* bias, int unperm_h, hipStream_t s) {
    dim3 grid((Nc + GEMM_BN - 1) / GEMM_BN, (Mr + GEMM_BM - 1) / GEMM_BM);
    hipLaunchKernelGGL((gemm_kernel<MODE, TA, TB, TRANS>), grid, dim3(GEMM_THREADS), 0, s, A, lda, B, ldb, C, ldc, Mr,
                       Nc, K, bias, unperm_h);
}

}  // namespace ver
