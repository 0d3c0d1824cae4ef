// Plain LDS-tiled FMA GEMM: C[M,N] = A[M,K] * Wt[N,K]^T with fp32 accumulation.
// Serves the fp32 configuration and any shape the MFMA kernel does not take
// (K not a multiple of 64).  64x64 output tile per 256-thread block, 16-deep
// K slices staged through LDS as floats, 4x4 outputs per thread.  Any M, N, K.
#include "ss_device.h"
#include "ss_kernels.h"

namespace SS_NS {
using namespace ssk;

template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T* __restrict__ A, int lda,
                                                           const T* __restrict__ Wt, void* __restrict__ Cv,
                                                           int ldc, const T* __restrict__ R, int M, int N, int K,
                                                           const float* __restrict__ RS) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    // loader mapping: thread -> (row = tid / 4, k = (tid % 4) * 4 .. +3)
    const int lr = threadIdx.x >> 2, lk = (threadIdx.x & 3) * 4;
    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = k0 + lk + j;
            const int am = m0 + lr, bn = n0 + lr;
            As[lk + j][lr] = (am < M && k < K) ? ldf(A + (size_t)am * lda + k) : 0.f;
            Bs[lk + j][lr] = (bn < N && k < K) ? ldf(Wt + (size_t)bn * K + k) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = acc[i][j];
            if (RS) v *= RS[m];
            if (EPI == EPI_RESIDUAL) v += ldf(R + (size_t)m * ldc + n);
            if (EPI == EPI_STORE_F32)
                reinterpret_cast<float*>(Cv)[(size_t)m * ldc + n] = v;
            else
                stf(reinterpret_cast<T*>(Cv) + (size_t)m * ldc + n, v);
        }
    }
}

template <typename T>
static hipError_t launch_generic(const void* A, int lda, const void* Wt, void* C, int ldc, const void* R, int M,
                                 int N, int K, int epi, hipStream_t s, const float* rs) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    if (grid.y > 65535) return hipErrorInvalidValue;
    const T* a = (const T*)A;
    const T* w = (const T*)Wt;
    const T* r = (const T*)R;
    switch (epi) {
        case EPI_STORE: gemm_generic_kernel<T, EPI_STORE><<<grid, 256, 0, s>>>(a, lda, w, C, ldc, r, M, N, K, rs); break;
        case EPI_RESIDUAL:
            if (!R) return hipErrorInvalidValue;
            gemm_generic_kernel<T, EPI_RESIDUAL><<<grid, 256, 0, s>>>(a, lda, w, C, ldc, r, M, N, K, rs);
            break;
        case EPI_STORE_F32: gemm_generic_kernel<T, EPI_STORE_F32><<<grid, 256, 0, s>>>(a, lda, w, C, ldc, r, M, N, K, rs); break;
        default: return hipErrorInvalidValue;   // the fused SwiGLU layout exists only for the MFMA kernel
    }
    return hipGetLastError();
}

hipError_t gemm_mfma_bf16(const void* A, int lda, const void* Wt, void* C, int ldc, const void* R, int M, int N,
                          int K, int epi, hipStream_t s, float* ws, size_t ws_bytes, int max_rounds, const float* rs);
bool gemm_mfma_supported(int M, int N, int K, int lda, int ldc, int epi);

hipError_t gemm_nt(int dt, const void* A, int lda, const void* Wt, void* C, int ldc, const void* R, int M, int N,
                   int K, int epi, bool force_generic, hipStream_t s, float* ws, size_t ws_bytes, int max_rounds,
                   const float* row_scale) {
    if (M <= 0 || N <= 0) return hipSuccess;
    if (K <= 0 || lda < K || !A || !Wt || !C) return hipErrorInvalidValue;
    if (dt == BF16 && !force_generic && gemm_mfma_supported(M, N, K, lda, ldc, epi))
        return gemm_mfma_bf16(A, lda, Wt, C, ldc, R, M, N, K, epi, s, ws, ws_bytes, max_rounds, row_scale);
    if (epi == EPI_SWIGLU) return hipErrorInvalidValue;
    if (dt == F32) return launch_generic<float>(A, lda, Wt, C, ldc, R, M, N, K, epi, s, row_scale);
    return launch_generic<bf16_t>(A, lda, Wt, C, ldc, R, M, N, K, epi, s, row_scale);
}

}  // namespace SS_NS
