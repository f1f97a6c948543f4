// fp32 GEMM for the single fp32 LoRA-adapted linear step (fp32 FMA, fp32 accumulate).
// C[M,N] = alpha * op(A)[M,K] op(B)[K,N] + beta * C.  64x64 tile, 4x4 outputs per thread, BK = 16.
#include "kernels.h"

template <int TA, int TB>
__global__ __launch_bounds__(256) void sgemm_kernel(int M, int N, int K, float alpha, const float* __restrict__ A,
                                                    int lda, const float* __restrict__ B, int ldb, float beta,
                                                    float* __restrict__ C, int ldc) {
    __shared__ float sA[16][65];  // [k][m]
    __shared__ float sB[16][65];  // [k][n]
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int i = tid; i < 64 * 16; i += 256) {
            int m, k;
            if (TA) { m = i & 63; k = i >> 6; } else { k = i & 15; m = i >> 4; }
            float v = 0.f;
            if (m0 + m < M && k0 + k < K) v = TA ? A[(long)(k0 + k) * lda + m0 + m] : A[(long)(m0 + m) * lda + k0 + k];
            sA[k][m] = v;
        }
        for (int i = tid; i < 64 * 16; i += 256) {
            int n, k;
            if (TB) { k = i & 15; n = i >> 4; } else { n = i & 63; k = i >> 6; }
            float v = 0.f;
            if (n0 + n < N && k0 + k < K) v = TB ? B[(long)(n0 + n) * ldb + k0 + k] : B[(long)(k0 + k) * ldb + n0 + n];
            sB[k][n] = v;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = sA[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = sB[k][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) {
                float v = alpha * acc[i][j];
                if (beta != 0.f) v += beta * C[(long)m * ldc + n];
                C[(long)m * ldc + n] = v;
            }
        }
}

hipError_t launch_sgemm(int ta, int tb, int M, int N, int K, float alpha, const float* A, int lda, const float* B,
                        int ldb, float beta, float* C, int ldc, hipStream_t s) {
    if (M <= 0 || N <= 0) return hipSuccess;
    dim3 grid(cdiv(N, 64), cdiv(M, 64));
    if (!ta && !tb) sgemm_kernel<0, 0><<<grid, 256, 0, s>>>(M, N, K, alpha, A, lda, B, ldb, beta, C, ldc);
    else if (!ta && tb) sgemm_kernel<0, 1><<<grid, 256, 0, s>>>(M, N, K, alpha, A, lda, B, ldb, beta, C, ldc);
    else if (ta && !tb) sgemm_kernel<1, 0><<<grid, 256, 0, s>>>(M, N, K, alpha, A, lda, B, ldb, beta, C, ldc);
    else sgemm_kernel<1, 1><<<grid, 256, 0, s>>>(M, N, K, alpha, A, lda, B, ldb, beta, C, ldc);
    return hipGetLastError();
}
