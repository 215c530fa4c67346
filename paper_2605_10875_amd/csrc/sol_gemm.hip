// GEMMs  C[M][N] = A[M][K] * W[N][K]^T  (both operands K-contiguous).
//   launch_gemm_generic : any shape / dtype, fp32 FMA on LDS tiles, fp32 output. Used for the
//                         fp32 configuration and for shapes the MFMA kernels do not cover.
#include "sol_internal.h"

namespace sol {

constexpr int GT = 64;    // tile M = tile N
constexpr int GK = 16;    // tile K

template <typename TA, typename TW>
__global__ void __launch_bounds__(256)
k_gemm_generic(const TA *__restrict__ A, int64_t lda, const TW *__restrict__ W, int64_t ldw, float *__restrict__ C,
               int64_t ldc, int64_t M, int N, int K)
{
    __shared__ float As[GK][GT + 4];
    __shared__ float Ws[GK][GT + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;          // 16 x 16 threads, 4 x 4 outputs each
    const int64_t m0 = (int64_t)blockIdx.y * GT;
    const int n0 = blockIdx.x * GT;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += GK) {
        // each thread loads 4 elements of A and of W: element (row = tid/4 + 0.., k = (tid%4)*4 ..)
        {
            const int rr = tid >> 2, kk = (tid & 3) * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = k0 + kk + e;
                const int64_t ar = m0 + rr;
                const int wr = n0 + rr;
                As[kk + e][rr] = (ar < M && k < K) ? ld(A + ar * lda + k) : 0.f;
                Ws[kk + e][rr] = (wr < N && k < K) ? ld(W + (int64_t)wr * ldw + k) : 0.f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Ws[k][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t r = m0 + ty * 4 + i;
        if (r >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = n0 + tx * 4 + j;
            if (c < N) C[r * ldc + c] = acc[i][j];
        }
    }
}

void launch_gemm_generic(const void *A, int a_dtype, int64_t lda, const void *W, int w_dtype, int64_t ldw, float *C,
                         int64_t ldc, int64_t M, int N, int K, hipStream_t st)
{
    if (M <= 0 || N <= 0) return;
    const dim3 grid((unsigned)((N + GT - 1) / GT), (unsigned)((M + GT - 1) / GT));
    if (a_dtype == 0 && w_dtype == 0)
        hipLaunchKernelGGL((k_gemm_generic<float, float>), grid, dim3(256), 0, st, (const float *)A, lda,
                           (const float *)W, ldw, C, ldc, M, N, K);
    else if (a_dtype == 1 && w_dtype == 1)
        hipLaunchKernelGGL((k_gemm_generic<bf16_t, bf16_t>), grid, dim3(256), 0, st, (const bf16_t *)A, lda,
                           (const bf16_t *)W, ldw, C, ldc, M, N, K);
}

}  // namespace sol
