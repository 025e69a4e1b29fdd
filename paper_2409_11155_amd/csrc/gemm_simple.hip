// Portable SIMT tile GEMM  c[M,N] = a[M,K] * w[N,K]^T  with fp32 accumulation, any M, N, K.
// It is the fp32 path of the small workload and the fallback for bf16 shapes the MFMA kernel does not
// take.  (Projections of the layer: paper Section 2.2.)
#include "iso_internal.h"

namespace {

constexpr int TS = 64;   // output tile edge
constexpr int TK = 16;   // k slice

template <typename T>
__global__ __launch_bounds__(256) void gemm_simple_kernel(const T *__restrict__ a, const T *__restrict__ w,
                                                          T *__restrict__ c, int M, int N, int K) {
    __shared__ float as[TK][TS + 1];
    __shared__ float ws[TK][TS + 1];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;       // 16 x 16 threads, 4 x 4 outputs each
    const int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += TK) {
        // 64 rows x 16 k = 1024 elements per operand, 4 per thread
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + i * 256;
            const int r = e / TK, kk = e % TK;
            const int gk = k0 + kk;
            const int gm = m0 + r, gn = n0 + r;
            as[kk][r] = (gm < M && gk < K) ? iso_to_f32(a[(size_t)gm * K + gk]) : 0.f;
            ws[kk][r] = (gn < N && gk < K) ? iso_to_f32(w[(size_t)gn * K + gk]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            float av[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = as[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) wv[j] = ws[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx * 4 + j;
            if (gn < N) c[(size_t)gm * N + gn] = iso_from_f32<T>(acc[i][j]);
        }
    }
}

}  // namespace

hipError_t iso_launch_gemm_simple(int dtype, const void *a, const void *w, void *c, int M, int N, int K,
                                  hipStream_t s) {
    dim3 grid((N + TS - 1) / TS, (M + TS - 1) / TS), block(256);
    if (dtype == ISO_F32)
        hipLaunchKernelGGL(gemm_simple_kernel<float>, grid, block, 0, s, (const float *)a, (const float *)w,
                           (float *)c, M, N, K);
    else
        hipLaunchKernelGGL(gemm_simple_kernel<bf16_t>, grid, block, 0, s, (const bf16_t *)a, (const bf16_t *)w,
                           (bf16_t *)c, M, N, K);
    return hipGetLastError();
}
