// FP8 (E4M3) projection GEMM for gfx950: launchers and launch rule of the direct-to-LDS kernel (gemm_dtl_kernel.h)
// with one-byte operands,  c[M,N] = (a8[M,K] * w8[N,K]^T) * sa[M] * sw[N], fp32 accumulate, bf16 output (RNE); and the
// row quantiser that produces a8 / sa (and, once per model, w8 / sw).
// (The paper runs its matrix products in 8 bits, Section 4.1; this is the 8-bit float the CDNA4 matrix cores take.)
// Requires K % 128 == 0, N % 8 == 0 and M*K, N*K < 2^31.
#include "gemm_dtl_kernel.h"

namespace {

constexpr int KE = Fp8Op::KE;          // k elements per slice
constexpr float FP8_MAX = 448.0f;
template <int BM, int BN, int WM, int WN> struct F8Cfg : DtlCfg<BM, BN, WM, WN> {
    static constexpr int LDS_BYTES = DtlCfg<BM, BN, WM, WN>::W3 ? DtlCfg<BM, BN, WM, WN>::LDS_BYTES_W3
                                                                 : DtlCfg<BM, BN, WM, WN>::LDS_BYTES;
};

template <int BM, int BN, int WM, int WN, bool SWIGLU>
hipError_t launch(const void *a, const void *w, const float *sa, const float *sw, void *c, int M, int N, int K,
                  hipStream_t s) {
    using Cfg = F8Cfg<BM, BN, WM, WN>;
    static iso_dev_mask lds_allowed{0};
    auto kern = gemm_fp8_dtl_kernel<BM, BN, WM, WN, SWIGLU, false>;
    if (hipError_t e = iso_allow_lds(reinterpret_cast<const void *>(kern), Cfg::LDS_BYTES, &lds_allowed); e != hipSuccess)
        return e;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    dim3 grid(tiles_m * tiles_n), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, Cfg::LDS_BYTES, s, (const unsigned char *)a, (const unsigned char *)w, sa, sw,
                       (bf16_t *)c, M, N, K, tiles_m, tiles_n, (unsigned char *)nullptr, 0u, (unsigned *)nullptr, 1, 0);
    return hipGetLastError();
}

// stream-K launch of the 256x256 tile: one workgroup per compute unit (shape from the planner shared with bf16)
template <bool SWIGLU>
hipError_t launch_sk(const void *a, const void *w, const float *sa, const float *sw, void *c, int M, int N, int K,
                     iso_sk_ws *sk, hipStream_t s) {
    using Cfg = F8Cfg<256, 256, 4, 2>;
    static iso_dev_mask lds_allowed{0};
    auto kern = gemm_fp8_dtl_kernel<256, 256, 4, 2, SWIGLU, true>;
    if (hipError_t e = iso_allow_lds(reinterpret_cast<const void *>(kern), Cfg::LDS_BYTES, &lds_allowed); e != hipSuccess)
        return e;
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    int TS, G, grouped;
    iso_gemm_sk_plan(M, N, K / KE, sk->num_wg, &TS, &G, &grouped);
    if (++sk->epoch == 0) sk->epoch = 1;   // 0 is what a never-raised flag holds
    dim3 grid(G), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, Cfg::LDS_BYTES, s, (const unsigned char *)a, (const unsigned char *)w, sa, sw,
                       (bf16_t *)c, M, N, K, tiles_m, tiles_n, (unsigned char *)sk->base, sk->epoch, sk->err, TS, grouped);
    return hipGetLastError();
}

// Stream-K from 40 k-slices per team (measured: 1024x8960x6656 at 28 slices per team 80 us against 74 us for one
// tile per workgroup; 4096x14336x8192 and 4096x2560x8192 at 80-224 slices +8-9 %).  The partial tiles are fp32 either
// way, so with twice the bf16 kernel's arithmetic rate their hand-over weighs twice as much.
bool sk_wanted(int M, int N, int K, const iso_sk_ws *sk) {
    if (!sk || !sk->base || sk->num_wg < 8) return false;
    int TS, G, grouped;
    return iso_gemm_sk_plan(M, N, K / KE, sk->num_wg, &TS, &G, &grouped) >= 40 && grouped;
}

// Row quantiser: one workgroup per row.  amax = max|row| (fp32), inv = 448 / amax, code = e4m3(x * inv) with round to
// nearest even, scale = amax / 448 (inv = scale = 1 for an all-zero row).  cols % 8 == 0.
__global__ __launch_bounds__(256) void quant_rows_fp8_kernel(const bf16_t *__restrict__ x, unsigned char *__restrict__ q,
                                                             float *__restrict__ scale, int cols) {
    __shared__ float red[4];
    const bf16_t *xr = x + (size_t)blockIdx.x * cols;
    unsigned char *qr = q + (size_t)blockIdx.x * cols;
    float amax = 0.f;
    for (int c = threadIdx.x * 8; c < cols; c += 256 * 8) {
        const bf16x8_t v = *reinterpret_cast<const bf16x8_t *>(xr + c);
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)v[i]));
    }
    amax = iso_wave_max(amax);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float inv = amax > 0.f ? FP8_MAX / amax : 1.0f;
    if (threadIdx.x == 0) scale[blockIdx.x] = amax > 0.f ? amax / FP8_MAX : 1.0f;
    for (int c = threadIdx.x * 8; c < cols; c += 256 * 8) {
        const bf16x8_t v = *reinterpret_cast<const bf16x8_t *>(xr + c);
        int w0 = 0, w1 = 0;
        // the conversion has no saturation above the format's range; x * inv cannot exceed 448 by more than rounding
        auto f = [&](int i) { return fminf(fmaxf((float)v[i] * inv, -FP8_MAX), FP8_MAX); };
        w0 = __builtin_amdgcn_cvt_pk_fp8_f32(f(0), f(1), w0, false);
        w0 = __builtin_amdgcn_cvt_pk_fp8_f32(f(2), f(3), w0, true);
        w1 = __builtin_amdgcn_cvt_pk_fp8_f32(f(4), f(5), w1, false);
        w1 = __builtin_amdgcn_cvt_pk_fp8_f32(f(6), f(7), w1, true);
        *reinterpret_cast<int2 *>(qr + c) = make_int2(w0, w1);
    }
}

}  // namespace

bool iso_gemm_fp8_supported(int M, int N, int K) {
    return M >= 1 && N >= 8 && (N % 8) == 0 && K >= KE && (K % KE) == 0 && (long long)M * K < (1ll << 31) &&
           (long long)N * K < (1ll << 31);
}

hipError_t iso_launch_quant_rows_fp8(const void *x, void *q, float *scale, int rows, int cols, hipStream_t s) {
    hipLaunchKernelGGL(quant_rows_fp8_kernel, dim3(rows), dim3(256), 0, s, (const bf16_t *)x, (unsigned char *)q, scale,
                       cols);
    return hipGetLastError();
}

// Stream-K when the planner's rule says so (sk may be null: never); else 256x256 tiles when they yield at least 128
// workgroups, else 128x128 (as the bf16 kernel chooses).
// variant 6 forces the stream-K launch (tests), anything else leaves the choice to the rule.
hipError_t iso_launch_gemm_fp8(const void *a8, const float *sa, const void *w8, const float *sw, void *c, int M, int N,
                               int K, int variant, iso_sk_ws *sk, hipStream_t s) {
    if ((variant & 7) == 6 && !(sk && sk->base)) return hipErrorInvalidValue;
    if ((variant & 7) == 6 || sk_wanted(M, N, K, sk)) return launch_sk<false>(a8, w8, sa, sw, c, M, N, K, sk, s);
    const long long tiles_256 = (long long)((M + 255) / 256) * ((N + 255) / 256);
    if (tiles_256 >= 128) return launch<256, 256, 4, 2, false>(a8, w8, sa, sw, c, M, N, K, s);
    return launch<128, 128, 2, 2, false>(a8, w8, sa, sw, c, M, N, K, s);
}

// act[M, F] = silu(gate) * up with w8 = [gate; up] of shape [2F, K], sw of length 2F
hipError_t iso_launch_gemm_swiglu_fp8(const void *a8, const float *sa, const void *w8, const float *sw, void *act, int M,
                                      int F, int K, int variant, iso_sk_ws *sk, hipStream_t s) {
    if ((variant & 7) == 6 && !(sk && sk->base)) return hipErrorInvalidValue;
    if ((variant & 7) == 6 || sk_wanted(M, 2 * F, K, sk))
        return launch_sk<true>(a8, w8, sa, sw, act, M, 2 * F, K, sk, s);
    const long long tiles_256 = (long long)((M + 255) / 256) * ((2 * F + 255) / 256);
    if (tiles_256 >= 128) return launch<256, 256, 4, 2, true>(a8, w8, sa, sw, act, M, 2 * F, K, s);
    return launch<128, 128, 2, 2, true>(a8, w8, sa, sw, act, M, 2 * F, K, s);
}
