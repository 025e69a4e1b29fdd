// Chunk attention over the KV cache, one wavefront per (query row, query head): online softmax over
// 64-key slices, fp32 throughout.  This is the fp32 path of the small workload and the fallback for
// shapes the MFMA kernel does not take.  (Chunk over the cache written by the earlier chunk: paper
// Section 3.1; chunked prefill, Section 2.1.)
#include "iso_internal.h"

namespace {

template <typename T> __device__ __forceinline__ float exp_f(float z);
template <> __device__ __forceinline__ float exp_f<float>(float z) { return expf(z); }
template <> __device__ __forceinline__ float exp_f<bf16_t>(float z) { return __expf(z); }

// D = head_dim (64 or 128).  Lane l owns output dims l, l+64 (D = 128) or l (D = 64).
template <typename T, int D>
__global__ __launch_bounds__(256) void attn_simple_kernel(const T *__restrict__ q, const T *__restrict__ kc,
                                                          const T *__restrict__ vc, T *__restrict__ out, int Tc,
                                                          int q_offset, int kv_len, int nq, int nkv, int q_stride) {
    __shared__ float qs[4][D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + wave;       // local query row
    const int h = blockIdx.y;
    const bool active = i < Tc;
    const int g = h / (nq / nkv);
    const float scale = 1.0f / sqrtf((float)D);
    if (active) {
        for (int e = lane; e < D; e += 64) qs[wave][e] = iso_to_f32(q[(size_t)i * q_stride + (size_t)h * D + e]) * scale;
    }
    __syncthreads();
    if (!active) return;
    int n_vis = q_offset + i + 1;
    if (n_vis > kv_len) n_vis = kv_len;
    constexpr int PER = D / 64;
    float o[PER] = {};
    float m = -INFINITY, l = 0.f;
    for (int j0 = 0; j0 < n_vis; j0 += 64) {
        const int j = j0 + lane;
        float sc = -INFINITY;
        if (j < n_vis) {
            const T *kr = kc + ((size_t)j * nkv + g) * D;
            float acc = 0.f;
#pragma unroll 8
            for (int e = 0; e < D; ++e) acc = fmaf(qs[wave][e], iso_to_f32(kr[e]), acc);
            sc = acc;
        }
        const float m_new = fmaxf(m, iso_wave_max(sc));
        const float p = (j < n_vis) ? exp_f<T>(sc - m_new) : 0.f;
        const float alpha = exp_f<T>(m - m_new);     // m = -inf on the first slice gives 0
        l = l * alpha + iso_wave_sum(p);
#pragma unroll
        for (int r = 0; r < PER; ++r) o[r] *= alpha;
        const int cnt = min(64, n_vis - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj, 64);
            const T *vr = vc + ((size_t)(j0 + jj) * nkv + g) * D;
#pragma unroll
            for (int r = 0; r < PER; ++r) o[r] = fmaf(pj, iso_to_f32(vr[lane + 64 * r]), o[r]);
        }
        m = m_new;
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int r = 0; r < PER; ++r) out[((size_t)i * nq + h) * D + lane + 64 * r] = iso_from_f32<T>(o[r] * inv);
}

}  // namespace

hipError_t iso_launch_attn_simple(int dtype, const void *q, const void *k, const void *v, void *out, int Tc,
                                  int q_offset, int kv_len, int nq, int nkv, int d, int q_stride, hipStream_t s) {
    dim3 grid((Tc + 3) / 4, nq), block(256);
#define ISO_ATTN_SIMPLE(TT, DD)                                                                              \
    hipLaunchKernelGGL((attn_simple_kernel<TT, DD>), grid, block, 0, s, (const TT *)q, (const TT *)k,        \
                       (const TT *)v, (TT *)out, Tc, q_offset, kv_len, nq, nkv, q_stride)
    if (dtype == ISO_F32 && d == 64) ISO_ATTN_SIMPLE(float, 64);
    else if (dtype == ISO_F32 && d == 128) ISO_ATTN_SIMPLE(float, 128);
    else if (dtype == ISO_BF16 && d == 64) ISO_ATTN_SIMPLE(bf16_t, 64);
    else if (dtype == ISO_BF16 && d == 128) ISO_ATTN_SIMPLE(bf16_t, 128);
    else return hipErrorInvalidValue;
#undef ISO_ATTN_SIMPLE
    return hipGetLastError();
}
