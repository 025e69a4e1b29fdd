// Bandwidth-bound steps of the layer: RMSNorm (optionally fused with the residual add), rotary
// embedding + KV-cache write, SwiGLU.  Each kernel moves every byte once with 16-byte accesses and
// does its arithmetic in fp32.  (Layer structure: paper Section 2.2; KV-cache write before the next
// chunk's attention: Section 3.1.)
#include "iso_internal.h"

namespace {

template <typename T> struct Vec16 {
    static constexpr int N = 16 / sizeof(T);
    T v[N];
};

template <typename T> __device__ __forceinline__ void load16(const T *p, float (&out)[16 / sizeof(T)]) {
    uint4 raw = *reinterpret_cast<const uint4 *>(p);
    const T *e = reinterpret_cast<const T *>(&raw);
#pragma unroll
    for (int i = 0; i < (int)(16 / sizeof(T)); ++i) out[i] = iso_to_f32(e[i]);
}

// The same for data that is read once (token rows): a non-temporal load leaves the L2 to the tiles of the GEMM that
// runs beside this kernel on the other chunk's stream (the residual kernels measure 6-7 % faster with it; the same
// hint on their stores costs 5 %).
template <typename T> __device__ __forceinline__ void load16_stream(const T *p, float (&out)[16 / sizeof(T)]) {
    typedef unsigned u32x4_nt __attribute__((ext_vector_type(4)));
    u32x4_nt raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt *>(p));
    const T *e = reinterpret_cast<const T *>(&raw);
#pragma unroll
    for (int i = 0; i < (int)(16 / sizeof(T)); ++i) out[i] = iso_to_f32(e[i]);
}

template <typename T> __device__ __forceinline__ void store16(T *p, const float (&in)[16 / sizeof(T)]) {
    uint4 raw;
    T *e = reinterpret_cast<T *>(&raw);
#pragma unroll
    for (int i = 0; i < (int)(16 / sizeof(T)); ++i) e[i] = iso_from_f32<T>(in[i]);
    *reinterpret_cast<uint4 *>(p) = raw;
}

// One 256-thread workgroup per token row.  x_new = x (+ delta (+ delta2)), added in that order in fp32; optionally
// written to x_out (which may be x itself); optionally y = x_new * rsqrt(mean(x_new^2) + eps) * g.  The first CACHE
// vectors of each thread stay in registers between the reduction and the scaling, so rows up to 256*CACHE*VEC
// elements are read once.
//
// NDELTA = 2 is how a bf16 layer keeps its mid-layer residual unrounded without storing it: the MLP block's norm
// computes x1 = x + (attention partial) in registers and writes only y, and the kernel that closes the layer
// rebuilds the same fp32 x1 from the same two bf16 tensors before it adds the MLP partial (paper Section 2.2: the
// two partial sums of a layer) -- 16 instead of 20 bytes per element and layer, same bits as an fp32 side buffer.
//
// Q8 (bf16 rows of at most 256*CACHE*VEC elements only): instead of y the kernel writes the FP8 (E4M3) codes of
// y and one fp32 scale per row, exactly as the row quantiser would from the bf16-rounded y: amax = max|y|,
// code = e4m3(y * (448 / amax)) round to nearest even, scale = amax / 448 (1 for an all-zero row).  The 8-bit
// projections of the layer (paper Section 4.1) then read their activation operand without a separate pass.
template <typename T, int NDELTA, bool WRITE_X, bool WRITE_Y, bool Q8 = false>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const T *x, const T *__restrict__ delta,
                                                      const T *__restrict__ delta2, T *x_out,
                                                      const T *__restrict__ g, T *__restrict__ y, int H, float eps,
                                                      unsigned char *__restrict__ q8 = nullptr,
                                                      float *__restrict__ q_scale = nullptr) {
    static_assert(WRITE_X || WRITE_Y, "nothing to write");
    static_assert(NDELTA > 0 || !WRITE_X, "x is only rewritten when something was added to it");
    constexpr int VEC = 16 / sizeof(T);
    constexpr int CACHE = 4;
    const int tid = threadIdx.x;
    const int nvec = H / VEC;
    const size_t row = (size_t)blockIdx.x * H;
    // x_new of one 16-byte piece, from the inputs
    auto load_new = [&](size_t at, float (&v)[VEC]) {
        load16_stream<T>(x + at, v);
        if (NDELTA >= 1) {
            float dv[VEC];
            load16_stream<T>(delta + at, dv);
#pragma unroll
            for (int i = 0; i < VEC; ++i) v[i] += dv[i];
        }
        if (NDELTA >= 2) {
            float dv[VEC];
            load16_stream<T>(delta2 + at, dv);
#pragma unroll
            for (int i = 0; i < VEC; ++i) v[i] += dv[i];
        }
    };
    float vals[CACHE][VEC];
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < CACHE; ++c) {
        const int idx = tid + c * 256;
        if (idx < nvec) {
            load_new(row + (size_t)idx * VEC, vals[c]);
            if (WRITE_X) store16<T>(x_out + row + (size_t)idx * VEC, vals[c]);
#pragma unroll
            for (int i = 0; i < VEC; ++i) ss += vals[c][i] * vals[c][i];
        }
    }
    for (int idx = tid + CACHE * 256; idx < nvec; idx += 256) {
        float xv[VEC];
        load_new(row + (size_t)idx * VEC, xv);
        if (WRITE_X) store16<T>(x_out + row + (size_t)idx * VEC, xv);
#pragma unroll
        for (int i = 0; i < VEC; ++i) ss += xv[i] * xv[i];
    }
    if (!WRITE_Y) return;

    __shared__ float red[4];
    ss = iso_wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float total = red[0] + red[1] + red[2] + red[3];
    const float scale = 1.0f / sqrtf(total / (float)H + eps);

    if constexpr (Q8) {
        static_assert(sizeof(T) == 2, "the fused quantiser takes bf16 rows");
        float amax = 0.f;
#pragma unroll
        for (int c = 0; c < CACHE; ++c) {
            const int idx = tid + c * 256;
            if (idx < nvec) {
                float gv[VEC];
                load16<T>(g + (size_t)idx * VEC, gv);
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    vals[c][i] = iso_to_f32(iso_from_f32<T>(vals[c][i] * scale * gv[i]));   // y as bf16 would hold it
                    amax = fmaxf(amax, fabsf(vals[c][i]));
                }
            }
        }
        __shared__ float redm[4];
        amax = iso_wave_max(amax);
        if ((tid & 63) == 0) redm[tid >> 6] = amax;
        __syncthreads();
        amax = fmaxf(fmaxf(redm[0], redm[1]), fmaxf(redm[2], redm[3]));
        const float inv = amax > 0.f ? 448.0f / amax : 1.0f;
        if (tid == 0) q_scale[blockIdx.x] = amax > 0.f ? amax / 448.0f : 1.0f;
#pragma unroll
        for (int c = 0; c < CACHE; ++c) {
            const int idx = tid + c * 256;
            if (idx < nvec) {
                // the conversion does not saturate; y * inv exceeds 448 by rounding at most
                auto f = [&](int i) { return fminf(fmaxf(vals[c][i] * inv, -448.0f), 448.0f); };
                int w0 = 0, w1 = 0;
                w0 = __builtin_amdgcn_cvt_pk_fp8_f32(f(0), f(1), w0, false);
                w0 = __builtin_amdgcn_cvt_pk_fp8_f32(f(2), f(3), w0, true);
                w1 = __builtin_amdgcn_cvt_pk_fp8_f32(f(4), f(5), w1, false);
                w1 = __builtin_amdgcn_cvt_pk_fp8_f32(f(6), f(7), w1, true);
                *reinterpret_cast<int2 *>(q8 + row + (size_t)idx * VEC) = make_int2(w0, w1);
            }
        }
        return;
    }

#pragma unroll
    for (int c = 0; c < CACHE; ++c) {
        const int idx = tid + c * 256;
        if (idx < nvec) {
            float gv[VEC];
            load16<T>(g + (size_t)idx * VEC, gv);
#pragma unroll
            for (int i = 0; i < VEC; ++i) gv[i] = vals[c][i] * scale * gv[i];
            store16<T>(y + row + (size_t)idx * VEC, gv);
        }
    }
    for (int idx = tid + CACHE * 256; idx < nvec; idx += 256) {
        // beyond the register cache: the row as this thread wrote it (x_out may be x, whose old value is gone),
        // else rebuilt from the untouched inputs
        float xv[VEC], gv[VEC];
        if (WRITE_X) load16<T>(x_out + row + (size_t)idx * VEC, xv);
        else load_new(row + (size_t)idx * VEC, xv);
        load16<T>(g + (size_t)idx * VEC, gv);
#pragma unroll
        for (int i = 0; i < VEC; ++i) gv[i] = xv[i] * scale * gv[i];
        store16<T>(y + row + (size_t)idx * VEC, gv);
    }
}

// One workgroup per token.  Work units of 16 bytes: (head, slice of the low half) for the rotation of
// q and k heads, then plain 16-byte copies for v.
template <typename T>
__global__ __launch_bounds__(256) void rope_kv_kernel(T *qkv, T *__restrict__ k_cache, T *__restrict__ v_cache,
                                                      const float *__restrict__ cos_t,
                                                      const float *__restrict__ sin_t, int q_offset, int nq,
                                                      int nkv, int d) {
    constexpr int VEC = 16 / sizeof(T);
    const int t = blockIdx.x;
    const int pos = q_offset + t;
    const int half = d / 2;
    const int upr = half / VEC;
    const int n_rot = (nq + nkv) * upr;
    const int n_v = nkv * d / VEC;
    T *row = qkv + (size_t)t * (nq + 2 * nkv) * d;
    for (int u = threadIdx.x; u < n_rot + n_v; u += 256) {
        if (u < n_rot) {
            const int head = u / upr;
            const int i0 = (u % upr) * VEC;
            T *lo_p = row + (size_t)head * d + i0;
            float lo[VEC], hi[VEC], olo[VEC], ohi[VEC];
            load16<T>(lo_p, lo);
            load16<T>(lo_p + half, hi);
            const float *cp = cos_t + (size_t)pos * half + i0;
            const float *sp = sin_t + (size_t)pos * half + i0;
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const float c = cp[i], s = sp[i];
                olo[i] = lo[i] * c - hi[i] * s;
                ohi[i] = hi[i] * c + lo[i] * s;
            }
            T *dst = (head < nq) ? lo_p : k_cache + ((size_t)pos * nkv + (head - nq)) * d + i0;
            store16<T>(dst, olo);
            store16<T>(dst + half, ohi);
        } else {
            const int uu = u - n_rot;
            const uint4 raw = *reinterpret_cast<const uint4 *>(row + (size_t)(nq + nkv) * d + (size_t)uu * VEC);
            *reinterpret_cast<uint4 *>(v_cache + (size_t)pos * nkv * d + (size_t)uu * VEC) = raw;
        }
    }
}

// Int8 payload for the communication point (paper Section 3.2, "communication dominates": the partial is
// quantised before it is sent).  One workgroup per token row: scale = max|p| / 127 (1 if the row is zero),
// code = round-to-nearest-even(p / scale) in [-127, 127].  Output row = H codes followed by the fp32 scale
// (row pitch H + 16 bytes, so one contiguous copy moves codes and scales).  The partial is rewritten in place
// with code * scale: that is what a receiver of the quantised payload would add to its residual stream.
template <typename T>
__global__ __launch_bounds__(256) void quant_rows_kernel(T *part, signed char *__restrict__ q8, int H) {
    constexpr int VEC = 16 / sizeof(T);
    constexpr int CACHE = 4;
    const int tid = threadIdx.x;
    const int nvec = H / VEC;
    const size_t row = (size_t)blockIdx.x * H;
    signed char *qrow = q8 + (size_t)blockIdx.x * (H + 16);
    float vals[CACHE][VEC];
    float amax = 0.f;
#pragma unroll
    for (int c = 0; c < CACHE; ++c) {
        const int idx = tid + c * 256;
        if (idx < nvec) {
            load16<T>(part + row + (size_t)idx * VEC, vals[c]);
#pragma unroll
            for (int i = 0; i < VEC; ++i) amax = fmaxf(amax, fabsf(vals[c][i]));
        }
    }
    for (int idx = tid + CACHE * 256; idx < nvec; idx += 256) {
        float xv[VEC];
        load16<T>(part + row + (size_t)idx * VEC, xv);
#pragma unroll
        for (int i = 0; i < VEC; ++i) amax = fmaxf(amax, fabsf(xv[i]));
    }
    __shared__ float red[4];
    amax = iso_wave_max(amax);
    if ((tid & 63) == 0) red[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float scale = amax > 0.f ? amax / 127.0f : 1.0f;
    if (tid == 0) *reinterpret_cast<float *>(qrow + H) = scale;
    auto emit = [&](int idx, float (&v)[VEC]) {
        signed char codes[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            float q = rintf(v[i] / scale);
            q = fminf(fmaxf(q, -127.f), 127.f);
            codes[i] = (signed char)(int)q;
            v[i] = q * scale;
        }
        if (VEC == 8) *reinterpret_cast<uint2 *>(qrow + (size_t)idx * VEC) = *reinterpret_cast<const uint2 *>(codes);
        else *reinterpret_cast<unsigned int *>(qrow + (size_t)idx * VEC) = *reinterpret_cast<const unsigned int *>(codes);
        store16<T>(part + row + (size_t)idx * VEC, v);
    };
#pragma unroll
    for (int c = 0; c < CACHE; ++c) {
        const int idx = tid + c * 256;
        if (idx < nvec) emit(idx, vals[c]);
    }
    for (int idx = tid + CACHE * 256; idx < nvec; idx += 256) {
        float xv[VEC];
        load16<T>(part + row + (size_t)idx * VEC, xv);
        emit(idx, xv);
    }
}

template <typename T> __device__ __forceinline__ float silu_f(float z);
template <> __device__ __forceinline__ float silu_f<float>(float z) { return z / (1.0f + expf(-z)); }
template <> __device__ __forceinline__ float silu_f<bf16_t>(float z) { return z / (1.0f + __expf(-z)); }

template <typename T>
__global__ __launch_bounds__(256) void swiglu_kernel(const T *__restrict__ gu, T *__restrict__ a, size_t n_units,
                                                     int F) {
    constexpr int VEC = 16 / sizeof(T);
    const int upr = F / VEC;
    for (size_t u = (size_t)blockIdx.x * 256 + threadIdx.x; u < n_units; u += (size_t)gridDim.x * 256) {
        const size_t t = u / upr;
        const int f0 = (int)(u % upr) * VEC;
        float gate[VEC], up[VEC];
        load16<T>(gu + t * 2 * F + f0, gate);
        load16<T>(gu + t * 2 * F + F + f0, up);
#pragma unroll
        for (int i = 0; i < VEC; ++i) gate[i] = silu_f<T>(gate[i]) * up[i];
        store16<T>(a + t * F + f0, gate);
    }
}

template <typename T, bool Q8>
hipError_t rmsnorm_dispatch(const void *x, const void *delta, const void *delta2, void *x_out, const void *g, void *y,
                            unsigned char *q8, float *q_scale, int T_, int H, float eps, hipStream_t s) {
    dim3 grid(T_), block(256);
    const T *xp = (const T *)x, *d1 = (const T *)delta, *d2 = (const T *)delta2, *gp = (const T *)g;
    T *xo = (T *)x_out, *yp = (T *)y;
    const bool wy = Q8 || y != nullptr;
    if ((delta2 && !delta) || (x_out && !delta) || (!x_out && !wy)) return hipErrorInvalidValue;
#define ISO_NORM_CASE(ND, WX, WY)                                                                                  \
    hipLaunchKernelGGL((rmsnorm_kernel<T, ND, WX, WY, Q8 && WY>), grid, block, 0, s, xp, d1, d2, xo, gp, yp, H, eps, q8, \
                       q_scale)
    const int nd = delta2 ? 2 : (delta ? 1 : 0);
    if (nd == 0) ISO_NORM_CASE(0, false, true);
    else if (nd == 1 && x_out && wy) ISO_NORM_CASE(1, true, true);
    else if (nd == 1 && x_out) { if (Q8) return hipErrorInvalidValue; ISO_NORM_CASE(1, true, false); }
    else if (nd == 1) ISO_NORM_CASE(1, false, true);
    else if (nd == 2 && x_out && wy) ISO_NORM_CASE(2, true, true);
    else if (nd == 2 && x_out) { if (Q8) return hipErrorInvalidValue; ISO_NORM_CASE(2, true, false); }
    else ISO_NORM_CASE(2, false, true);
#undef ISO_NORM_CASE
    return hipGetLastError();
}

}  // namespace

hipError_t iso_launch_rmsnorm(int dtype, const void *x, const void *delta, const void *delta2, void *x_out,
                              const void *g, void *y, int T, int H, float eps, hipStream_t s) {
    if (dtype == ISO_F32) return rmsnorm_dispatch<float, false>(x, delta, delta2, x_out, g, y, nullptr, nullptr, T, H, eps, s);
    return rmsnorm_dispatch<bf16_t, false>(x, delta, delta2, x_out, g, y, nullptr, nullptr, T, H, eps, s);
}

// bf16 only: q8[T, H] / q_scale[T] = FP8 row quantisation of rmsnorm(x (+ delta (+ delta2))) * g; x_out, when given,
// receives the sum.  H <= 8192 (the row stays in registers), H % 8 == 0.
bool iso_rmsnorm_fp8_supported(int H) { return H >= 8 && H <= 8192 && (H % 8) == 0; }

hipError_t iso_launch_rmsnorm_fp8(const void *x, const void *delta, const void *delta2, void *x_out, const void *g,
                                  void *q8, float *q_scale, int T, int H, float eps, hipStream_t s) {
    if (!iso_rmsnorm_fp8_supported(H)) return hipErrorInvalidValue;
    return rmsnorm_dispatch<bf16_t, true>(x, delta, delta2, x_out, g, nullptr, (unsigned char *)q8, q_scale, T, H, eps, s);
}

hipError_t iso_launch_rope_kv(int dtype, void *qkv, void *k_cache, void *v_cache, const float *cos_t,
                              const float *sin_t, int Tc, int q_offset, int nq, int nkv, int d, hipStream_t s) {
    dim3 grid(Tc), block(256);
    if (dtype == ISO_F32)
        hipLaunchKernelGGL(rope_kv_kernel<float>, grid, block, 0, s, (float *)qkv, (float *)k_cache,
                           (float *)v_cache, cos_t, sin_t, q_offset, nq, nkv, d);
    else
        hipLaunchKernelGGL(rope_kv_kernel<bf16_t>, grid, block, 0, s, (bf16_t *)qkv, (bf16_t *)k_cache,
                           (bf16_t *)v_cache, cos_t, sin_t, q_offset, nq, nkv, d);
    return hipGetLastError();
}

hipError_t iso_launch_swiglu(int dtype, const void *gu, void *a, int T, int F, hipStream_t s) {
    const size_t vec = dtype == ISO_F32 ? 4 : 8;
    const size_t n_units = (size_t)T * (F / vec);
    size_t blocks = (n_units + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    dim3 grid((unsigned)blocks), block(256);
    if (dtype == ISO_F32)
        hipLaunchKernelGGL(swiglu_kernel<float>, grid, block, 0, s, (const float *)gu, (float *)a, n_units, F);
    else
        hipLaunchKernelGGL(swiglu_kernel<bf16_t>, grid, block, 0, s, (const bf16_t *)gu, (bf16_t *)a, n_units, F);
    return hipGetLastError();
}

hipError_t iso_launch_quant_rows(int dtype, void *part, void *q8, int T, int H, hipStream_t s) {
    dim3 grid(T), block(256);
    if (dtype == ISO_F32)
        hipLaunchKernelGGL(quant_rows_kernel<float>, grid, block, 0, s, (float *)part, (signed char *)q8, H);
    else
        hipLaunchKernelGGL(quant_rows_kernel<bf16_t>, grid, block, 0, s, (bf16_t *)part, (signed char *)q8, H);
    return hipGetLastError();
}
