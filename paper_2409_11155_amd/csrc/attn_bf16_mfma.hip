// Chunk attention over the KV cache on the gfx950 matrix cores (bf16 operands, fp32 online softmax),
// head_dim 128.  Local query row i of the chunk is token q_offset + i and sees keys
// j <= q_offset + i, j < kv_len (paper Section 3.1: the second chunk reads the cache the first chunk
// wrote, plus its own causal block).
//
// Layout of the computation.  A workgroup of 4 wavefronts owns 128 query rows of one query head; wave w
// owns rows 32w..32w+31.  Scores are computed TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16:
// the accumulator then holds, in lane l, query column l%32 and 16 keys per 32-key block, so every
// softmax statistic (running max, running sum, rescale factor) is a per-lane scalar and the
// probabilities are already in the register layout of the B operand of the second product
// O^T = V^T P^T -- they never pass through LDS.  The contraction index of that second product may be
// enumerated in any order as long as both operands agree, so V^T is staged in LDS with its keys
// permuted to the order in which the accumulator registers hold them (16-byte operand reads).
#include "iso_internal.h"

namespace {

constexpr int D = 128;
constexpr int BM = 128;           // query rows per workgroup
constexpr int BN = 64;            // keys per iteration
constexpr int KP = D + 8;         // K tile row pitch (elements)
constexpr int VP = BN + 8;        // V^T tile row pitch (elements)

// Position, inside a 16-key block, at which key k (0..15) is stored: the 32x32 accumulator gives lane
// group g (= lane / 32) registers 8t..8t+7 = keys {16t + 4g + 0..3} and {16t + 8 + 4g + 0..3}; the
// operand wants those eight keys contiguous at 8g.
__device__ __forceinline__ int vt_pos(int k) { return ((k >> 2) & 1) * 8 + (k >> 3) * 4 + (k & 3); }

__global__ __launch_bounds__(256) void attn_bf16_mfma_kernel(const bf16_t *__restrict__ Q,
                                                             const bf16_t *__restrict__ Kc,
                                                             const bf16_t *__restrict__ Vc,
                                                             bf16_t *__restrict__ Out, int Tc, int q_offset,
                                                             int kv_len, int nq, int nkv, int q_stride) {
    __shared__ __attribute__((aligned(16))) bf16_t Ks[BN * KP];
    __shared__ __attribute__((aligned(16))) bf16_t Vt[D * VP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lcol = lane & 31, lgrp = lane >> 5;
    const int n_tiles_m = (Tc + BM - 1) / BM;
    const int tile_m = n_tiles_m - 1 - blockIdx.x;      // longest rows first
    const int h = blockIdx.y;
    const int g = h / (nq / nkv);
    const int m0 = tile_m * BM;

    // --- this wave's 32 query rows as the B operand (k = head dim): 8 k-steps of 16
    const int q_row = min(m0 + wave * 32 + lcol, Tc - 1);
    const int q_abs = q_offset + m0 + wave * 32 + lcol;            // absolute position (may exceed the chunk)
    const int wave_q_max = q_offset + m0 + wave * 32 + 31;
    bf16x8_t qf[D / 16];
    {
        const bf16_t *qp = Q + (size_t)q_row * q_stride + (size_t)h * D + lgrp * 8;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qf[ks] = *reinterpret_cast<const bf16x8_t *>(qp + ks * 16);
    }

    f32x16_t o[D / 32];
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    float m_run = -1e30f;     // running max of scaled scores (log2 domain)
    float l_run = 0.f;        // this lane group's share of the running sum
    const float sc = 1.4426950408889634f / sqrtf((float)D);

    const int kv_end = min(kv_len, q_offset + min(m0 + BM, Tc));    // exclusive
    const size_t kv_stride = (size_t)nkv * D;

    for (int j0 = 0; j0 < kv_end; j0 += BN) {
        __syncthreads();       // previous tile fully consumed
        // --- K tile: 64 rows x 16 chunks of 16 B
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * 256;
            const int r = c >> 4, kc = (c & 15) * 8;
            const int key = min(j0 + r, kv_len - 1);
            *reinterpret_cast<uint4 *>(&Ks[r * KP + kc]) =
                *reinterpret_cast<const uint4 *>(Kc + (size_t)key * kv_stride + (size_t)g * D + kc);
        }
        // --- V tile, transposed through registers: thread = (4 keys) x (8 dims)
        {
            const int dg = tid & 15, kg = tid >> 4;
            __attribute__((aligned(16))) bf16_t vals[4][8];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int key = min(j0 + kg * 4 + r, kv_len - 1);
                *reinterpret_cast<uint4 *>(vals[r]) =
                    *reinterpret_cast<const uint4 *>(Vc + (size_t)key * kv_stride + (size_t)g * D + dg * 8);
            }
            const int kpos = (kg >> 2) * 16 + vt_pos((kg & 3) * 4);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                bf16x4_t col = {vals[0][c], vals[1][c], vals[2][c], vals[3][c]};
                *reinterpret_cast<bf16x4_t *>(&Vt[(dg * 8 + c) * VP + kpos]) = col;
            }
        }
        __syncthreads();
        if (j0 > wave_q_max) continue;      // every key of this tile is above this wave's diagonal

        // --- S^T = K Q^T for two 32-key blocks
        f32x16_t s[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
            const bf16_t *kp = &Ks[(sub * 32 + lcol) * KP + lgrp * 8];
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                const bf16x8_t kf = *reinterpret_cast<const bf16x8_t *>(kp + ks * 16);
                s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[sub], 0, 0, 0);
            }
        }
        // --- mask (only tiles that touch the diagonal or the end of the cache), scale to log2 domain
        const bool need_mask = (j0 + BN - 1 > q_offset + m0 + wave * 32) || (j0 + BN > kv_len);
        float mx = -INFINITY;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v = s[sub][r] * sc;
                if (need_mask) {
                    const int key = j0 + sub * 32 + 8 * (r / 4) + 4 * lgrp + (r % 4);
                    if (key > q_abs || key >= kv_len) v = -INFINITY;
                }
                s[sub][r] = v;
                mx = fmaxf(mx, v);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        bf16x8_t pb[2][2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(s[sub][r] - m_new);
                psum += p;
                pb[sub][r / 8][r % 8] = (bf16_t)p;
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        // --- O^T += V^T P^T
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) {
            const bf16_t *vp = &Vt[(dt * 32 + lcol) * VP + lgrp * 8];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const bf16x8_t vf = *reinterpret_cast<const bf16x8_t *>(vp + sub * 32 + t * 16);
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[sub][t], o[dt], 0, 0, 0);
                }
        }
    }

    // --- normalise and store: lane holds column q = lcol, rows d = 32 dt + 8 (r/4) + 4 lgrp + r%4
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    const int row = m0 + wave * 32 + lcol;
    if (row < Tc) {
        bf16_t *op = Out + ((size_t)row * nq + h) * D;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                bf16x4_t v = {(bf16_t)(o[dt][r4 * 4 + 0] * inv), (bf16_t)(o[dt][r4 * 4 + 1] * inv),
                              (bf16_t)(o[dt][r4 * 4 + 2] * inv), (bf16_t)(o[dt][r4 * 4 + 3] * inv)};
                *reinterpret_cast<bf16x4_t *>(op + dt * 32 + 8 * r4 + 4 * lgrp) = v;
            }
    }
}

}  // namespace

bool iso_attn_bf16_mfma_supported(int d) { return d == D; }

hipError_t iso_launch_attn_bf16_mfma(const void *q, const void *k, const void *v, void *out, int Tc, int q_offset,
                                     int kv_len, int nq, int nkv, int d, int q_stride, hipStream_t s) {
    if (d != D) return hipErrorInvalidValue;
    dim3 grid((Tc + BM - 1) / BM, nq), block(256);
    hipLaunchKernelGGL(attn_bf16_mfma_kernel, grid, block, 0, s, (const bf16_t *)q, (const bf16_t *)k,
                       (const bf16_t *)v, (bf16_t *)out, Tc, q_offset, kv_len, nq, nkv, q_stride);
    return hipGetLastError();
}
