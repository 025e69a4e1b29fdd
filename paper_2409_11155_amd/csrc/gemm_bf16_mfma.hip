// bf16 projection GEMM on the gfx950 matrix cores:  c[M,N] = a[M,K] * w[N,K]^T, fp32 accumulation,
// bf16 output (round to nearest even).  Both operands are K-contiguous, which is exactly the operand
// layout of v_mfma_f32_32x32x16_bf16 (each lane supplies 8 consecutive k of one row), so tiles go
// global -> LDS -> registers without any transpose.  (Projections of the layer: paper Section 2.2.)
//
// Workgroup = 256 threads = 4 wavefronts in a 2 x 2 grid; workgroup tile BM x BN, k slice BK, two LDS
// stages (global loads of slice k+1 are in flight while slice k is multiplied).  Rows past M / N are
// clamped on load and predicated on store; k chunks past K are zero-filled, so any M, N and any K that is
// a multiple of 8 are accepted.
#include "iso_internal.h"

namespace {

constexpr int PAD = 8;  // bf16 elements of padding per LDS row: 16 B, keeps 16-byte row reads conflict-free

template <int BM, int BN, int BK> struct GemmCfg {
    static constexpr int PITCH = BK + PAD;
    static constexpr int A_ELEMS = BM * PITCH;
    static constexpr int W_ELEMS = BN * PITCH;
    static constexpr int STAGE = A_ELEMS + W_ELEMS;
    static constexpr size_t LDS_BYTES = 2 * (size_t)STAGE * sizeof(bf16_t);
    static constexpr int CPR = BK / 8;                 // 16-byte chunks per row
    static constexpr int A_CHUNKS = BM * CPR / 256;    // per thread
    static constexpr int W_CHUNKS = BN * CPR / 256;
    static constexpr int TM = BM / 2 / 32;             // 32x32 MFMA tiles per wave along m
    static constexpr int TN = BN / 2 / 32;
};

template <int BM, int BN, int BK>
__global__ __launch_bounds__(256) void gemm_bf16_mfma_kernel(const bf16_t *__restrict__ A,
                                                             const bf16_t *__restrict__ W,
                                                             bf16_t *__restrict__ C, int M, int N, int K,
                                                             int tiles_m, int tiles_n) {
    using Cfg = GemmCfg<BM, BN, BK>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    bf16_t *lds = reinterpret_cast<bf16_t *>(lds_raw);

    // --- workgroup -> tile: consecutive ids go round-robin over the 8 XCDs, so give each XCD a contiguous
    //     range of tiles (its L2 then serves a compact set of A and W panels), and walk that range in
    //     groups of 8 tile rows.
    int pid = blockIdx.x;
    const int nt = tiles_m * tiles_n;
    const int per_xcd = nt / 8;
    if (pid < per_xcd * 8) pid = (pid % 8) * per_xcd + pid / 8;
    constexpr int GROUP = 8;
    const int width = GROUP * tiles_n;
    const int group_id = pid / width;
    const int first_m = group_id * GROUP;
    const int gsize = min(tiles_m - first_m, GROUP);
    const int tile_m = first_m + (pid % width) % gsize;
    const int tile_n = (pid % width) / gsize;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lgrp = lane >> 5;

    // --- per-thread global chunk coordinates (fixed over the k loop)
    const bf16_t *a_src[Cfg::A_CHUNKS];
    const bf16_t *w_src[Cfg::W_CHUNKS];
    int a_dst[Cfg::A_CHUNKS], w_dst[Cfg::W_CHUNKS];
    int a_k[Cfg::A_CHUNKS], w_k[Cfg::W_CHUNKS];
#pragma unroll
    for (int i = 0; i < Cfg::A_CHUNKS; ++i) {
        const int c = tid + i * 256;
        const int r = c / Cfg::CPR, kc = (c % Cfg::CPR) * 8;
        const int gm = min(m0 + r, M - 1);
        a_src[i] = A + (size_t)gm * K + kc;
        a_dst[i] = r * Cfg::PITCH + kc;
        a_k[i] = kc;
    }
#pragma unroll
    for (int i = 0; i < Cfg::W_CHUNKS; ++i) {
        const int c = tid + i * 256;
        const int r = c / Cfg::CPR, kc = (c % Cfg::CPR) * 8;
        const int gn = min(n0 + r, N - 1);
        w_src[i] = W + (size_t)gn * K + kc;
        w_dst[i] = Cfg::A_ELEMS + r * Cfg::PITCH + kc;
        w_k[i] = kc;
    }

    uint4 a_reg[Cfg::A_CHUNKS], w_reg[Cfg::W_CHUNKS];
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < Cfg::A_CHUNKS; ++i)
            a_reg[i] = (k0 + a_k[i] < K) ? *reinterpret_cast<const uint4 *>(a_src[i] + k0) : zero4;
#pragma unroll
        for (int i = 0; i < Cfg::W_CHUNKS; ++i)
            w_reg[i] = (k0 + w_k[i] < K) ? *reinterpret_cast<const uint4 *>(w_src[i] + k0) : zero4;
    };
    auto store_lds = [&](int stage) {
        bf16_t *base = lds + stage * Cfg::STAGE;
#pragma unroll
        for (int i = 0; i < Cfg::A_CHUNKS; ++i) *reinterpret_cast<uint4 *>(base + a_dst[i]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < Cfg::W_CHUNKS; ++i) *reinterpret_cast<uint4 *>(base + w_dst[i]) = w_reg[i];
    };

    f32x16_t acc[Cfg::TM][Cfg::TN];
#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = (K + BK - 1) / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) load_global((kt + 1) * BK);
        const bf16_t *as = lds + (kt & 1) * Cfg::STAGE + (wm * (BM / 2) + lrow) * Cfg::PITCH + lgrp * 8;
        const bf16_t *ws = lds + (kt & 1) * Cfg::STAGE + Cfg::A_ELEMS + (wn * (BN / 2) + lrow) * Cfg::PITCH + lgrp * 8;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t af[Cfg::TM], wf[Cfg::TN];
#pragma unroll
            for (int i = 0; i < Cfg::TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8_t *>(as + i * 32 * Cfg::PITCH + ks * 16);
#pragma unroll
            for (int j = 0; j < Cfg::TN; ++j)
                wf[j] = *reinterpret_cast<const bf16x8_t *>(ws + j * 32 * Cfg::PITCH + ks * 16);
#pragma unroll
            for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
                for (int j = 0; j < Cfg::TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // --- epilogue: accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i) {
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j) {
            const int gn = n0 + wn * (BN / 2) + j * 32 + lrow;
            if (gn >= N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int gm = m0 + wm * (BM / 2) + i * 32 + 8 * (r / 4) + 4 * lgrp + (r % 4);
                if (gm < M) C[(size_t)gm * N + gn] = (bf16_t)acc[i][j][r];
            }
        }
    }
}

template <int BM, int BN, int BK>
hipError_t launch(const void *a, const void *w, void *c, int M, int N, int K, hipStream_t s) {
    using Cfg = GemmCfg<BM, BN, BK>;
    static iso_dev_mask lds_allowed{0};
    auto kern = gemm_bf16_mfma_kernel<BM, BN, BK>;
    if (hipError_t e = iso_allow_lds(reinterpret_cast<const void *>(kern), (int)Cfg::LDS_BYTES, &lds_allowed); e != hipSuccess)
        return e;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    dim3 grid(tiles_m * tiles_n), block(256);
    hipLaunchKernelGGL(kern, grid, block, Cfg::LDS_BYTES, s, (const bf16_t *)a, (const bf16_t *)w, (bf16_t *)c, M, N,
                       K, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

bool iso_gemm_bf16_mfma_supported(int M, int N, int K) { return M >= 1 && N >= 1 && K >= 8 && (K % 8) == 0; }

hipError_t iso_launch_gemm_bf16_mfma(const void *a, const void *w, void *c, int M, int N, int K, hipStream_t s) {
    return launch<128, 128, 64>(a, w, c, M, N, K, s);
}
