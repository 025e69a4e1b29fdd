// bf16 projection GEMM for gfx950, large-tile variant:  c[M,N] = a[M,K] * w[N,K]^T, fp32 accumulate,
// bf16 output (RNE).  (Projections of the layer: paper Section 2.2.)
//
//   * Tiles travel global -> LDS directly (buffer_load_dwordx4 ... lds): no staging registers, no LDS
//     store instructions.  One wave-load deposits 1 KB = 8 rows x 128 B contiguously in LDS; the per-lane
//     byte offset is fixed for the whole k loop and the k advance is the instruction's scalar offset.
//   * Because the LDS position of a lane's 16 bytes is fixed by the lane number, the bank-conflict
//     avoiding swizzle is applied on the GLOBAL side: lane (row r, slot p) fetches 16-byte chunk
//     p ^ swz(r) of its row, so chunk c of row r lives in slot c ^ swz(r); the 16-byte operand reads of
//     32 consecutive rows then spread over all 64 banks (measured: 0 bank conflicts).
//   * Workgroup tile BM x BN (up to 256 x 256), k slice 64, two LDS stages; WM x WN wavefronts, each
//     owning a (BM/WM) x (BN/WN) block of 32x32x16 MFMA tiles.  The 8-wave shapes put two waves on every
//     SIMD, which is what keeps the matrix pipe fed: a single wave cannot issue MFMAs back to back without
//     gaps (a register-only MFMA loop reaches ~82 % of peak with one wave per SIMD, ~99 % with two).
//   * Operand fragments are double-buffered in registers, and the slice hand-over (wait for the next
//     slice's loads, barrier, first fragment reads of the next slice, issue of the loads two slices ahead)
//     sits before the last k-step's MFMAs, which run from registers.
//   * Epilogue: accumulators -> bf16 -> LDS (per-wave region) -> 16-byte row-contiguous global stores.
// Requires K % 64 == 0, N % 8 == 0 and M*K, N*K < 2^31 elements; other shapes take the 128x128 staged kernel.
#include "iso_internal.h"

namespace {

constexpr int BK = 64;                 // k slice: 128 bytes per row
constexpr int ROW_BYTES = BK * 2;

template <int SWZ> __device__ __forceinline__ int swz(int row) {
    if (SWZ == 0) return row & 7;
    return (row >> 1) & 7;
}

template <int BM, int BN, int WM, int WN> struct DtlCfg {
    static constexpr int NWAVES = WM * WN;
    static constexpr int NT = NWAVES * 64;
    static constexpr int A_BYTES = BM * ROW_BYTES, W_BYTES = BN * ROW_BYTES, STAGE = A_BYTES + W_BYTES;
    static constexpr int A_LOADS = BM / 8 / NWAVES, W_LOADS = BN / 8 / NWAVES;   // wave-loads per wave per slice
    static constexpr int WTM = BM / WM, WTN = BN / WN;                          // wave tile
    static constexpr int TM = WTM / 32, TN = WTN / 32;                          // MFMA tiles per wave
    static constexpr int CP = WTN + 8;                                          // epilogue LDS row pitch (elements)
    static constexpr int EPI_BYTES = NWAVES * WTM * CP * 2;
    static constexpr int LDS_BYTES = (2 * STAGE > EPI_BYTES) ? 2 * STAGE : EPI_BYTES;
    static_assert(BM % (8 * NWAVES) == 0 && BN % (8 * NWAVES) == 0, "wave-loads must divide evenly");
};

// SWIGLU = true: W is the [2F, K] gate/up matrix (gate rows first) and the kernel writes
// act[M, F] = silu(gate) * up directly.  The W tile is assembled so that, inside every wave, the MFMA column
// blocks alternate gate / up for the same 32 MLP columns; a lane then holds gate and up of one output element
// in the same register slot of two neighbouring accumulators and the activation needs no data exchange and
// no rounding of the projection output.  N is 2F and the output row stride is F.
template <int BM, int BN, int WM, int WN, int SWZ, bool SWIGLU>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bf16_dtl_kernel(const bf16_t *__restrict__ A,
                                                                     const bf16_t *__restrict__ W,
                                                                     bf16_t *__restrict__ C, int M, int N, int K,
                                                                     int tiles_m, int tiles_n) {
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-resource builtins exist in the device pass only
    using Cfg = DtlCfg<BM, BN, WM, WN>;
    constexpr int NWAVES = Cfg::NWAVES, A_BYTES = Cfg::A_BYTES, STAGE = Cfg::STAGE;
    constexpr int A_LOADS = Cfg::A_LOADS, W_LOADS = Cfg::W_LOADS, TM = Cfg::TM, TN = Cfg::TN;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    // workgroup -> tile: contiguous tile range per XCD (ids go round-robin over 8 XCDs), groups of 8 tile rows
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

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane & 31, lgrp = lane >> 5;

    // ---- global side of the direct-to-LDS loads
    const int ld_row = lane >> 3;          // row inside the 8-row wave-load
    const int ld_slot = lane & 7;          // 16-byte slot this lane's data lands in
    const __amdgpu_buffer_rsrc_t rs_a =
        __builtin_amdgcn_make_buffer_rsrc((void *)A, 0, (int)((uint32_t)M * (uint32_t)K * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w =
        __builtin_amdgcn_make_buffer_rsrc((void *)W, 0, (int)((uint32_t)N * (uint32_t)K * 2u), 0x00020000);
    uint32_t a_off[A_LOADS], w_off[W_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int r = (wave + NWAVES * i) * 8 + ld_row;
        const int chunk = ld_slot ^ swz<SWZ>(r);
        a_off[i] = ((uint32_t)min(m0 + r, M - 1) * (uint32_t)K + chunk * 8) * 2u;
    }
#pragma unroll
    for (int i = 0; i < W_LOADS; ++i) {
        const int r = (wave + NWAVES * i) * 8 + ld_row;
        const int chunk = ld_slot ^ swz<SWZ>(r);
        int grow;
        if (SWIGLU) {
            const int F = N / 2;
            const int jt = (r % Cfg::WTN) / 32;          // MFMA column block inside the wave tile
            const int f = tile_n * (BN / 2) + (r / Cfg::WTN) * (Cfg::WTN / 2) + (jt / 2) * 32 + (r % 32);
            grow = (jt & 1) * F + min(f, F - 1);
        } else {
            grow = min(n0 + r, N - 1);
        }
        w_off[i] = ((uint32_t)grow * (uint32_t)K + chunk * 8) * 2u;
    }
    auto issue = [&](int stage, int k0) {
        unsigned char *base = lds + stage * STAGE;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_a, (__attribute__((address_space(3))) void *)(base + (wave + NWAVES * i) * 1024), 16, a_off[i],
                k0 * 2, 0, 0);
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_w, (__attribute__((address_space(3))) void *)(base + A_BYTES + (wave + NWAVES * i) * 1024), 16,
                w_off[i], k0 * 2, 0, 0);
    };

    // ---- LDS side: byte offsets of this lane's operand rows; the k chunk is XOR-ed in per k-step
    int a_row_off[TM], w_row_off[TN], a_sw[TM], w_sw[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int r = wm * Cfg::WTM + i * 32 + lrow;
        a_row_off[i] = r * ROW_BYTES;
        a_sw[i] = swz<SWZ>(r);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int r = wn * Cfg::WTN + j * 32 + lrow;
        w_row_off[j] = A_BYTES + r * ROW_BYTES;
        w_sw[j] = swz<SWZ>(r);
    }

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ---- main loop
    const int nk = K / BK;
    bf16x8_t af[2][TM], wf[2][TN];
    auto read_frags = [&](const unsigned char *base, int buf, int ks) {
        const int chunk = ks * 2 + lgrp;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            af[buf][i] = *reinterpret_cast<const bf16x8_t *>(base + a_row_off[i] + ((chunk ^ a_sw[i]) << 4));
#pragma unroll
        for (int j = 0; j < TN; ++j)
            wf[buf][j] = *reinterpret_cast<const bf16x8_t *>(base + w_row_off[j] + ((chunk ^ w_sw[j]) << 4));
    };
    auto mfma_step = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], wf[buf][j], acc[i][j], 0, 0, 0);
    };

    issue(0, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    read_frags(lds, 0, 0);
    if (nk > 1) issue(1, BK);
    for (int kt = 0; kt < nk; ++kt) {
        const unsigned char *base = lds + (kt & 1) * STAGE;
#pragma unroll
        for (int ks = 0; ks < BK / 16 - 1; ++ks) {
            read_frags(base, (ks + 1) & 1, ks + 1);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(ks & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (kt + 1 < nk) {
            __builtin_amdgcn_s_waitcnt(0);   // next slice's loads landed; my last fragments are in registers
            __syncthreads();                 // ... for every wave: stage (kt & 1) is free, stage (kt+1)&1 is full
            read_frags(lds + ((kt + 1) & 1) * STAGE, 0, 0);
            if (kt + 2 < nk) issue(kt & 1, (kt + 2) * BK);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_step((BK / 16 - 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- epilogue.  Accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its
    //      32x32 tile.  Each wave parks its tile as bf16 in its own LDS region, then streams it out in
    //      16-byte pieces so that every store instruction covers whole 256-byte row segments.
    __syncthreads();                         // every wave is done reading operand tiles
    if (!SWIGLU) {
        bf16_t *ct = reinterpret_cast<bf16_t *>(lds) + (size_t)wave * Cfg::WTM * Cfg::CP;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    ct[(i * 32 + 8 * (r / 4) + 4 * lgrp + (r % 4)) * Cfg::CP + j * 32 + lrow] = (bf16_t)acc[i][j][r];
        // only this wave reads what it wrote: LDS accesses of one wave are ordered, no barrier needed
        constexpr int CPR = Cfg::WTN / 8;        // 16-byte pieces per row
        constexpr int PIECES = Cfg::WTM * CPR;
        const int gm0 = m0 + wm * Cfg::WTM, gn0 = n0 + wn * Cfg::WTN;
#pragma unroll
        for (int p = lane; p < PIECES; p += 64) {
            const int row = p / CPR, cc = (p % CPR) * 8;
            const int gm = gm0 + row, gn = gn0 + cc;
            if (gm < M && gn < N)                // N % 8 == 0: a piece is entirely inside or outside
                *reinterpret_cast<uint4 *>(C + (size_t)gm * N + gn) =
                    *reinterpret_cast<const uint4 *>(ct + row * Cfg::CP + cc);
        }
    } else {
        constexpr int HW = Cfg::WTN / 2;         // output columns per wave
        constexpr int HP = HW + 8;               // LDS pitch
        const int F = N / 2;
        bf16_t *ct = reinterpret_cast<bf16_t *>(lds) + (size_t)wave * Cfg::WTM * HP;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int jp = 0; jp < TN / 2; ++jp)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float g = acc[i][2 * jp][r], u = acc[i][2 * jp + 1][r];
                    const float a = g / (1.0f + __expf(-g)) * u;
                    ct[(i * 32 + 8 * (r / 4) + 4 * lgrp + (r % 4)) * HP + jp * 32 + lrow] = (bf16_t)a;
                }
        constexpr int CPR = HW / 8;
        constexpr int PIECES = Cfg::WTM * CPR;
        const int gm0 = m0 + wm * Cfg::WTM, gf0 = tile_n * (BN / 2) + wn * HW;
#pragma unroll
        for (int p = lane; p < PIECES; p += 64) {
            const int row = p / CPR, cc = (p % CPR) * 8;
            const int gm = gm0 + row, gf = gf0 + cc;
            if (gm < M && gf < F)                // F % 8 == 0
                *reinterpret_cast<uint4 *>(C + (size_t)gm * F + gf) =
                    *reinterpret_cast<const uint4 *>(ct + row * HP + cc);
        }
    }
#endif
}

template <int BM, int BN, int WM, int WN, int SWZ, bool SWIGLU>
hipError_t launch(const void *a, const void *w, void *c, int M, int N, int K, hipStream_t s) {
    using Cfg = DtlCfg<BM, BN, WM, WN>;
    static bool attr_set = false;
    auto kern = gemm_bf16_dtl_kernel<BM, BN, WM, WN, SWZ, SWIGLU>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    dim3 grid(tiles_m * tiles_n), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, Cfg::LDS_BYTES, s, (const bf16_t *)a, (const bf16_t *)w, (bf16_t *)c, M, N,
                       K, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

bool iso_gemm_bf16_dtl_supported(int M, int N, int K) {
    return M >= 1 && N >= 8 && (N % 8) == 0 && K >= BK && (K % BK) == 0 && (long long)M * K < (1ll << 31) &&
           (long long)N * K < (1ll << 31);
}

// Tile shape.  Measured on MI355X over the projection shapes of the 30B/70B shards: the 256x256 tile wins as
// soon as it yields at least ~128 workgroups (half the compute units: the chip is power-limited, so fewer busy
// units clock higher and a half-filled launch of big tiles still beats a full launch of small ones); below that
// the 128x128 tile (two workgroups per compute unit) is best.
static int pick_variant(int M, int N) {
    const long long tiles_256 = (long long)((M + 255) / 256) * ((N + 255) / 256);
    return tiles_256 >= 128 ? 1 : 3;
}

// variant: 0 = pick by shape; 1 = 256x256 8 waves, 2 = 256x128 8 waves, 3 = 128x128 4 waves, 4 = 128x256 8 waves,
//          5 = 256x256 4 waves; +8 selects the other LDS swizzle
hipError_t iso_launch_gemm_bf16_dtl(const void *a, const void *w, void *c, int M, int N, int K, int variant,
                                    hipStream_t s) {
    int v = variant & 7;
    const int sw = (variant >> 3) & 1;
    if (v == 0) v = pick_variant(M, N);
#define ISO_DTL(BM_, BN_, WM_, WN_)                                                          \
    return sw ? launch<BM_, BN_, WM_, WN_, 0, false>(a, w, c, M, N, K, s)                    \
              : launch<BM_, BN_, WM_, WN_, 1, false>(a, w, c, M, N, K, s)
    switch (v) {
        case 1: ISO_DTL(256, 256, 4, 2);
        case 2: ISO_DTL(256, 128, 4, 2);
        case 4: ISO_DTL(128, 256, 2, 4);
        case 5: ISO_DTL(256, 256, 2, 2);
        default: ISO_DTL(128, 128, 2, 2);
    }
#undef ISO_DTL
}

// act[M, F] = silu(a w_gate^T) * (a w_up^T) with w = [gate; up] of shape [2F, K].
bool iso_gemm_swiglu_bf16_supported(int M, int F, int K) {
    return iso_gemm_bf16_dtl_supported(M, 2 * F, K) && (F % 8) == 0;
}

hipError_t iso_launch_gemm_swiglu_bf16(const void *a, const void *w, void *act, int M, int F, int K, int variant,
                                       hipStream_t s) {
    int v = variant & 7;
    if (v == 0) v = pick_variant(M, 2 * F);
    switch (v) {
        case 1: return launch<256, 256, 4, 2, 1, true>(a, w, act, M, 2 * F, K, s);
        case 2: return launch<256, 128, 4, 2, 1, true>(a, w, act, M, 2 * F, K, s);
        case 4: return launch<128, 256, 2, 4, 1, true>(a, w, act, M, 2 * F, K, s);
        default: return launch<128, 128, 2, 2, 1, true>(a, w, act, M, 2 * F, K, s);
    }
}
