// The direct-to-LDS projection GEMM of libiso for gfx950, one kernel body for both element types:
//   bf16:  c[M,N] = a[M,K] * w[N,K]^T, fp32 accumulate, bf16 output (RNE)            (projections: paper Section 2.2)
//   FP8:   c[M,N] = (a8[M,K] * w8[N,K]^T) * sa[M] * sw[N], E4M3 operands             (8-bit products: paper Section 4.1)
// Included by gemm_bf16_dtl.hip and gemm_fp8_dtl.hip, which hold the launchers and launch rules.
//
//   * Tiles travel global -> LDS directly (buffer_load_dwordx4 ... lds): no staging registers, no LDS
//     store instructions.  One wave-load deposits 1 KB = 8 rows x 128 B contiguously in LDS; the per-lane
//     byte offset is fixed for the whole k loop and the k advance is the instruction's scalar offset.  An LDS row is
//     128 bytes for both element types: a k slice is 64 bf16 or 128 FP8 elements.
//   * Because the LDS position of a lane's 16 bytes is fixed by the lane number, the bank-conflict
//     avoiding swizzle is applied on the GLOBAL side: lane (row r, slot p) fetches 16-byte chunk
//     p ^ swz(r) of its row, so chunk c of row r lives in slot c ^ swz(r); the 16-byte operand reads of
//     32 consecutive rows then spread over all 64 banks (measured: 0 bank conflicts).
//   * Workgroup tile BM x BN (up to 256 x 256), two LDS stages (a third one for W where the LDS allows,
//     so that weight slices are requested two slices ahead); WM x WN wavefronts, each
//     owning a (BM/WM) x (BN/WN) block of MFMA tiles (bf16: 32x32x16, or 16x16x32 in the tile-per-workgroup launch of
//     the 256x256 tile, which does more arithmetic per watt -- this chip runs into its power limit first; FP8:
//     32x32x64, an operand fragment is then 32 bytes per lane = two 16-byte LDS reads).  The 8-wave shapes put two
//     waves on every SIMD, which is what keeps the matrix pipe fed: a single wave cannot issue MFMAs back to back
//     without gaps (a register-only MFMA loop reaches ~82 % of peak with one wave per SIMD, ~99 % with two).
//   * Operand fragments are double-buffered in registers, and the slice hand-over (wait for the next
//     slice's loads, barrier, first fragment reads of the next slice, issue of the loads two slices ahead)
//     sits before the last k-step's MFMAs, which run from registers.
//   * Epilogue: accumulators (FP8: times the two row scales) -> bf16 -> LDS (per-wave region) -> 16-byte
//     row-contiguous global stores.
// Requires K a multiple of the slice (64 bf16 / 128 FP8 elements), N % 8 == 0 and M*K, N*K < 2^31 elements.
#pragma once
#include "iso_internal.h"
#include <type_traits>

namespace {

constexpr int ROW_BYTES = 128;         // bytes of one operand row in an LDS tile = one k slice (64 bf16 or 128 FP8 elements)
constexpr int SK_HDR = 4096;           // stream-K workspace: flag words first, partial-sum slots behind
constexpr int SK_MAX_WG = 512;
constexpr int SK_COHERENT = 1 | 16;    // buffer cache policy bits sc0 | sc1: system scope, bypasses the XCD-local L2
constexpr unsigned SK_SPIN_LIMIT = 4000000u;   // bounded wait (about 2-4 s) so no wave can spin forever

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x8_t __attribute__((ext_vector_type(8)));

// ---- element traits: what differs between the bf16 and the FP8 projection ------------------------------------------
// EB bytes per element; KE elements per k slice; MR rows / columns of one MFMA block; CPS 16-byte chunks of a row per
// k-step of one MFMA (so a slice is 8 / CPS k-steps); RPF 16-byte LDS reads per operand fragment (lane l holds row
// l % MR and chunks (l / MR) * RPF .. + RPF - 1 of the k-step); HS phases a k-step is worked off in (halves of the W
// fragments, to bound the registers of the double-buffered fragments); SCALED: one fp32 scale per A row and per W row
// multiplies the accumulators in the epilogue.
template <bool M16> struct Bf16Op {      // v_mfma_f32_32x32x16_bf16, or 16x16x32 (more arithmetic per watt)
    typedef bf16_t elem;
    typedef bf16x8_t frag_t;
    static constexpr int EB = 2, KE = 64, MR = M16 ? 16 : 32, CPS = M16 ? 4 : 2, RPF = 1, HS = M16 ? 2 : 1;
    static constexpr bool SCALED = false;
    static __device__ __forceinline__ frag_t load(const unsigned char *row, int c0, int sw) {
        return *reinterpret_cast<const frag_t *>(row + ((c0 ^ sw) << 4));
    }
    static __device__ __forceinline__ f32x16_t mfma32(frag_t a, frag_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4_t mfma16(frag_t a, frag_t b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
struct Fp8Op {                           // v_mfma_f32_32x32x64_f8f6f4 on E4M3 x E4M3, no block scales
    typedef unsigned char elem;
    typedef i32x8_t frag_t;
    static constexpr int EB = 1, KE = 128, MR = 32, CPS = 4, RPF = 2, HS = 1;
    static constexpr bool SCALED = true;
    static __device__ __forceinline__ frag_t load(const unsigned char *row, int c0, int sw) {
        const i32x4_t lo = *reinterpret_cast<const i32x4_t *>(row + ((c0 ^ sw) << 4));
        const i32x4_t hi = *reinterpret_cast<const i32x4_t *>(row + (((c0 + 1) ^ sw) << 4));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    static __device__ __forceinline__ f32x16_t mfma32(frag_t a, frag_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4_t mfma16(frag_t, frag_t, f32x4_t c) { return c; }   // not used
};

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
    // Interleaved main loop: a third LDS stage for the W tile only, wherever the 160 KB of a compute unit allow it
    // (the 256x256 tile then takes all of it; the four-wave 128x128 tile, two workgroups per unit, 80 KB each).  W
    // slices are then requested two slices ahead instead of one; weights come from HBM (a layer's weights pass through
    // the memory-side cache once per step), the activations from cache, so only W needs the distance.
    static constexpr int LDS_BYTES_W3 = 2 * A_BYTES + 3 * W_BYTES;
    static constexpr int WGS_PER_CU = (NWAVES == 4 && 2 * LDS_BYTES <= 160 * 1024) ? 2 : 1;
    static constexpr bool W3 = LDS_BYTES_W3 * WGS_PER_CU <= 160 * 1024 && LDS_BYTES_W3 >= EPI_BYTES;
    static constexpr size_t SLOT_BYTES = (size_t)BM * BN * 4;                   // one fp32 partial tile
    static_assert(BM % (8 * NWAVES) == 0 && BN % (8 * NWAVES) == 0, "wave-loads must divide evenly");
};

// SWIGLU = true: W is the [2F, K] gate/up matrix (gate rows first) and the kernel writes
// act[M, F] = silu(gate) * up directly.  The W tile is assembled so that, inside every wave, the MFMA column
// blocks alternate gate / up for the same 32 MLP columns; a lane then holds gate and up of one output element
// in the same register slot of two neighbouring accumulators and the activation needs no data exchange and
// no rounding of the projection output.  N is 2F and the output row stride is F.
//
// SK = true (stream-K): the grid is one workgroup per compute unit and the (tile, k-slice) units are dealt out in
// equal contiguous spans, so a launch whose tile count does not fill the chip still keeps every unit busy.  A span
// that stops inside a tile leaves an fp32 partial tile in the workspace slot of its workgroup and raises that
// workgroup's flag; the workgroup that reaches the tile's last k-slice adds the partials (in team order, so the sum
// is reproducible) and writes the tile.  Progress: every workgroup does its partial segment FIRST and raises its flag
// before it waits for anything, so a workgroup that has been dispatched always publishes its partial; a finisher
// waits only for teams with a lower number, and both mappings place team q - 1 at a lower workgroup id than team q,
// i.e. at a workgroup the dispatcher started earlier.  The grid never exceeds the compute units of the device and a
// workgroup takes a whole unit, so on an otherwise idle chip all of them are resident; beside other kernels a
// workgroup may have to wait for a unit, but only behind kernels that end by themselves or behind stream-K
// workgroups whose own waits point at workgroups dispatched before them.  Every wait is bounded as well: one that
// exceeds the spin limit raises *sk_err (a pinned host word that the library reads at its next entry point and in
// iso_sync) and carries on with a wrong tile.
//
// ROPE = true (the QKV projection of a layer with head_dim 128; W = [q heads | k heads | v heads] x 128 rows): the
// epilogue finishes the step that follows the projection (rotary embedding and KV-cache write, what the next chunk's
// attention waits for, paper Section 3.1).  A wave's 128 output columns are exactly one head, and the rotation pairs
// (c, c + 64) of a row are both in the wave's staging area, so q and k heads are rotated at position q_offset + row
// on their way from the staging area to memory (same arithmetic and roundings as the separate rotary kernel: the
// bf16 projection output is rotated in fp32 and rounded again), q heads go to C, k and v heads straight to rows
// q_offset + row of the caches; the k/v columns of C are not written.
struct RopeArgs {
    const float *cos_t, *sin_t;      // [max_seq, 64] fp32 tables
    bf16_t *k_cache, *v_cache;       // [max_seq, nkv, 128]
    int q_offset, nq, nkv;
};

template <typename OP, int BM, int BN, int WM, int WN, bool SWIGLU, bool PIPE, bool SK, bool ROPE>
__device__ __forceinline__ void gemm_dtl_body(const typename OP::elem *__restrict__ A,
                                              const typename OP::elem *__restrict__ W, const float *__restrict__ sa,
                                              const float *__restrict__ sw, bf16_t *__restrict__ C, int M, int N, int K,
                                              int tiles_m, int tiles_n, unsigned char *sk_ws, unsigned sk_epoch,
                                              unsigned *sk_err, int sk_team, int sk_grouped, const RopeArgs &rope) {
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-resource builtins exist in the device pass only
    using Cfg = DtlCfg<BM, BN, WM, WN>;
    constexpr bool M16 = OP::MR == 16;
    constexpr int NWAVES = Cfg::NWAVES, A_BYTES = Cfg::A_BYTES, STAGE = Cfg::STAGE;
    constexpr int A_LOADS = Cfg::A_LOADS, W_LOADS = Cfg::W_LOADS, TM = Cfg::TM, TN = Cfg::TN;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int nt = tiles_m * tiles_n;
    const int nk = K / OP::KE;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: LDS bases of the wave-loads stay scalar
    const int wm = wave / WN, wn = wave % WN;

    // ---- global side of the direct-to-LDS loads
    const int ld_row = lane >> 3;          // row inside the 8-row wave-load
    const int ld_slot = lane & 7;          // 16-byte slot this lane's data lands in
    const __amdgpu_buffer_rsrc_t rs_a =
        __builtin_amdgcn_make_buffer_rsrc((void *)A, 0, (int)((uint32_t)M * (uint32_t)K * (uint32_t)OP::EB), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w =
        __builtin_amdgcn_make_buffer_rsrc((void *)W, 0, (int)((uint32_t)N * (uint32_t)K * (uint32_t)OP::EB), 0x00020000);
    int m0 = 0, n0 = 0, tile_n = 0;
    uint32_t a_off[A_LOADS], w_off[W_LOADS];
    auto set_tile = [&](int tile_m, int tile_n_) {
        tile_n = tile_n_;
        m0 = tile_m * BM;
        n0 = tile_n * BN;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const int r = (wave + NWAVES * i) * 8 + ld_row;
            const int chunk = ld_slot ^ swz(r);
            a_off[i] = (uint32_t)min(m0 + r, M - 1) * (uint32_t)K * (uint32_t)OP::EB + chunk * 16;
        }
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i) {
            const int r = (wave + NWAVES * i) * 8 + ld_row;
            const int chunk = ld_slot ^ swz(r);
            int grow;
            if (SWIGLU) {
                const int F = N / 2;
                const int jt = (r % Cfg::WTN) / 32;          // MFMA column block inside the wave tile
                const int f = tile_n * (BN / 2) + (r / Cfg::WTN) * (Cfg::WTN / 2) + (jt / 2) * 32 + (r % 32);
                grow = (jt & 1) * F + min(f, F - 1);
            } else {
                grow = min(n0 + r, N - 1);
            }
            w_off[i] = (uint32_t)grow * (uint32_t)K * (uint32_t)OP::EB + chunk * 16;
        }
    };
    // LDS layout.  Two stages of [A tile | W tile]; or, with three W stages, the two A tiles first and the three W
    // tiles behind them.
    constexpr bool W3 = PIPE && Cfg::W3;
    constexpr int WS = W3 ? 3 : 2;
    constexpr int A_STRIDE = W3 ? A_BYTES : STAGE, W_ORIGIN = W3 ? 2 * A_BYTES : A_BYTES;
    constexpr int W_STRIDE = W3 ? Cfg::W_BYTES : STAGE;
    auto issue_a = [&](int stage, int kt) {      // kt: k slice of the tile row; one slice is ROW_BYTES of every row
        unsigned char *base = lds + stage * A_STRIDE;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_a, (__attribute__((address_space(3))) void *)(base + (wave + NWAVES * i) * 1024), 16, a_off[i],
                kt * ROW_BYTES, 0, 0);
    };
    auto issue_w = [&](int stage, int kt) {
        unsigned char *base = lds + W_ORIGIN + stage * W_STRIDE;
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_w, (__attribute__((address_space(3))) void *)(base + (wave + NWAVES * i) * 1024), 16, w_off[i],
                kt * ROW_BYTES, 0, 0);
    };
    auto issue = [&](int stage, int kt) {
        issue_a(stage, kt);
        issue_w(stage, kt);
    };

    // ---- LDS side: byte offsets of this lane's operand rows; the k chunk is XOR-ed in per k-step.
    // bf16, M16: the products are issued as v_mfma_f32_16x16x32_bf16 (k-steps of 32: lane l holds row l % 16 and the
    // 16-byte chunk l / 16 of the step) instead of 32x32x16 (k-steps of 16: row l % 32, chunk l / 32).  Same LDS tiles,
    // same bytes read per FLOP; the smaller instruction moves a quarter of the accumulator registers per issue and
    // measured 15 % more arithmetic per watt on random data (register-only loops: 1.91 against 1.66 PFLOP/s).
    // FP8: 32x32x64, a k-step is 64 bytes of the row, lane l holds row l % 32 and chunks 2 (l / 32), + 1 of the step.
    constexpr int MR = OP::MR;                              // rows / columns of one MFMA block
    constexpr int NKS = 8 / OP::CPS;                        // k-steps per slice
    constexpr int FM = Cfg::WTM / MR, FN = Cfg::WTN / MR;   // operand fragments per k-step
    const int frow = lane & (MR - 1), fgrp = lane / MR;
    // The rows a lane reads (frow + a multiple of 16) all have the same swizzle term, and their offsets from the
    // first one are compile-time constants: one base address per operand, the rest is instruction offsets.
    static_assert(Cfg::WTM % 16 == 0 && Cfg::WTN % 16 == 0, "swizzle term shared by a lane's rows");
    const int f_sw = swz(frow);
    const int a_row0 = (wm * Cfg::WTM + frow) * ROW_BYTES, w_row0 = W_ORIGIN + (wn * Cfg::WTN + frow) * ROW_BYTES;

    // Accumulators: one f32x16 per 32x32 block of the wave tile.  M16 keeps the four 16x16 sub-blocks (si, sj) of a
    // block in registers 4 * (2 si + sj) .. + 3 of that vector.
    f32x16_t acc[TM][TN];
    // A k-step is worked off in HS phases over the W fragments (M16: two halves of four, so that the double-buffered
    // fragments take 64 registers instead of 96; 32x32x16: one).  Phase p = (k-step p / HS, half p % HS) reads its W
    // fragments into wf[p & 1] and, in the first half of a k-step, the A fragments into af[k-step & 1].
    constexpr int HS = OP::HS, FNH = FN / HS, NPH = NKS * HS;
    static_assert(!M16 || PIPE, "the 16x16x32 path exists for the interleaved main loop");
    static_assert(NKS % 2 == 0 && FN % HS == 0, "buffers alternate cleanly across slices");
    typename OP::frag_t af[2][FM], wf[2][FNH];
    auto read_phase = [&](const unsigned char *abase, const unsigned char *wbase, int ph) {
        const int ks = ph / HS, h = ph % HS;
        const int c0 = ks * OP::CPS + fgrp * OP::RPF;      // first 16-byte chunk of this lane's part of the k-step
        if (h == 0) {
            const unsigned char *ap = abase + a_row0;
#pragma unroll
            for (int i = 0; i < FM; ++i) af[ks & 1][i] = OP::load(ap + i * MR * ROW_BYTES, c0, f_sw);
        }
        const unsigned char *wp = wbase + w_row0 + h * FNH * MR * ROW_BYTES;
#pragma unroll
        for (int j = 0; j < FNH; ++j) wf[ph & 1][j] = OP::load(wp + j * MR * ROW_BYTES, c0, f_sw);
    };
    auto mfma_phase = [&](int ph) {
        const int ks = ph / HS, h = ph % HS;
        if constexpr (M16) {
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int jj = 0; jj < FNH; ++jj) {
                    const int j = h * FNH + jj;
                    f32x16_t &blk = acc[i / 2][j / 2];
                    const int q = 4 * (2 * (i & 1) + (j & 1));
                    f32x4_t sub = {blk[q], blk[q + 1], blk[q + 2], blk[q + 3]};
                    sub = OP::mfma16(af[ks & 1][i], wf[ph & 1][jj], sub);
                    blk[q] = sub[0]; blk[q + 1] = sub[1]; blk[q + 2] = sub[2]; blk[q + 3] = sub[3];
                }
        } else {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = OP::mfma32(af[ks & 1][i], wf[ph & 1][j], acc[i][j]);
        }
    };
    // k-step forms for the plain loop (one phase per k-step there)
    auto read_frags = [&](const unsigned char *base, int buf, int ks) { (void)buf; read_phase(base, base, ks); };
    auto mfma_step = [&](int buf) { mfma_phase(buf); };
    // Row and column, inside its 32x32 block, of accumulator register r of this lane.
    auto blk_row = [&](int r) { return M16 ? 16 * (r / 8) + 4 * fgrp + (r % 4) : 8 * (r / 4) + 4 * fgrp + (r % 4); };
    auto blk_col = [&](int r) { return M16 ? 16 * ((r / 4) & 1) + frow : frow; };

    // ---- k slices [kb, ke) of the current tile into acc
    auto run = [&](int kb, int ke) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
        const int n = ke - kb;
        if (SK) __syncthreads();   // the previous segment's epilogue may still be reading its LDS staging area
        issue(0, kb);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        read_frags(lds, 0, 0);
        if (n > 1) issue(1, kb + 1);
        if (W3 && n > 1) issue_w(2, kb + min(2, n - 1));
        if (!PIPE) {
            for (int kt = 0; kt < n; ++kt) {
                const unsigned char *base = lds + (kt & 1) * STAGE;
#pragma unroll
                for (int ks = 0; ks < NKS - 1; ++ks) {
                    read_frags(base, (ks + 1) & 1, ks + 1);
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_step(ks & 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (kt + 1 < n) {
                    __builtin_amdgcn_s_waitcnt(0);   // next slice's loads landed; my last fragments are in registers
                    __syncthreads();                 // ... for every wave: stage (kt & 1) is free, the other is full
                    read_frags(lds + ((kt + 1) & 1) * STAGE, 0, 0);
                    if (kt + 2 < n) issue(kt & 1, kb + kt + 2);
                }
                __builtin_amdgcn_sched_barrier(0);
                mfma_step((NKS - 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            // Interleaved schedule: inside every k-step the fragment reads of the next step (and, in the
            // hand-over step, the direct-to-LDS loads two slices ahead) are slotted between the MFMAs, one
            // memory instruction per MFMA, so a wave's memory issue runs in the shadow of its own matrix
            // instructions instead of leaving the matrix pipe idle.
            constexpr int NMFMA = FM * FNH, NREAD = OP::RPF * (FM + FNH), NLOAD = A_LOADS + W_LOADS;   // per phase (reads: at most)
            auto weave = [&](bool with_loads) {
                if constexpr (NREAD <= NMFMA) {      // fewer reads than MFMAs: one behind each, the loads behind the rest
#pragma unroll
                    for (int i = 0; i < NREAD; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
                    }
                    if (with_loads) {
                        constexpr int REST = NMFMA - NREAD > 0 ? NMFMA - NREAD : 1;
                        constexpr int PER = (NLOAD + REST - 1) / REST;
#pragma unroll
                        for (int i = 0; i < REST; ++i) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                            __builtin_amdgcn_sched_group_barrier(0x020, PER, 0);   // global -> LDS loads
                        }
                    }
                } else {                             // two 16-byte reads per fragment: reads and loads share the MFMAs
                    constexpr int RPM = (NREAD + NMFMA - 1) / NMFMA, PER = (NLOAD + NMFMA - 1) / NMFMA;
#pragma unroll
                    for (int i = 0; i < NMFMA; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);
                        if (with_loads) __builtin_amdgcn_sched_group_barrier(0x020, PER, 0);
                    }
                }
            };
            // With three W stages the hand-over waits for everything but the W_LOADS youngest requests (vector-memory
            // loads complete in order and a hand-over issues its A requests before its W requests, so what may still be
            // out is the W tile two slices ahead); a request past the last slice re-reads the last slice into a free
            // stage, which keeps that count the same to the end.
            constexpr int WAIT_HANDOVER = W3 ? ((W_LOADS & 15) | (7 << 4)) : 0;
            int wst = 0;                             // W stage of the current slice (kt % WS)
            auto slice = [&](int kt, auto handover, auto more) {
                const int wnx = wst + 1 == WS ? 0 : wst + 1;
                const unsigned char *abase = lds + (kt & 1) * A_STRIDE, *wbase = lds + wst * W_STRIDE;
#pragma unroll
                for (int ph = 0; ph < NPH - 1; ++ph) {
                    read_phase(abase, wbase, ph + 1);
                    mfma_phase(ph);
                    weave(false);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (handover) {
                    __builtin_amdgcn_s_waitcnt(WAIT_HANDOVER);   // next slice's loads landed; my last fragments are in registers
                    // ... for every wave: A stage (kt & 1) and W stage wst are free, the next slice is complete.  The
                    // bare instruction: the barrier intrinsic brings a fence that waits for ALL outstanding loads; the
                    // wait above is the fence this hand-over needs, and the memory clobber keeps LDS accesses in place.
                    if (W3) asm volatile("s_barrier" ::: "memory");
                    else __syncthreads();
                    read_phase(lds + ((kt + 1) & 1) * A_STRIDE, lds + wnx * W_STRIDE, 0);
                    if (more) {
                        issue_a(kt & 1, kb + kt + 2);
                        if (W3) issue_w(wst, kb + min(kt + 3, n - 1));
                        else issue_w(kt & 1, kb + kt + 2);
                    }
                }
                mfma_phase(NPH - 1);
                if (handover) weave(more);
                __builtin_amdgcn_sched_barrier(0);
                wst = wnx;
            };
            for (int kt = 0; kt < n - 2; ++kt) slice(kt, std::true_type{}, std::true_type{});
            if (n >= 2) slice(n - 2, std::true_type{}, std::false_type{});
            slice(n - 1, std::false_type{}, std::false_type{});
        }
    };

    // ---- epilogue.  Accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its
    //      32x32 tile (16x16x32 path: row 16*(r/8) + 4*(l/16) + r%4, column 16*((r/4)%2) + l%16).  Each wave parks its tile as bf16 in its own LDS region, then streams it out in
    //      16-byte pieces so that every store instruction covers whole 256-byte row segments.
    auto store_tile = [&]() {
        __syncthreads();                         // every wave is done reading operand tiles
        // SCALED: the accumulators are sums of products of quantised values; row scale x column scale restores them
        float sa_r[OP::SCALED ? TM : 1][16];
        if constexpr (OP::SCALED) {
            static_assert(!OP::SCALED || OP::MR == 32, "a lane's accumulators share one column per 32x32 block");
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) sa_r[i][r] = sa[min(m0 + wm * Cfg::WTM + i * 32 + blk_row(r), M - 1)];
        }
        if (!SWIGLU) {
            const int gm0 = m0 + wm * Cfg::WTM, gn0 = n0 + wn * Cfg::WTN;
            // where this wave's columns go: C, or (ROPE) the head's place in a cache row
            bf16_t *dst = C + gn0;
            size_t dst_stride = (size_t)N;
            int dst_row0 = gm0;
            bool rotate = false;                                 // wave-uniform
            if constexpr (ROPE) {
                static_assert(Cfg::WTN == 128 && TN == 4, "a wave's columns are one head of 128");
                const int head = gn0 / 128;                      // wave-uniform
                rotate = head < rope.nq + rope.nkv;              // q and k heads
                if (head >= rope.nq) {                           // k or v head: rows q_offset + m of its cache
                    const bool is_k = head < rope.nq + rope.nkv;
                    dst = (is_k ? rope.k_cache : rope.v_cache) + (size_t)(head - rope.nq - (is_k ? 0 : rope.nkv)) * 128;
                    dst_stride = (size_t)rope.nkv * 128;
                    dst_row0 = rope.q_offset + gm0;
                }
            }
            bf16_t *ct = reinterpret_cast<bf16_t *>(lds) + (size_t)wave * Cfg::WTM * Cfg::CP;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                float swj = 1.0f;
                if constexpr (OP::SCALED) swj = sw[min(gn0 + j * 32 + frow, N - 1)];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float v = acc[i][j][r];
                        if constexpr (OP::SCALED) v *= sa_r[i][r] * swj;
                        ct[(i * 32 + blk_row(r)) * Cfg::CP + j * 32 + blk_col(r)] = (bf16_t)v;
                    }
            }
            // only this wave reads what it wrote: LDS accesses of one wave are ordered, no barrier needed
            constexpr int CPR = Cfg::WTN / 8;        // 16-byte pieces per row
            constexpr int PIECES = Cfg::WTM * CPR;
            static_assert(PIECES % 64 == 0, "whole wave-stores");
            if (ROPE && rotate) {
                // rotary embedding on the way out: a lane takes the 16-byte piece at columns cc .. cc + 7 (cc < 64) of
                // a row together with its partner at cc + 64, the row's cos / sin for those eight pairs as four
                // 16-byte loads, and writes both rotated pieces (the accumulators are no longer live here, so the
                // table loads of several pieces can be in flight at once)
                constexpr int HPR = CPR / 2;         // piece pairs per row
#pragma unroll
                for (int it = 0; it < PIECES / 128; ++it) {
                    const int p = lane + it * 64;
                    const int row = p / HPR, cc = (p % HPR) * 8;
                    const int gm = gm0 + row;
                    if (gm < M && gn0 < N) {         // a head is entirely inside or outside the matrix
                        const size_t t = (size_t)(rope.q_offset + gm) * 64 + cc;
                        const float4 c0 = *reinterpret_cast<const float4 *>(rope.cos_t + t);
                        const float4 c1 = *reinterpret_cast<const float4 *>(rope.cos_t + t + 4);
                        const float4 s0 = *reinterpret_cast<const float4 *>(rope.sin_t + t);
                        const float4 s1 = *reinterpret_cast<const float4 *>(rope.sin_t + t + 4);
                        const float cs[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
                        const float sn[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
                        const bf16x8_t lo = *reinterpret_cast<const bf16x8_t *>(ct + row * Cfg::CP + cc);
                        const bf16x8_t hi = *reinterpret_cast<const bf16x8_t *>(ct + row * Cfg::CP + cc + 64);
                        bf16x8_t olo, ohi;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float l = (float)lo[e], h = (float)hi[e];
                            olo[e] = (bf16_t)(l * cs[e] - h * sn[e]);
                            ohi[e] = (bf16_t)(h * cs[e] + l * sn[e]);
                        }
                        bf16_t *o = dst + (size_t)(dst_row0 + row) * dst_stride + cc;
                        *reinterpret_cast<bf16x8_t *>(o) = olo;
                        *reinterpret_cast<bf16x8_t *>(o + 64) = ohi;
                    }
                }
            } else {
#pragma unroll
                for (int it = 0; it < PIECES / 64; ++it) {
                    const int p = lane + it * 64;
                    const int row = p / CPR, cc = (p % CPR) * 8;
                    const int gm = gm0 + row, gn = gn0 + cc;
                    if (gm < M && gn < N)            // N % 8 == 0: a piece is entirely inside or outside
                        *reinterpret_cast<uint4 *>(dst + (size_t)(dst_row0 + row) * dst_stride + cc) =
                            *reinterpret_cast<const uint4 *>(ct + row * Cfg::CP + cc);
                }
            }
        } else {
            constexpr int HW = Cfg::WTN / 2;         // output columns per wave
            constexpr int HP = HW + 8;               // LDS pitch
            const int F = N / 2;
            bf16_t *ct = reinterpret_cast<bf16_t *>(lds) + (size_t)wave * Cfg::WTM * HP;
            const int gm0 = m0 + wm * Cfg::WTM, gf0 = tile_n * (BN / 2) + wn * HW;
#pragma unroll
            for (int jp = 0; jp < TN / 2; ++jp) {
                float swg = 1.0f, swu = 1.0f;        // scales of the gate row and the up row of this MLP column
                if constexpr (OP::SCALED) {
                    const int f = min(gf0 + jp * 32 + frow, F - 1);
                    swg = sw[f];
                    swu = sw[F + f];
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float g = acc[i][2 * jp][r], u = acc[i][2 * jp + 1][r];
                        if constexpr (OP::SCALED) {
                            g *= sa_r[i][r] * swg;
                            u *= sa_r[i][r] * swu;
                        }
                        const float a = g / (1.0f + __expf(-g)) * u;
                        ct[(i * 32 + blk_row(r)) * HP + jp * 32 + blk_col(r)] = (bf16_t)a;
                    }
            }
            constexpr int CPR = HW / 8;
            constexpr int PIECES = Cfg::WTM * CPR;
            static_assert(PIECES % 64 == 0, "whole wave-stores");
#pragma unroll
            for (int it = 0; it < PIECES / 64; ++it) {
                const int p = lane + it * 64;
                const int row = p / CPR, cc = (p % CPR) * 8;
                const int gm = gm0 + row, gf = gf0 + cc;
                if (gm < M && gf < F)                // F % 8 == 0
                    *reinterpret_cast<uint4 *>(C + (size_t)gm * F + gf) =
                        *reinterpret_cast<const uint4 *>(ct + row * HP + cc);
            }
        }
    };

    if (!SK) {
        // workgroup -> tile: contiguous tile range per XCD (workgroup ids go round-robin over the 8 XCDs),
        // groups of 8 tile rows, tile row fastest inside a group (neighbours share the W tile)
        int pid = blockIdx.x;
        const int per_xcd = nt / 8;
        if (pid < per_xcd * 8) pid = (pid % 8) * per_xcd + pid / 8;
        constexpr int GROUP = 8;
        const int width = GROUP * tiles_n;
        const int first_m = (pid / width) * GROUP;
        const int gsize = min(tiles_m - first_m, GROUP);
        set_tile(first_m + (pid % width) % gsize, (pid % width) / gsize);
        run(0, nk);
        store_tile();
    } else {
        // Teams of TS workgroups: member r of a team owns tile row gm*TS + r of the team's current column
        // (gm, tile_n), and all members walk the same k range, so the W slices they fetch are shared in L2.
        // The (column, k-slice) units are dealt to the teams in equal contiguous spans.
        const int TS = sk_team, bid = blockIdx.x;
        const int GT = gridDim.x / TS;
        int q, r;                                // team, member
        if (sk_grouped) {                        // team members share an XCD (workgroup ids go round-robin over the 8
            const int idx = bid >> 3;            // XCDs); team q - 1 sits at a lower workgroup id than team q
            q = (idx / TS) * 8 + (bid & 7);
            r = idx % TS;
        } else {
            q = bid / TS;
            r = bid % TS;
        }
        auto wg_of = [&](int qq) { return sk_grouped ? ((qq >> 3) * TS + r) * 8 + (qq & 7) : qq * TS + r; };
        const int ngm = (tiles_m + TS - 1) / TS;
        const long long U = (long long)ngm * tiles_n * nk;
        auto span_begin = [&](int j) { return (int)(U * j / GT); };
        const int u0 = span_begin(q), u1 = span_begin(q + 1);
        unsigned *flags = reinterpret_cast<unsigned *>(sk_ws);
        const __amdgpu_buffer_rsrc_t rs_p = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(sk_ws + SK_HDR), 0, (int)((uint32_t)gridDim.x * (uint32_t)Cfg::SLOT_BYTES), 0x00020000);
        // column -> (tile row of this member, tile column); false if the member has no tile row there
        auto set_col = [&](int col) {
            const int tm = (col / tiles_n) * TS + r;
            if (tm < tiles_m) set_tile(tm, col % tiles_n);
            return tm < tiles_m;
        };

        int owner_end = u1;
        if (u1 % nk != 0) {                      // the span stops inside a column: partial segment, done first
            const int col = u1 / nk;
            const int kb = max(u0, col * nk) - col * nk, ke = u1 - col * nk;
            if (set_col(col)) {
                run(kb, ke);
                // Partials and flags bypass the per-XCD L2 caches in both directions (system-scope loads and
                // stores), so the hand-over needs no cache write-back or invalidate, which would evict the
                // operand tiles of every workgroup on the XCD.
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int v4 = 0; v4 < 4; ++v4) {
                            f32x4_t v = {acc[i][j][4 * v4], acc[i][j][4 * v4 + 1], acc[i][j][4 * v4 + 2],
                                         acc[i][j][4 * v4 + 3]};
                            __builtin_amdgcn_raw_buffer_store_b128(
                                __builtin_bit_cast(u32x4_t, v), rs_p,
                                (uint32_t)(bid * (int)Cfg::SLOT_BYTES +
                                           (((i * TN + j) * 4 + v4) * Cfg::NT + tid) * 16),
                                0, SK_COHERENT);
                        }
                __builtin_amdgcn_s_waitcnt(0);   // my stores have reached memory ...
                __syncthreads();                 // ... and so have everybody's, before the flag goes up
                if (tid == 0)
                    __hip_atomic_store(&flags[bid], sk_epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
            owner_end = col * nk;
        }
        // Finishing segments.  The one that starts inside a column depends on the partial of lower teams, which
        // can be almost a whole column long: it goes last, after the columns that start in this span.
        const int head_col = u0 / nk, head_kb = u0 - head_col * nk;
        const int first_full = head_kb ? head_col + 1 : head_col;
        const int n_full = max(0, owner_end / nk - first_full);
        const int n_own = n_full + ((head_kb && (head_col + 1) * nk <= owner_end) ? 1 : 0);
        for (int o = 0; o < n_own; ++o) {
            const int col = o < n_full ? first_full + o : head_col;
            const int kb = o < n_full ? 0 : head_kb;
            if (!set_col(col)) continue;
            run(kb, nk);
            if (kb > 0) {                        // lower teams hold the first kb slices of this column
                int qfirst = q - 1;
                while (qfirst > 0 && span_begin(qfirst) > col * nk) --qfirst;
                if (tid == 0) {
                    for (int j = qfirst; j < q; ++j) {
                        unsigned spins = 0;
                        while (__hip_atomic_load(&flags[wg_of(j)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) !=
                               sk_epoch) {
                            __builtin_amdgcn_s_sleep(32);
                            if (++spins > SK_SPIN_LIMIT) {
                                __hip_atomic_store(sk_err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                                break;
                            }
                        }
                    }
                }
                __syncthreads();
                // Sixteen 16-byte loads in flight at a time, then their adds: left to itself the compiler waits for
                // every load before the next one, and a cache-bypassing load is a trip to memory (8 us per partial
                // tile that way, measured).
                constexpr int NV = TM * TN * 4, BATCH = 16;
                static_assert(NV % BATCH == 0, "partial tile is a whole number of load batches");
                for (int j = qfirst; j < q; ++j) {
                    const uint32_t src_off = (uint32_t)(wg_of(j) * (int)Cfg::SLOT_BYTES) + (uint32_t)tid * 16u;
#pragma unroll
                    for (int b0 = 0; b0 < NV; b0 += BATCH) {
                        f32x4_t t[BATCH];
#pragma unroll
                        for (int k = 0; k < BATCH; ++k)
                            t[k] = __builtin_bit_cast(
                                f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                                             rs_p, src_off + (uint32_t)((b0 + k) * Cfg::NT * 16), 0, SK_COHERENT));
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int k = 0; k < BATCH; ++k) {
                            const int e = b0 + k, ij = e / 4, v4 = e % 4;
#pragma unroll
                            for (int c = 0; c < 4; ++c) acc[ij / TN][ij % TN][4 * v4 + c] += t[k][c];
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            store_tile();
        }
    }
#endif
}

// The two kernels: the body above with the element traits bound.
template <int BM, int BN, int WM, int WN, bool SWIGLU, bool PIPE, bool SK, bool M16 = false, bool ROPE = false>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bf16_dtl_kernel(const bf16_t *__restrict__ A,
                                                                     const bf16_t *__restrict__ W,
                                                                     bf16_t *__restrict__ C, int M, int N, int K,
                                                                     int tiles_m, int tiles_n,
                                                                     unsigned char *sk_ws, unsigned sk_epoch,
                                                                     unsigned *sk_err, int sk_team, int sk_grouped,
                                                                     RopeArgs rope) {
    gemm_dtl_body<Bf16Op<M16>, BM, BN, WM, WN, SWIGLU, PIPE, SK, ROPE>(A, W, nullptr, nullptr, C, M, N, K, tiles_m, tiles_n,
                                                                      sk_ws, sk_epoch, sk_err, sk_team, sk_grouped, rope);
}

template <int BM, int BN, int WM, int WN, bool SWIGLU, bool SK>
__global__ __launch_bounds__(WM * WN * 64) void gemm_fp8_dtl_kernel(const unsigned char *__restrict__ A,
                                                                    const unsigned char *__restrict__ W,
                                                                    const float *__restrict__ sa,
                                                                    const float *__restrict__ sw,
                                                                    bf16_t *__restrict__ C, int M, int N, int K,
                                                                    int tiles_m, int tiles_n, unsigned char *sk_ws,
                                                                    unsigned sk_epoch, unsigned *sk_err, int sk_team,
                                                                    int sk_grouped) {
    gemm_dtl_body<Fp8Op, BM, BN, WM, WN, SWIGLU, true, SK, false>(A, W, sa, sw, C, M, N, K, tiles_m, tiles_n, sk_ws, sk_epoch,
                                                                  sk_err, sk_team, sk_grouped, RopeArgs{});
}

}  // namespace
