// FP8 (E4M3) projection GEMM for gfx950:  c[M,N] = (a8[M,K] * w8[N,K]^T) * sa[M] * sw[N], fp32 accumulate, bf16
// output (RNE); and the row quantiser that produces a8 / sa (and, once per model, w8 / sw).
// (The paper runs its matrix products in 8 bits, Section 4.1; this is the 8-bit float the CDNA4 matrix cores take.)
//
// Same structure as the bf16 direct-to-LDS kernel: tiles travel global -> LDS with buffer_load ... lds, 16-byte chunks
// XOR-swizzled on the global side, two LDS stages, fragments double-buffered in registers, MFMAs and LDS reads
// interleaved one to one, epilogue through LDS.  What changes with one-byte elements:
//   * an LDS row is still 128 bytes, so a k slice is 128 elements and a slice holds two k-steps of
//     v_mfma_f32_32x32x64_f8f6f4 (64 k each) instead of four of the bf16 instruction;
//   * an operand fragment is 32 bytes per lane (row l%32, k = 32*(l/32) .. +31 of the step): two 16-byte LDS reads;
//   * the accumulators are sums of products of quantised values; the two row scales are applied in the epilogue.
// Requires K % 128 == 0, N % 8 == 0 and M*K, N*K < 2^31.
#include "iso_internal.h"
#include <type_traits>

namespace {

constexpr int KE = 128;                // k elements per slice = 128 bytes per row
constexpr int ROW_BYTES = 128;
constexpr int KSTEP = 64;              // k of one MFMA
constexpr float FP8_MAX = 448.0f;

constexpr int SK_HDR = 4096;            // stream-K workspace: flag words first, partial-sum slots behind (as the bf16 kernel)
constexpr int SK_COHERENT = 1 | 16;    // buffer cache policy bits sc0 | sc1: system scope, bypasses the XCD-local L2
constexpr unsigned SK_SPIN_LIMIT = 4000000u;

typedef int i32x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4sk_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x4sk_t __attribute__((ext_vector_type(4)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

template <int BM, int BN, int WM, int WN> struct F8Cfg {
    static constexpr int NWAVES = WM * WN;
    static constexpr int NT = NWAVES * 64;
    static constexpr int A_BYTES = BM * ROW_BYTES, W_BYTES = BN * ROW_BYTES, STAGE = A_BYTES + W_BYTES;
    static constexpr int A_LOADS = BM / 8 / NWAVES, W_LOADS = BN / 8 / NWAVES;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int CP = WTN + 8;
    static constexpr int EPI_BYTES = NWAVES * WTM * CP * 2;
    // two stages of [A tile | W tile], or -- where the 160 KB of a compute unit allow it -- two A tiles followed by
    // three W tiles: weight slices are then requested two slices ahead (they come from HBM, the activations from cache)
    static constexpr int LDS_BYTES_2 = (2 * STAGE > EPI_BYTES) ? 2 * STAGE : EPI_BYTES;
    static constexpr int LDS_BYTES_W3 = 2 * A_BYTES + 3 * W_BYTES;
    static constexpr int WGS_PER_CU = (NWAVES == 4 && 2 * LDS_BYTES_2 <= 160 * 1024) ? 2 : 1;
    static constexpr bool W3 = LDS_BYTES_W3 * WGS_PER_CU <= 160 * 1024 && LDS_BYTES_W3 >= EPI_BYTES;
    static constexpr int LDS_BYTES = W3 ? LDS_BYTES_W3 : LDS_BYTES_2;
    static constexpr size_t SLOT_BYTES = (size_t)BM * BN * 4;   // one fp32 partial tile
    static_assert(BM % (8 * NWAVES) == 0 && BN % (8 * NWAVES) == 0, "wave-loads must divide evenly");
};

// SWIGLU = true: W is the [2F, K] gate/up matrix (gate rows first, sw has 2F entries) and the kernel writes
// act[M, F] = silu(gate) * up; the W tile rows are arranged as in the bf16 kernel (MFMA column blocks alternate
// gate / up for the same 32 MLP columns).
//
// SK = true: the stream-K launch of the bf16 kernel with the same protocol (one workgroup per compute unit, teams of
// sk_team workgroups on one XCD, equal spans of (column, k-slice) units, fp32 partial tiles and flags in the
// workspace with cache-bypassing accesses, partial segment first and the dependent segment last, bounded waits).
template <int BM, int BN, int WM, int WN, bool SWIGLU, bool SK>
__global__ __launch_bounds__(WM * WN * 64) void gemm_fp8_dtl_kernel(const unsigned char *__restrict__ A,
                                                                    const unsigned char *__restrict__ W,
                                                                    const float *__restrict__ sa,
                                                                    const float *__restrict__ sw,
                                                                    bf16_t *__restrict__ C, int M, int N, int K,
                                                                    int tiles_m, int tiles_n, unsigned char *sk_ws,
                                                                    unsigned sk_epoch, unsigned *sk_err, int sk_team,
                                                                    int sk_grouped) {
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-resource builtins exist in the device pass only
    using Cfg = F8Cfg<BM, BN, WM, WN>;
    constexpr int NWAVES = Cfg::NWAVES, A_BYTES = Cfg::A_BYTES, STAGE = Cfg::STAGE;
    constexpr int A_LOADS = Cfg::A_LOADS, W_LOADS = Cfg::W_LOADS, TM = Cfg::TM, TN = Cfg::TN;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int nt = tiles_m * tiles_n;
    const int nk = K / KE;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane & 31, lgrp = lane >> 5;

    // ---- global side of the direct-to-LDS loads
    const int ld_row = lane >> 3, ld_slot = lane & 7;
    const __amdgpu_buffer_rsrc_t rs_a =
        __builtin_amdgcn_make_buffer_rsrc((void *)A, 0, (int)((uint32_t)M * (uint32_t)K), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w =
        __builtin_amdgcn_make_buffer_rsrc((void *)W, 0, (int)((uint32_t)N * (uint32_t)K), 0x00020000);
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
            a_off[i] = (uint32_t)min(m0 + r, M - 1) * (uint32_t)K + chunk * 16;
        }
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i) {
            const int r = (wave + NWAVES * i) * 8 + ld_row;
            const int chunk = ld_slot ^ swz(r);
            int grow;
            if (SWIGLU) {
                const int F = N / 2;
                const int jt = (r % Cfg::WTN) / 32;
                const int f = tile_n * (BN / 2) + (r / Cfg::WTN) * (Cfg::WTN / 2) + (jt / 2) * 32 + (r % 32);
                grow = (jt & 1) * F + min(f, F - 1);
            } else {
                grow = min(n0 + r, N - 1);
            }
            w_off[i] = (uint32_t)grow * (uint32_t)K + chunk * 16;
        }
    };
    constexpr bool W3 = Cfg::W3;
    constexpr int WS = W3 ? 3 : 2;
    constexpr int A_STRIDE = W3 ? A_BYTES : STAGE, W_ORIGIN = W3 ? 2 * A_BYTES : A_BYTES;
    constexpr int W_STRIDE = W3 ? Cfg::W_BYTES : STAGE;
    auto issue_a = [&](int stage, int kt) {
        unsigned char *base = lds + stage * A_STRIDE;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_a, (__attribute__((address_space(3))) void *)(base + (wave + NWAVES * i) * 1024), 16, a_off[i],
                kt * KE, 0, 0);
    };
    auto issue_w = [&](int stage, int kt) {
        unsigned char *base = lds + W_ORIGIN + stage * W_STRIDE;
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_w, (__attribute__((address_space(3))) void *)(base + (wave + NWAVES * i) * 1024), 16, w_off[i],
                kt * KE, 0, 0);
    };

    // ---- LDS side
    int a_row_off[TM], w_row_off[TN], a_sw[TM], w_sw[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int r = wm * Cfg::WTM + i * 32 + lrow;
        a_row_off[i] = r * ROW_BYTES;
        a_sw[i] = swz(r);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int r = wn * Cfg::WTN + j * 32 + lrow;
        w_row_off[j] = W_ORIGIN + r * ROW_BYTES;
        w_sw[j] = swz(r);
    }

    f32x16_t acc[TM][TN];
    i32x8_t af[2][TM], wf[2][TN];
    // k-step ks of a slice covers bytes 64 ks .. 64 ks + 63 of the row; this lane's half is chunks 4 ks + 2 lgrp, +1
    auto read_frag = [&](const unsigned char *row, int sw_, int ks) {
        const int c0 = 4 * ks + 2 * lgrp;
        const i32x4_t lo = *reinterpret_cast<const i32x4_t *>(row + ((c0 ^ sw_) << 4));
        const i32x4_t hi = *reinterpret_cast<const i32x4_t *>(row + (((c0 + 1) ^ sw_) << 4));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    auto read_frags = [&](const unsigned char *abase, const unsigned char *wbase, int buf, int ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i) af[buf][i] = read_frag(abase + a_row_off[i], a_sw[i], ks);
#pragma unroll
        for (int j = 0; j < TN; ++j) wf[buf][j] = read_frag(wbase + w_row_off[j], w_sw[j], ks);
    };
    auto mfma_step = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(af[buf][i], wf[buf][j], acc[i][j], 0, 0, 0, 0,
                                                                          0, 0);   // E4M3 x E4M3, no block scales
    };
    constexpr int NMFMA = TM * TN, NREAD = 2 * (TM + TN), NLOAD = A_LOADS + W_LOADS;
    auto weave = [&](bool with_loads) {      // one LDS read (then one global->LDS load) per MFMA
        constexpr int RPM = (NREAD + NMFMA - 1) / NMFMA;
#pragma unroll
        for (int i = 0; i < NMFMA; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);
            if (with_loads) {
                constexpr int PER = (NLOAD + NMFMA - 1) / NMFMA;
                __builtin_amdgcn_sched_group_barrier(0x020, PER, 0);
            }
        }
    };
    // With three W stages the hand-over waits for everything but the W_LOADS youngest requests (vector-memory loads
    // complete in order and a hand-over issues its A requests before its W requests, so what may still be out is the W
    // tile two slices ahead); a request past the last slice re-reads the last slice into a free stage, which keeps
    // that count the same to the end.
    constexpr int WAIT_HANDOVER = W3 ? ((W_LOADS & 15) | (7 << 4)) : 0;

    // ---- k slices [kb, ke) of the current tile into acc
    auto run = [&](int kb, int ke) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
        const int n = ke - kb;
        int wst = 0;                             // W stage of the current slice (kt % WS)
        auto slice = [&](int kt, auto handover, auto more) {
            const int wnx = wst + 1 == WS ? 0 : wst + 1;
            read_frags(lds + (kt & 1) * A_STRIDE, lds + wst * W_STRIDE, 1, 1);   // second k-step of this slice
            mfma_step(0);
            weave(false);
            __builtin_amdgcn_sched_barrier(0);
            if (handover) {
                __builtin_amdgcn_s_waitcnt(WAIT_HANDOVER);   // next slice's loads landed; my last fragments are in registers
                // ... for every wave: A stage (kt & 1) and W stage wst are free, the next slice is complete.  The bare
                // instruction where loads stay outstanding: the barrier intrinsic brings a fence that waits for all.
                if (W3) asm volatile("s_barrier" ::: "memory");
                else __syncthreads();
                read_frags(lds + ((kt + 1) & 1) * A_STRIDE, lds + wnx * W_STRIDE, 0, 0);
                if (more) {
                    issue_a(kt & 1, kb + kt + 2);
                    issue_w(W3 ? wst : (kt & 1), kb + (W3 ? min(kt + 3, n - 1) : kt + 2));
                }
            }
            mfma_step(1);
            if (handover) weave(more);
            __builtin_amdgcn_sched_barrier(0);
            wst = wnx;
        };
        if (SK) __syncthreads();   // the previous segment's epilogue may still be reading its LDS staging area
        issue_a(0, kb);
        issue_w(0, kb);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        read_frags(lds, lds, 0, 0);
        if (n > 1) {
            issue_a(1, kb + 1);
            issue_w(1, kb + 1);
            if (W3) issue_w(2, kb + min(2, n - 1));
        }
        for (int kt = 0; kt < n - 2; ++kt) slice(kt, std::true_type{}, std::true_type{});
        if (n >= 2) slice(n - 2, std::true_type{}, std::false_type{});
        slice(n - 1, std::false_type{}, std::false_type{});
    };

    // ---- epilogue: scale, convert, park in LDS per wave, stream out in 16-byte pieces
    auto store_tile = [&]() {
        __syncthreads();
        float sa_r[TM][16];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int gm = m0 + wm * Cfg::WTM + i * 32 + 8 * (r / 4) + 4 * lgrp + (r % 4);
                sa_r[i][r] = sa[min(gm, M - 1)];
            }
        if (!SWIGLU) {
            bf16_t *ct = reinterpret_cast<bf16_t *>(lds) + (size_t)wave * Cfg::WTM * Cfg::CP;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float swj = sw[min(n0 + wn * Cfg::WTN + j * 32 + lrow, N - 1)];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        ct[(i * 32 + 8 * (r / 4) + 4 * lgrp + (r % 4)) * Cfg::CP + j * 32 + lrow] =
                            (bf16_t)(acc[i][j][r] * (sa_r[i][r] * swj));
            }
            constexpr int CPR = Cfg::WTN / 8;
            constexpr int PIECES = Cfg::WTM * CPR;
            static_assert(PIECES % 64 == 0, "whole wave-stores");
            const int gm0 = m0 + wm * Cfg::WTM, gn0 = n0 + wn * Cfg::WTN;
#pragma unroll
            for (int it = 0; it < PIECES / 64; ++it) {
                const int p = lane + it * 64;
                const int row = p / CPR, cc = (p % CPR) * 8;
                const int gm = gm0 + row, gn = gn0 + cc;
                if (gm < M && gn < N)
                    *reinterpret_cast<uint4 *>(C + (size_t)gm * N + gn) =
                        *reinterpret_cast<const uint4 *>(ct + row * Cfg::CP + cc);
            }
        } else {
            constexpr int HW = Cfg::WTN / 2;
            constexpr int HP = HW + 8;
            const int F = N / 2;
            bf16_t *ct = reinterpret_cast<bf16_t *>(lds) + (size_t)wave * Cfg::WTM * HP;
            const int gf0 = tile_n * (BN / 2) + wn * HW;
#pragma unroll
            for (int jp = 0; jp < TN / 2; ++jp) {
                const int f = min(gf0 + jp * 32 + lrow, F - 1);
                const float swg = sw[f], swu = sw[F + f];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float g = acc[i][2 * jp][r] * (sa_r[i][r] * swg);
                        const float u = acc[i][2 * jp + 1][r] * (sa_r[i][r] * swu);
                        const float a = g / (1.0f + __expf(-g)) * u;
                        ct[(i * 32 + 8 * (r / 4) + 4 * lgrp + (r % 4)) * HP + jp * 32 + lrow] = (bf16_t)a;
                    }
            }
            constexpr int CPR = HW / 8;
            constexpr int PIECES = Cfg::WTM * CPR;
            static_assert(PIECES % 64 == 0, "whole wave-stores");
            const int gm0 = m0 + wm * Cfg::WTM;
#pragma unroll
            for (int it = 0; it < PIECES / 64; ++it) {
                const int p = lane + it * 64;
                const int row = p / CPR, cc = (p % CPR) * 8;
                const int gm = gm0 + row, gf = gf0 + cc;
                if (gm < M && gf < F)
                    *reinterpret_cast<uint4 *>(C + (size_t)gm * F + gf) =
                        *reinterpret_cast<const uint4 *>(ct + row * HP + cc);
            }
        }
    };

    if (!SK) {
        // workgroup -> tile: contiguous tile range per XCD, groups of 8 tile rows, tile row fastest inside a group
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
        auto set_col = [&](int col) {            // false if this member has no tile row in the column
            const int tm = (col / tiles_n) * TS + r;
            if (tm < tiles_m) set_tile(tm, col % tiles_n);
            return tm < tiles_m;
        };
        constexpr int NV = TM * TN * 4, BATCH = 16;
        static_assert(NV % BATCH == 0, "partial tile is a whole number of load batches");

        int owner_end = u1;
        if (u1 % nk != 0) {                      // the span stops inside a column: partial segment, done first
            const int col = u1 / nk;
            const int kb = max(u0, col * nk) - col * nk, ke = u1 - col * nk;
            if (set_col(col)) {
                run(kb, ke);
#pragma unroll
                for (int e = 0; e < NV; ++e) {
                    const int ij = e / 4, v4 = e % 4;
                    const f32x4sk_t v = {acc[ij / TN][ij % TN][4 * v4], acc[ij / TN][ij % TN][4 * v4 + 1],
                                         acc[ij / TN][ij % TN][4 * v4 + 2], acc[ij / TN][ij % TN][4 * v4 + 3]};
                    __builtin_amdgcn_raw_buffer_store_b128(
                        __builtin_bit_cast(u32x4sk_t, v), rs_p,
                        (uint32_t)(bid * (int)Cfg::SLOT_BYTES + (e * Cfg::NT + tid) * 16), 0, SK_COHERENT);
                }
                __builtin_amdgcn_s_waitcnt(0);   // my stores have reached memory ...
                __syncthreads();                 // ... and so have everybody's, before the flag goes up
                if (tid == 0)
                    __hip_atomic_store(&flags[bid], sk_epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
            owner_end = col * nk;
        }
        // Finishing segments; the one that starts inside a column (it needs lower teams' partials) goes last.
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
                for (int j = qfirst; j < q; ++j) {   // sixteen 16-byte loads in flight at a time, then their adds
                    const uint32_t src_off = (uint32_t)(wg_of(j) * (int)Cfg::SLOT_BYTES) + (uint32_t)tid * 16u;
#pragma unroll
                    for (int b0 = 0; b0 < NV; b0 += BATCH) {
                        f32x4sk_t t[BATCH];
#pragma unroll
                        for (int k = 0; k < BATCH; ++k)
                            t[k] = __builtin_bit_cast(
                                f32x4sk_t, __builtin_amdgcn_raw_buffer_load_b128(
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
    ++sk->epoch;
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
