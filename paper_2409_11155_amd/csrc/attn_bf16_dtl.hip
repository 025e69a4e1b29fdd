// Chunk attention over the KV cache on the gfx950 matrix cores, pipelined variant (bf16, head_dim 128).
// Local query row i of the chunk is token q_offset + i and sees keys j <= q_offset + i, j < kv_len
// (paper Section 3.1: the second chunk reads the cache the first chunk wrote, plus its own causal block).
//
// Same mathematics and register layout as the staged kernel (scores transposed, S^T = K Q^T, so that the
// softmax statistics are per-lane scalars and the probabilities feed the second product O^T = V^T P^T
// straight from registers).  What differs is how K and V reach the matrix cores:
//   * K and V tiles (64 keys x 128 dims) go global -> LDS directly (buffer_load ... lds) into two stages;
//     the loads of tile j+1 are in flight while tile j is multiplied; one barrier per tile.  Rows past
//     kv_len are out of the buffer's range and read as zero.
//   * Both tiles keep their natural row-major layout; the 16-byte chunks of a row are XOR-swizzled on the
//     global side (the LDS slot of a lane's 16 bytes is fixed by the lane number) so that the operand reads
//     are free of bank conflicts.
//   * V is read with ds_read_b64_tr_b16: 16 lanes fetch a 4-key x 16-dim block and receive it transposed,
//     i.e. each lane gets 4 consecutive keys of one dim -- the k-contiguous operand layout the MFMA wants
//     for V^T -- with no transposing pass over V anywhere.
#include "iso_internal.h"
#include <type_traits>

namespace {

constexpr int D = 128;
constexpr int BM = 128;            // query rows per workgroup (4 waves x 32)
constexpr int BN = 64;             // keys per tile
constexpr int ROW_B = D * 2;       // bytes per K/V row in LDS
constexpr int TILE_B = BN * ROW_B; // 16 KB
constexpr int STAGE_B = 2 * TILE_B;
// Key split across workgroups (launches that leave most compute units idle): one partial state of a row block =
// 16 float4 of unnormalised output + (running maximum, partial sum) for each of the 256 lanes that hold it.
constexpr int PART_O_BYTES = 16 * 256 * 16;
constexpr int PART_BYTES = PART_O_BYTES + 256 * 8;
constexpr int PART_COHERENT = 1 | 16;    // buffer cache policy sc0 | sc1: system scope, bypasses the XCD-local L2

typedef __bf16 bf16x4_v __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_v __attribute__((ext_vector_type(2)));

// Transposing LDS read (ds_read_b64_tr_b16) at LDS byte address `addr` + OFF, written as an instruction: the
// compiler treats the intrinsic form as possibly aliasing the global -> LDS loads in flight and puts a wait for all
// of them (the NEXT tile's loads) in front of it, which serialises the prefetch with the second product.  The data
// being read was landed and fenced by the barrier at the top of the tile loop.  The compiler does not track the
// completion of these reads either: lds_tr_wait<N>() is the matching s_waitcnt, tied to the registers it guards.
template <int OFF> __device__ __forceinline__ bf16x4_v lds_read_tr16(uint32_t addr) {
    bf16x4_v r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
// Waits until at most N LDS reads issued later than the guarded ones are outstanding (LDS reads complete in order).
template <int N> __device__ __forceinline__ void lds_tr_wait(bf16x8_t &a, bf16x8_t &b, bf16x8_t &c, bf16x8_t &d) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}

// max of a value with the one held by the lane 32 places away (the other half of the wave): v_permlane32_swap
// exchanges the upper half of its first operand with the lower half of its second, so with both operands equal the
// two results hold {low, low} and {high, high}; no LDS round trip as a lane shuffle would take.
__device__ __forceinline__ float half_swap_max(float v) {
    const unsigned u = __float_as_uint(v);
    const u32x2_v r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// NSTAGE LDS stages per group of four waves: tile j + NSTAGE - 1 is requested while tile j is multiplied.  Two stages
// (64 KB) let two workgroups share a compute unit and hide each other's latency.
//
// KVS = 2 (launches too small to fill the chip even once): the workgroup has eight waves; waves 0-3 take the first half
// of the row block's key tiles and waves 4-7 the second half, each group with its own LDS stages, and the two partial
// results (running maximum, sum and unnormalised output of every row) are merged through LDS at the end.  That
// halves the serial chain of tiles of a row block and puts two waves on every SIMD, so the softmax arithmetic of one
// overlaps the matrix instructions of the other.  SKEW (with KVS = 2): the second group runs one phase behind the
// first (its second product is deferred to the next iteration), so that the two waves of a SIMD, which leave every
// barrier together, do not ask for the same pipe at the same time (measured 2-5 %).
//
// ksplit > 1 (gridDim.z = ksplit; launches of far fewer workgroups than the chip has compute units): the key tiles of
// a row block are dealt to ksplit workgroups in contiguous shares (each share split again between the two wave groups).
// Every workgroup parks its partial state (maximum, sum, unnormalised output) in its slot of `part_ws` with
// cache-bypassing stores and then raises the row block's arrival counter; the workgroup that arrives last fetches all
// ksplit states and folds them in share order -- the result does not depend on who arrived last -- normalises, writes
// the rows and puts the counter back to zero for the next launch.  Nobody waits for anybody.
template <int NSTAGE, int KVS, bool SKEW>
__global__ __launch_bounds__(256 * KVS, KVS == 1 ? 2 : 1) void attn_bf16_dtl_kernel(const bf16_t *__restrict__ Q,
                                                            const bf16_t *__restrict__ Kc,
                                                            const bf16_t *__restrict__ Vc,
                                                            bf16_t *__restrict__ Out, int Tc, int q_offset,
                                                            int kv_len, int nq, int nkv, int q_stride, int pair,
                                                            int ksplit, unsigned char *part_ws, unsigned *part_cnt) {
#if defined(__HIP_DEVICE_COMPILE__)
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    __shared__ int last_arriver;

    const int tid = threadIdx.x, lane = tid & 63;
    // wave-uniform values are made scalar explicitly: LDS bases of the wave-loads, the diagonal tests and the mask
    // branch then cost scalar instructions instead of per-lane compares and exec-mask juggling
    const int wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);   // wave inside its group of four: 32 query rows
    const int kgrp = KVS == 1 ? 0 : __builtin_amdgcn_readfirstlane(tid >> 8);   // which part of the key tiles
    unsigned char *const lds_g = lds + kgrp * (NSTAGE * STAGE_B);
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds_g;
    const int lcol = lane & 31, lgrp = lane >> 5;
    const int n_tiles_m = (Tc + BM - 1) / BM;
    // pair != 0: the workgroup takes row block n-1-x and then row block x.  The causal work of a row block grows
    // linearly with its index, so every workgroup of the launch then has the same amount of work; with one row
    // block each, a launch of about as many workgroups as the chip holds at once ends when its longest one does,
    // with most compute units idle by then.
    const int n_pass = (pair && (int)blockIdx.x != n_tiles_m - 1 - (int)blockIdx.x) ? 2 : 1;
#pragma nounroll
    for (int pass = 0; pass < n_pass; ++pass) {
    if (pass) __syncthreads();                          // the merge of the previous row block is done with the LDS
    const int tile_m = pass ? (int)blockIdx.x : n_tiles_m - 1 - (int)blockIdx.x;      // longest rows first
    const int h = blockIdx.y;
    const int g = h / (nq / nkv);
    const int m0 = tile_m * BM;

    // ---- this wave's 32 query rows as the B operand (k = head dim): 8 k-steps of 16
    const int q_row = min(m0 + wave * 32 + lcol, Tc - 1);
    const int q_abs = q_offset + m0 + wave * 32 + lcol;
    const int wave_q_max = q_offset + m0 + wave * 32 + 31;
    bf16x8_t qf[D / 16];
    {
        const bf16_t *qp = Q + (size_t)q_row * q_stride + (size_t)h * D + lgrp * 8;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qf[ks] = *reinterpret_cast<const bf16x8_t *>(qp + ks * 16);
    }

    // ---- direct-to-LDS loads: wave-load = 4 rows x 256 B; lane = (row l/16, slot l%16)
    const uint32_t row_stride = (uint32_t)nkv * D * 2u;                         // bytes between cache rows
    const uint32_t n_rec = (uint32_t)(kv_len - 1) * row_stride + (uint32_t)ROW_B;  // this head's slice, rows < kv_len
    const __amdgpu_buffer_rsrc_t rs_k =
        __builtin_amdgcn_make_buffer_rsrc((void *)(Kc + (size_t)g * D), 0, (int)n_rec, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_v =
        __builtin_amdgcn_make_buffer_rsrc((void *)(Vc + (size_t)g * D), 0, (int)n_rec, 0x00020000);
    uint32_t k_off[4], v_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = (wave + 4 * i) * 4 + (lane >> 4);
        const int slot = lane & 15;
        k_off[i] = (uint32_t)r * row_stride + (uint32_t)((slot ^ (r & 15)) << 4);
        v_off[i] = (uint32_t)r * row_stride + (uint32_t)((slot ^ ((r & 3) << 2)) << 4);
    }
    auto issue = [&](int stage, int j0) {
        unsigned char *base = lds_g + stage * STAGE_B;
        const uint32_t tile_off = (uint32_t)j0 * row_stride;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_k, (__attribute__((address_space(3))) void *)(base + (wave + 4 * i) * 1024), 16, k_off[i] + tile_off, 0,
                0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_v, (__attribute__((address_space(3))) void *)(base + TILE_B + (wave + 4 * i) * 1024), 16,
                v_off[i] + tile_off, 0, 0, 0);
    };

    auto issue_half = [&](int stage, int j0, int which) {    // which = 0: the K tile, 1: the V tile
        unsigned char *base = lds_g + stage * STAGE_B + which * TILE_B;
        const uint32_t tile_off = (uint32_t)j0 * row_stride;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                which ? rs_v : rs_k, (__attribute__((address_space(3))) void *)(base + (wave + 4 * i) * 1024), 16,
                (which ? v_off[i] : k_off[i]) + tile_off, 0, 0, 0);
    };

    // ---- LDS read addressing
    // K (A operand of S^T): lane = key row lcol of the 32-key block, 16-byte chunk 2*ks + lgrp, swizzled by row & 15
    const int k_row_off = lcol * ROW_B;
    const int k_sw = lcol & 15;
    // V (A operand of O^T, transposing read): 16-lane group = 4 keys x 16 dims
    const int s16 = lane & 15, half16 = (lane >> 4) & 1;
    const int v_row_base = 4 * lgrp + (s16 >> 2);                 // + 32 sub + 16 t + 8 h
    const int v_sw = ((s16 >> 2) & 3) << 2;
    const int v_chunk_base = 2 * half16 + ((s16 & 3) >> 1);       // + 4 dt
    const int v_byte = (s16 & 1) << 3;

    f32x16_t o[D / 32];
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    float m_run = -1e30f;
    float l_run = 0.f;
    const float sc = 1.4426950408889634f / sqrtf((float)D);

    const int kv_end = min(kv_len, q_offset + min(m0 + BM, Tc));    // exclusive
    const int n_tiles_blk = (kv_end + BN - 1) / BN;                  // key tiles of the row block
    // this workgroup's share [wg_lo, wg_lo + n_tiles_all) of them (all, unless the keys are split across workgroups)
    const int share = (n_tiles_blk + ksplit - 1) / ksplit;
    const int wg_lo = (int)blockIdx.z * share;
    const int n_tiles_all = max(0, min(share, n_tiles_blk - wg_lo));
    // this group's tiles [t_lo, t_lo + n_tiles); with KVS == 2 the first group takes the larger half and both groups
    // run the loop n_iter times so that they meet at every barrier
    const int half = (n_tiles_all + KVS - 1) / KVS;
    const int t_lo = wg_lo + kgrp * half;
    const int n_tiles = max(0, min(half, n_tiles_all - kgrp * half));
    // SKEW: the second group is one phase behind (see below) and needs one iteration more than it has tiles
    const int n_iter = KVS == 1 ? n_tiles : (SKEW ? max(half, n_tiles_all - half + 1) : half);

    // Tiles that lie entirely at or below the diagonal of the block's first row and inside the cache need neither
    // a mask nor a per-wave skip: they run a branch-free body.  The few tiles that touch the diagonal or the end of
    // the cache (and the idle iterations of the shorter key group) take the general body.
    const int n_plain_all = min((q_offset + m0 + 1) / BN, kv_len / BN);
    const int n_main = max(0, min(n_plain_all - t_lo, n_tiles));
    static_assert(NSTAGE == 2, "tile jt+1 is requested while tile jt is multiplied: two stages");

    // this wave's loads have landed, everyone's have, and the stages of the previous iteration are no longer read
    auto wait_and_sync = [&]() {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };

    // --- S^T = K Q^T of tile jt (K stage jt % 2) for two 32-key blocks.  The 16 K fragments are fetched four at a
    //     time, one group ahead of the MFMAs that use them (left to itself the compiler issues every LDS read right
    //     before its MFMA and the matrix pipe waits out the LDS latency sixteen times per tile).  WEAVE: once the last
    //     K fragment reads are out (LDS writes keep their order against LDS reads), requests(0) and requests(1) -- four
    //     global -> LDS loads each -- go one load behind each MFMA of the third and fourth group; issued in one burst
    //     at the top of the tile they hold the wave for some 500 cycles.
    auto qk_scores = [&](int jt, f32x16_t (&sc_t)[2], auto weave_c, auto &&requests) {
        constexpr bool WEAVE = decltype(weave_c)::value;
        const unsigned char *kb = lds_g + (jt % NSTAGE) * STAGE_B;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) sc_t[sub][r] = 0.f;
        bf16x8_t kf[2][4];
        auto read_k = [&](int buf, int grp) {          // group = (sub, half of the head dim): 4 k-steps
            const int sub = grp >> 1, ks0 = (grp & 1) * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                kf[buf][i] = *reinterpret_cast<const bf16x8_t *>(kb + sub * 32 * ROW_B + k_row_off +
                                                                (((2 * (ks0 + i) + lgrp) ^ k_sw) << 4));
        };
        read_k(0, 0);
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            if (grp + 1 < 4) read_k((grp + 1) & 1, grp + 1);
            __builtin_amdgcn_sched_barrier(0);
            const int sub = grp >> 1, ks0 = (grp & 1) * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                sc_t[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[grp & 1][i], qf[ks0 + i], sc_t[sub], 0, 0, 0);
            if (WEAVE && grp >= 2) {
                requests(grp - 2);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // --- mask (only tiles that touch the diagonal or the end of the cache), running maximum and sum, probabilities.
    //     The scores stay unscaled: the softmax scale is positive, so the running maximum can be kept in raw units and
    //     the scale folded into the exponent's multiply-add.
    auto softmax = [&](int j0, auto tail_c, f32x16_t (&sc_t)[2], bf16x8_t (&pb)[2][2]) {
        constexpr bool TAIL = decltype(tail_c)::value;
        if (TAIL && ((j0 + BN - 1 > q_offset + m0 + wave * 32) || (j0 + BN > kv_len))) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = j0 + sub * 32 + 8 * (r / 4) + 4 * lgrp + (r % 4);
                    if (key > q_abs || key >= kv_len) sc_t[sub][r] = -INFINITY;
                }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc_t[sub][r]);
        mx = half_swap_max(mx);
        const float m_new = fmaxf(m_run, mx);
        const float neg_m = -m_new * sc;
        float psum = 0.f;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sc_t[sub][r], sc, neg_m));
                psum += p;
                pb[sub][r / 8][r % 8] = (bf16_t)p;
            }
        // rescale the running sums only when some row of this wave saw a new maximum (wave-uniform branch):
        // deep into a long cache the maxima have settled and the 64 multiplies per tile are skipped
        if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        }
        l_run += psum;
    };

    // --- O^T += V^T P^T with V tile vt (V stage vt % 2).  k-slots 8*lgrp .. +8 of MFMA step (sub, t) hold keys
    //     32 sub + 16 t + 4 lgrp + {0..3} and 32 sub + 16 t + 8 + 4 lgrp + {0..3}: two transposing reads.
    //     The V fragments of one 32-dim block (4 MFMAs) are fetched while the previous block is multiplied.
    auto pv = [&](int vt, bf16x8_t (&pb)[2][2]) {
        bf16x8_t vf[2][4];
        const uint32_t vb_addr = lds_addr + (uint32_t)((vt % NSTAGE) * STAGE_B + TILE_B + v_row_base * ROW_B + v_byte);
        auto read_v = [&](int buf, int dt) {
            const uint32_t a = vb_addr + (uint32_t)(((4 * dt + v_chunk_base) ^ v_sw) << 4);
            // MFMA step st = (sub, t) takes key rows 32 sub + 16 t + {0, 8} (+ the lane's row inside the block)
            vf[buf][0] = __builtin_shufflevector(lds_read_tr16<0 * ROW_B>(a), lds_read_tr16<8 * ROW_B>(a), 0, 1, 2, 3, 4, 5, 6, 7);
            vf[buf][1] = __builtin_shufflevector(lds_read_tr16<16 * ROW_B>(a), lds_read_tr16<24 * ROW_B>(a), 0, 1, 2, 3, 4, 5, 6, 7);
            vf[buf][2] = __builtin_shufflevector(lds_read_tr16<32 * ROW_B>(a), lds_read_tr16<40 * ROW_B>(a), 0, 1, 2, 3, 4, 5, 6, 7);
            vf[buf][3] = __builtin_shufflevector(lds_read_tr16<48 * ROW_B>(a), lds_read_tr16<56 * ROW_B>(a), 0, 1, 2, 3, 4, 5, 6, 7);
        };
        read_v(0, 0);
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) {
            if (dt + 1 < D / 32) {
                read_v((dt + 1) & 1, dt + 1);
                __builtin_amdgcn_sched_barrier(0);
                lds_tr_wait<8>(vf[dt & 1][0], vf[dt & 1][1], vf[dt & 1][2], vf[dt & 1][3]);   // 8 younger reads may pend
            } else {
                __builtin_amdgcn_sched_barrier(0);
                lds_tr_wait<0>(vf[dt & 1][0], vf[dt & 1][1], vf[dt & 1][2], vf[dt & 1][3]);
            }
#pragma unroll
            for (int st = 0; st < 4; ++st)
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt & 1][st], pb[st >> 1][st & 1], o[dt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (!(SKEW && KVS > 1) || kgrp == 0) {
        // One tile per iteration: scores, softmax, second product.  In the branch-free body the eight requests for
        // tile jt+1 ride behind the MFMAs of the first product (no test for the end of the range: a tile past this
        // group's share is never used, its stage is free, and rows past the cache read as zero).
        auto tile = [&](int jt, auto tail_c) {
            constexpr bool TAIL = decltype(tail_c)::value;
            const int j0 = (t_lo + jt) * BN;
            wait_and_sync();
            if (TAIL && jt + 1 < n_tiles) issue((jt + 1) % NSTAGE, j0 + BN);
            if (TAIL) {
                if (KVS > 1 && jt >= n_tiles) return;   // idle iterations: the other group has more to do
                if (j0 > wave_q_max) return;            // every key of this tile is above this wave's diagonal
            }
            f32x16_t sc_t[2];
            bf16x8_t pb[2][2];
            qk_scores(jt, sc_t, std::integral_constant<bool, !TAIL>{},
                      [&](int which) { issue_half((jt + 1) % NSTAGE, j0 + BN, which); });
            softmax(j0, tail_c, sc_t, pb);
            pv(jt, pb);
        };
        if (0 < n_tiles) issue(0, t_lo * BN);
        for (int jt = 0; jt < n_main; ++jt) tile(jt, std::false_type{});
        for (int jt = n_main; jt < n_iter; ++jt) tile(jt, std::true_type{});
    } else {
        // The second key group runs one phase behind: iteration jt does the SECOND product of tile jt-1 and then the
        // scores and softmax of tile jt.  Waves w and w+4 of a 512-thread workgroup share a SIMD (one from each group)
        // and leave every barrier together; with the same order of phases both would want the matrix pipe and then
        // both the vector ALU.  Shifted, one group's softmax runs under the other group's MFMAs.  Same arithmetic in
        // the same order as the plain loop, so the results are bit-identical.
        // K tile jt+1 and V tile jt are requested in iteration jt: V stage jt % 2 was last read (tile jt-2) in
        // iteration jt-1, K stage (jt+1) % 2 (tile jt-1) likewise.
        bf16x8_t pb[2][2];
        bool have_p = false;                            // wave-uniform
        auto tile = [&](int jt, auto tail_c) {
            constexpr bool TAIL = decltype(tail_c)::value;
            const int j0 = (t_lo + jt) * BN;
            wait_and_sync();
            f32x16_t sc_t[2];
            if (TAIL) {
                if (jt + 1 < n_tiles) issue_half((jt + 1) % NSTAGE, j0 + BN, 0);
                if (jt < n_tiles) issue_half(jt % NSTAGE, j0, 1);
                if (have_p) pv(jt - 1, pb);
                have_p = false;
                if (jt >= n_tiles || j0 > wave_q_max) return;
                qk_scores(jt, sc_t, std::false_type{}, [](int) {});
            } else {
                pv(jt - 1, pb);
                qk_scores(jt, sc_t, std::true_type{}, [&](int which) {
                    if (which == 0) issue_half((jt + 1) % NSTAGE, j0 + BN, 0);
                    else issue_half(jt % NSTAGE, j0, 1);
                });
            }
            softmax(j0, tail_c, sc_t, pb);
            have_p = true;
        };
        if (0 < n_tiles) issue_half(0, t_lo * BN, 0);
        tile(0, std::true_type{});
        for (int jt = 1; jt < n_main; ++jt) tile(jt, std::false_type{});
        for (int jt = max(1, n_main); jt < n_iter; ++jt) tile(jt, std::true_type{});
    }

    if (KVS > 1) {
        // merge the two groups: group 1 parks (m, l, o) of its rows in LDS, group 0 folds them into its own.
        // A lane of group 0 and the lane with the same wave and lane number in group 1 hold the same rows and dims.
        __syncthreads();                    // every wave is done with the K/V stages
        float *xo = reinterpret_cast<float *>(lds);                       // [64 values][256 threads]
        float *xm = xo + 64 * 256;                                        // [2][256]
        const int t4 = tid & 255;
        if (kgrp == 1) {
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) xo[(dt * 16 + r) * 256 + t4] = o[dt][r];
            xm[t4] = m_run;
            xm[256 + t4] = l_run;
        }
        __syncthreads();
        if (kgrp == 0) {
            const float m_b = xm[t4], l_b = xm[256 + t4];
            const float m_new = fmaxf(m_run, m_b);
            const float fa = __builtin_amdgcn_exp2f((m_run - m_new) * sc), fb = __builtin_amdgcn_exp2f((m_b - m_new) * sc);
            m_run = m_new;
            l_run = l_run * fa + l_b * fb;
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] = o[dt][r] * fa + xo[(dt * 16 + r) * 256 + t4] * fb;
        }
    }
    bool writes_rows = true;                // workgroup-uniform
    if (ksplit > 1) {
        // park this workgroup's state, count the arrival, and let the last arriver fold all states in share order
        const int t4 = tid & 255;
        const int blk = tile_m * nq + h;
        const __amdgpu_buffer_rsrc_t rs_part = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(part_ws + (size_t)blk * ksplit * PART_BYTES), 0, ksplit * PART_BYTES, 0x00020000);
        if (kgrp == 0) {
            const uint32_t slot = (uint32_t)blockIdx.z * PART_BYTES;
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    f32x4_t v = {o[dt][4 * r4], o[dt][4 * r4 + 1], o[dt][4 * r4 + 2], o[dt][4 * r4 + 3]};
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), rs_part,
                                                           slot + (uint32_t)(((dt * 4 + r4) * 256 + t4) * 16), 0,
                                                           PART_COHERENT);
                }
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(m_run), rs_part, slot + PART_O_BYTES + t4 * 8, 0,
                                                  PART_COHERENT);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(l_run), rs_part, slot + PART_O_BYTES + t4 * 8 + 4, 0,
                                                  PART_COHERENT);
        }
        __builtin_amdgcn_s_waitcnt(0);      // my stores have reached memory ...
        __syncthreads();                    // ... and so have everybody's, before the arrival is counted
        if (tid == 0) {
            const unsigned before =
                __hip_atomic_fetch_add(&part_cnt[blk], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            last_arriver = before == (unsigned)(ksplit - 1);
            if (last_arriver) __hip_atomic_store(&part_cnt[blk], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        __syncthreads();
        writes_rows = last_arriver != 0;
        if (writes_rows && kgrp == 0) {
            m_run = -1e30f;
            l_run = 0.f;
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
            for (int sp = 0; sp < ksplit; ++sp) {
                const uint32_t slot = (uint32_t)sp * PART_BYTES;
                f32x4_t po[16];
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    po[v] = __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                                                            rs_part, slot + (uint32_t)((v * 256 + t4) * 16), 0, PART_COHERENT));
                const float m_b = __uint_as_float(
                    __builtin_amdgcn_raw_buffer_load_b32(rs_part, slot + PART_O_BYTES + t4 * 8, 0, PART_COHERENT));
                const float l_b = __uint_as_float(
                    __builtin_amdgcn_raw_buffer_load_b32(rs_part, slot + PART_O_BYTES + t4 * 8 + 4, 0, PART_COHERENT));
                const float m_new = fmaxf(m_run, m_b);
                const float fa = __builtin_amdgcn_exp2f((m_run - m_new) * sc), fb = __builtin_amdgcn_exp2f((m_b - m_new) * sc);
                m_run = m_new;
                l_run = l_run * fa + l_b * fb;
#pragma unroll
                for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[dt][r] = o[dt][r] * fa + po[dt * 4 + r / 4][r % 4] * fb;
            }
        }
    }
    // --- normalise and store: lane holds column q = lcol, rows d = 32 dt + 8 (r/4) + 4 lgrp + r%4
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    const int row = m0 + wave * 32 + lcol;
    if (writes_rows && kgrp == 0 && row < Tc) {
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
    }   // row blocks of this workgroup
#endif
}

}  // namespace

bool iso_attn_bf16_dtl_supported(int d, int kv_len, int nkv) {
    // the K/V slice of one head must be addressable with 32-bit byte offsets
    return d == D && (long long)kv_len * nkv * D * 2 < (1ll << 31);
}

// shape: 0 = chosen from the size; forced by tests and measurement: 1 = key split inside the workgroup, 2 = key split
// and two row blocks per workgroup, 3 = one row block, two workgroups per compute unit.
// ksplit_req: 0 = key split across workgroups chosen from the size, 1 = never, 2..4 = that many shares (forced by tests;
// ignored when the workspace is missing or too small).
hipError_t iso_launch_attn_bf16_dtl(const void *q, const void *k, const void *v, void *out, int Tc, int q_offset,
                                    int kv_len, int nq, int nkv, int d, int q_stride, int shape, int ksplit_req,
                                    const iso_attn_ws *ws, hipStream_t s) {
    if (d != D) return hipErrorInvalidValue;
    static iso_dev_mask lds_allowed[2];
    if (hipError_t e = iso_allow_lds(reinterpret_cast<const void *>(attn_bf16_dtl_kernel<2, 1, false>), 2 * STAGE_B, &lds_allowed[0]);
        e != hipSuccess)
        return e;
    if (hipError_t e = iso_allow_lds(reinterpret_cast<const void *>(attn_bf16_dtl_kernel<2, 2, true>), 2 * 2 * STAGE_B, &lds_allowed[1]);
        e != hipSuccess)
        return e;
    const int n_blocks = (Tc + BM - 1) / BM;
    const long long wgs = (long long)n_blocks * nq;
    // Launches that cannot put two workgroups on every compute unit split the keys inside the workgroup (measured:
    // 1.2-1.4x at 100-500 workgroups).  From about one workgroup per unit up to four times what the chip holds at
    // once (beyond that, deep in a long cache, plain launches measured 4 % better), the workgroups also take two row blocks each (longest with shortest), so that all of them carry the same
    // work -- provided the halved count fills its last round of the chip to 90 % (measured 1.05-1.36x; a three-quarter
    // full third round loses instead).  Larger launches balance by themselves (longest row blocks first) and run two
    // independent workgroups per unit (3-8 % better there).
    const int ncu = iso_num_cu();
    const long long paired = (long long)((n_blocks + 1) / 2) * nq;
    const long long rounds = (paired + ncu - 1) / ncu;
    const bool pair_ok = wgs >= 320 && wgs <= 2048 && (paired <= ncu || paired * 10 >= 9 * rounds * ncu);
    const int mode = shape >= 1 && shape <= 3 ? shape - 1 : (pair_ok ? 1 : wgs < 512 ? 0 : 2);
    // Launches of at most half as many workgroups as the chip has compute units also split the keys ACROSS
    // workgroups, into as many shares as fit the chip once (at most 4, and at least two key tiles per share and wave
    // group on the longest row block): the serial chain of key tiles per workgroup, which is what such a launch takes,
    // shrinks by that factor.
    int ksplit = 1;
    if (ws && ws->part && ws->cnt && wgs <= ws->max_blocks) {
        if (ksplit_req >= 2) {
            ksplit = ksplit_req;
        } else if (ksplit_req == 0 && mode == 0 && wgs * 2 <= ncu) {
            const int longest = (min(kv_len, q_offset + Tc) + BN - 1) / BN;      // key tiles of the last row block
            ksplit = (int)min((long long)4, (long long)ncu / wgs);
            while (ksplit > 1 && longest < 4 * ksplit) --ksplit;
        }
        if (wgs * ksplit > ws->max_slots) ksplit = 1;
    }
    if (mode == 0 || mode == 1)
        hipLaunchKernelGGL((attn_bf16_dtl_kernel<2, 2, true>), dim3(mode == 0 ? n_blocks : (n_blocks + 1) / 2, nq, ksplit),
                           dim3(512), 2 * 2 * STAGE_B, s, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                           (bf16_t *)out, Tc, q_offset, kv_len, nq, nkv, q_stride, mode, ksplit,
                           ws ? ws->part : nullptr, ws ? ws->cnt : nullptr);
    else
        hipLaunchKernelGGL((attn_bf16_dtl_kernel<2, 1, false>), dim3(n_blocks, nq, ksplit), dim3(256), 2 * STAGE_B, s,
                           (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v, (bf16_t *)out, Tc, q_offset, kv_len, nq,
                           nkv, q_stride, 0, ksplit, ws ? ws->part : nullptr, ws ? ws->cnt : nullptr);
    return hipGetLastError();
}

size_t iso_attn_part_bytes(void) { return PART_BYTES; }
