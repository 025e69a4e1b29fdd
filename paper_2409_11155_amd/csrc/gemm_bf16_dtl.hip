// bf16 projection GEMM for gfx950: launchers and launch rules of the direct-to-LDS kernel (gemm_dtl_kernel.h) with
// bf16 operands:  c[M,N] = a[M,K] * w[N,K]^T, fp32 accumulate, bf16 output (RNE).  (Projections of the layer: paper
// Section 2.2.)  Requires K % 64 == 0, N % 8 == 0 and M*K, N*K < 2^31 elements; other shapes take the 128x128 staged
// kernel.
#include "gemm_dtl_kernel.h"

// Stream-K workspace of the entry point that allocates nothing (iso_gemm_rowpar_static): flag words (4 KiB) and one
// fp32 partial tile of 256 x 256 for each of at most 256 workgroups.  Every GPU the library runs on holds its own
// copy of this array, at its own address, until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; kernels and copies get the per-device address looked up in iso_gemm_static_setup.
#define ISO_STATIC_SK_MAX_WG 256
#define ISO_STATIC_SK_BYTES (4096 + (size_t)ISO_STATIC_SK_MAX_WG * 256 * 256 * 4)
static __device__ __align__(256) unsigned char scratch[ISO_STATIC_SK_BYTES];

namespace {

constexpr int BK = Bf16Op<false>::KE;  // k elements per slice

template <int BM, int BN, int WM, int WN, bool SWIGLU, bool PIPE, bool M16 = false>
hipError_t launch(const void *a, const void *w, void *c, int M, int N, int K, hipStream_t s) {
    using Cfg = DtlCfg<BM, BN, WM, WN>;
    constexpr int LDS_BYTES = (PIPE && Cfg::W3) ? Cfg::LDS_BYTES_W3 : Cfg::LDS_BYTES;
    static iso_dev_mask lds_allowed{0};
    auto kern = gemm_bf16_dtl_kernel<BM, BN, WM, WN, SWIGLU, PIPE, false, M16>;
    if (hipError_t e = iso_allow_lds(reinterpret_cast<const void *>(kern), LDS_BYTES, &lds_allowed); e != hipSuccess)
        return e;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    dim3 grid(tiles_m * tiles_n), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, s, (const bf16_t *)a, (const bf16_t *)w, (bf16_t *)c, M, N,
                       K, tiles_m, tiles_n, (unsigned char *)nullptr, 0u, (unsigned *)nullptr, 1, 0, RopeArgs{});
    return hipGetLastError();
}

// Stream-K launch shape of this kernel (64-element k-slices): see iso_gemm_sk_plan below.
long long sk_plan(int M, int N, int K, int num_wg, int *TS_, int *G_, int *grouped_) {
    return iso_gemm_sk_plan(M, N, K / BK, num_wg, TS_, G_, grouped_);
}

// stream-K launch of the 256x256 tile: one workgroup per compute unit
template <bool SWIGLU>
hipError_t launch_sk(const void *a, const void *w, void *c, int M, int N, int K, iso_sk_ws *sk, hipStream_t s) {
    using Cfg = DtlCfg<256, 256, 4, 2>;
    constexpr int LDS_BYTES = Cfg::W3 ? Cfg::LDS_BYTES_W3 : Cfg::LDS_BYTES;
    static iso_dev_mask lds_allowed{0};
    auto kern = gemm_bf16_dtl_kernel<256, 256, 4, 2, SWIGLU, true, true>;
    if (hipError_t e = iso_allow_lds(reinterpret_cast<const void *>(kern), LDS_BYTES, &lds_allowed); e != hipSuccess)
        return e;
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    int TS, G, grouped;
    sk_plan(M, N, K, sk->num_wg, &TS, &G, &grouped);
    if (++sk->epoch == 0) sk->epoch = 1;   // 0 is what a never-raised flag holds
    dim3 grid(G), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, s, (const bf16_t *)a, (const bf16_t *)w, (bf16_t *)c, M, N,
                       K, tiles_m, tiles_n, (unsigned char *)sk->base, sk->epoch, sk->err, TS, grouped, RopeArgs{});
    return hipGetLastError();
}

// ---- stream-K launch whose workspace is the static device array above
std::atomic<unsigned char *> g_static_ptr[64];      // per device: address of `scratch` on that device
iso_dev_mask g_static_lds{0};

__global__ void sk_clear_flags_kernel(unsigned *flags, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) flags[i] = 0u;
}

}  // namespace

size_t iso_gemm_static_scratch_bytes(void) { return ISO_STATIC_SK_BYTES; }

// Once per device, with that device current (iso_create calls it): looks up the device address of the static
// workspace and raises the stream-K kernel's LDS limit, so that the entry point itself only launches.
hipError_t iso_gemm_static_setup(void) {
    int dev = -1;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (g_static_ptr[dev].load(std::memory_order_acquire)) return hipSuccess;
    void *p = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    using Cfg = DtlCfg<256, 256, 4, 2>;
    auto kern = gemm_bf16_dtl_kernel<256, 256, 4, 2, false, true, true>;
    if (hipError_t e = iso_allow_lds(reinterpret_cast<const void *>(kern), Cfg::W3 ? Cfg::LDS_BYTES_W3 : Cfg::LDS_BYTES,
                                     &g_static_lds);
        e != hipSuccess)
        return e;
    g_static_ptr[dev].store((unsigned char *)p, std::memory_order_release);
    return hipSuccess;
}

// c = a w^T through the stream-K kernel with the static workspace of the current device.  Two launches, no
// allocation, no memset node: a small kernel clears the flag words the launch uses (the array keeps the last call's
// contents), then the GEMM runs with launch number 1.  hipErrorNotReady if iso_gemm_static_setup has not run on this
// device.
hipError_t iso_launch_gemm_bf16_sk_static(const void *a, const void *w, void *c, int M, int N, int K, unsigned *err_word,
                                          hipStream_t s) {
    int dev = -1;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    unsigned char *ptr = g_static_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) return hipErrorNotReady;
    using Cfg = DtlCfg<256, 256, 4, 2>;
    constexpr int LDS_BYTES = Cfg::W3 ? Cfg::LDS_BYTES_W3 : Cfg::LDS_BYTES;
    int ncu = iso_num_cu();
    if (ncu > ISO_STATIC_SK_MAX_WG) ncu = ISO_STATIC_SK_MAX_WG;
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    int TS, G, grouped;
    sk_plan(M, N, K, ncu, &TS, &G, &grouped);
    if (G < 1 || G > ISO_STATIC_SK_MAX_WG) return hipErrorInvalidValue;
    hipLaunchKernelGGL(sk_clear_flags_kernel, dim3((G + 255) / 256), dim3(256), 0, s, reinterpret_cast<unsigned *>(ptr), G);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    auto kern = gemm_bf16_dtl_kernel<256, 256, 4, 2, false, true, true>;
    hipLaunchKernelGGL(kern, dim3(G), dim3(Cfg::NT), LDS_BYTES, s, (const bf16_t *)a, (const bf16_t *)w, (bf16_t *)c, M, N,
                       K, tiles_m, tiles_n, ptr, 1u, err_word, TS, grouped, RopeArgs{});
    return hipGetLastError();
}

// Stream-K launch shape for an M x N product of nk k-slices on num_wg compute units (shared by the bf16 and FP8
// kernels).  Team size: the largest power of two (at most 8) that tiles the tile rows without idle members; the grouped
// mapping needs 8 * TS to divide the grid and every team a non-empty span, otherwise teams of one in launch order.
// Returns the k-slices each team gets.
long long iso_gemm_sk_plan(int M, int N, int nk, int num_wg, int *TS_, int *G_, int *grouped_) {
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    int TS = 1;
    for (int t = 2; t <= 8; t *= 2)
        if (tiles_m % t == 0) TS = t;
    int G = (num_wg / (8 * TS)) * 8 * TS, grouped = 1;
    long long units = (long long)(tiles_m / TS) * tiles_n * nk;
    if (G < 8 * TS || units < G / TS) {   // tiny problem or odd device
        TS = 1;
        grouped = 0;
        units = (long long)tiles_m * tiles_n * nk;
        G = units < num_wg ? (int)units : num_wg;
    }
    *TS_ = TS;
    *G_ = G;
    *grouped_ = grouped;
    return units / (G / TS);
}


size_t iso_gemm_sk_ws_bytes(int num_wg) { return SK_HDR + (size_t)num_wg * DtlCfg<256, 256, 4, 2>::SLOT_BYTES; }
int iso_gemm_sk_max_wg(void) { return SK_MAX_WG; }

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

// Stream-K or one tile per workgroup?  Measured over the same shapes: with at least ~20 k-slices per team the
// stream-K launch wins or ties (every compute unit busy whatever the tile count, and team members share their W slices
// in L2: 1024x4992x6656 at 32 slices per team +13 %, 2048x1280x8192 at 20 +29 %, 2048x8192x1024 at 16 even); with less
// k depth the cost of parking and fetching the partial tiles (about 6 us per workgroup) dominates (1024x6656x1664 at
// 11 slices per team: 52 against 37 us).
// Not when whole 256x256 tiles already fill their rounds of the chip to 85 %: there the tile-per-workgroup launch with
// 16x16x32 MFMAs is ahead or even (4096x8192x7168 353 against 369 us, 8192x7168x8192 719 against 742, 2048x7168x8192
// at 224 tiles 196 against 207; 4096x2560x8192 at 160 tiles 179 against 156 the other way).
static bool sk_wanted(int M, int N, int K, const iso_sk_ws *sk) {
    if (!sk || !sk->base || sk->num_wg < 8) return false;
    const long long tiles = (long long)((M + 255) / 256) * ((N + 255) / 256);
    const long long rounds = (tiles + sk->num_wg - 1) / sk->num_wg;
    if (tiles * 100 >= 85 * rounds * sk->num_wg) return false;
    int TS, G, grouped;
    return sk_plan(M, N, K, sk->num_wg, &TS, &G, &grouped) >= 20 && grouped;
}

// What a launch with variant 0 would do on a device with num_wg compute units (host only, no device call).
// kind: 6 = stream-K (then *team and *grid are its team size and workgroup count), else the tile variant.
void iso_gemm_bf16_dtl_plan(int M, int N, int K, int num_wg, int *kind, int *team, int *grid) {
    iso_sk_ws probe;
    probe.base = &probe;       // non-null: only looked at, never dereferenced
    probe.err = nullptr;
    probe.epoch = 0;
    probe.num_wg = num_wg;
    int TS = 1, G = 0, grouped = 0;
    if (num_wg > 0 && sk_wanted(M, N, K, &probe)) {
        sk_plan(M, N, K, num_wg, &TS, &G, &grouped);
        *kind = 6;
    } else {
        *kind = pick_variant(M, N);
        const int b = *kind == 1 ? 256 : 128;
        G = ((M + b - 1) / b) * ((N + b - 1) / b);
    }
    *team = TS;
    *grid = G;
}

// variant: 0 = pick by shape; 1 = 256x256 8 waves (16x16x32 MFMAs: measured 6-8 % ahead of 32x32x16 on the launches
//          that fill the chip, 2-6 % behind on the smaller tiles and in the stream-K launch, which keep 32x32x16),
//          2 = 256x128 8 waves, 3 = 128x128 4 waves, 4 = 128x256 8 waves, 5 = 256x256 4 waves, 6 = 256x256 stream-K;
//          +8 selects the plain (non-interleaved) main loop.
// sk may be null: then the stream-K kernel is not considered (variant 6 is an error).
hipError_t iso_launch_gemm_bf16_dtl(const void *a, const void *w, void *c, int M, int N, int K, int variant,
                                    iso_sk_ws *sk, hipStream_t s) {
    int v = variant & 7;
    const int plain = (variant >> 3) & 1;
    if (v == 0) v = sk_wanted(M, N, K, sk) ? 6 : pick_variant(M, N);
#define ISO_DTL(BM_, BN_, WM_, WN_)                                                       \
    return plain ? launch<BM_, BN_, WM_, WN_, false, false>(a, w, c, M, N, K, s)          \
                 : launch<BM_, BN_, WM_, WN_, false, true>(a, w, c, M, N, K, s)
    switch (v) {
        case 1:   // the interleaved loop of the full-size tile issues its products as 16x16x32 MFMAs
            return plain ? launch<256, 256, 4, 2, false, false>(a, w, c, M, N, K, s)
                         : launch<256, 256, 4, 2, false, true, true>(a, w, c, M, N, K, s);
        case 2: ISO_DTL(256, 128, 4, 2);
        case 4: ISO_DTL(128, 256, 2, 4);
        case 5: ISO_DTL(256, 256, 2, 2);
        case 6: return (sk && sk->base) ? launch_sk<false>(a, w, c, M, N, K, sk, s) : hipErrorInvalidValue;
        default: ISO_DTL(128, 128, 2, 2);
    }
#undef ISO_DTL
}

// The kernel variant a launch with `variant` (0 = pick by shape) resolves to, without launching.
int iso_gemm_bf16_dtl_resolve(int M, int N, int K, int variant, const iso_sk_ws *sk) {
    int v = variant & 7;
    if (v == 0) v = sk_wanted(M, N, K, sk) ? 6 : pick_variant(M, N);
    if (v == 6 && !(sk && sk->base)) v = -1;
    return ((variant >> 3) & 1) ? v + 8 : v;
}

// QKV projection with rotary embedding and KV-cache write in its epilogue (head_dim 128).  Only the variants whose
// waves own 128 output columns take it: `resolved` must be 1 (256x256 tile per workgroup) or 6 (its stream-K launch),
// as given by iso_gemm_bf16_dtl_resolve; anything else is hipErrorInvalidValue and the caller runs the plain
// projection followed by the separate rotary kernel.
hipError_t iso_launch_gemm_qkv_rope_bf16(const void *a, const void *w, void *qkv, int M, int N, int K, int resolved,
                                         iso_sk_ws *sk, const float *cos_t, const float *sin_t, void *k_cache,
                                         void *v_cache, int q_offset, int nq, int nkv, hipStream_t s) {
    if (N != (nq + 2 * nkv) * 128 || (resolved != 1 && resolved != 6)) return hipErrorInvalidValue;
    using Cfg = DtlCfg<256, 256, 4, 2>;
    constexpr int LDS_BYTES = Cfg::W3 ? Cfg::LDS_BYTES_W3 : Cfg::LDS_BYTES;
    const RopeArgs rope{cos_t, sin_t, (bf16_t *)k_cache, (bf16_t *)v_cache, q_offset, nq, nkv};
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    if (resolved == 1) {
        static iso_dev_mask lds_allowed{0};
        auto kern = gemm_bf16_dtl_kernel<256, 256, 4, 2, false, true, false, true, true>;
        if (hipError_t e = iso_allow_lds(reinterpret_cast<const void *>(kern), LDS_BYTES, &lds_allowed); e != hipSuccess)
            return e;
        hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(Cfg::NT), LDS_BYTES, s, (const bf16_t *)a, (const bf16_t *)w,
                           (bf16_t *)qkv, M, N, K, tiles_m, tiles_n, (unsigned char *)nullptr, 0u, (unsigned *)nullptr, 1, 0,
                           rope);
        return hipGetLastError();
    }
    if (!(sk && sk->base)) return hipErrorInvalidValue;
    static iso_dev_mask lds_allowed_sk{0};
    auto kern = gemm_bf16_dtl_kernel<256, 256, 4, 2, false, true, true, false, true>;
    if (hipError_t e = iso_allow_lds(reinterpret_cast<const void *>(kern), LDS_BYTES, &lds_allowed_sk); e != hipSuccess)
        return e;
    int TS, G, grouped;
    sk_plan(M, N, K, sk->num_wg, &TS, &G, &grouped);
    if (++sk->epoch == 0) sk->epoch = 1;   // 0 is what a never-raised flag holds
    hipLaunchKernelGGL(kern, dim3(G), dim3(Cfg::NT), LDS_BYTES, s, (const bf16_t *)a, (const bf16_t *)w, (bf16_t *)qkv, M, N,
                       K, tiles_m, tiles_n, (unsigned char *)sk->base, sk->epoch, sk->err, TS, grouped, rope);
    return hipGetLastError();
}

// act[M, F] = silu(a w_gate^T) * (a w_up^T) with w = [gate; up] of shape [2F, K].
bool iso_gemm_swiglu_bf16_supported(int M, int F, int K) {
    return iso_gemm_bf16_dtl_supported(M, 2 * F, K) && (F % 8) == 0;
}

hipError_t iso_launch_gemm_swiglu_bf16(const void *a, const void *w, void *act, int M, int F, int K, int variant,
                                       iso_sk_ws *sk, hipStream_t s) {
    int v = variant & 7;
    if (v == 0) v = sk_wanted(M, 2 * F, K, sk) ? 6 : pick_variant(M, 2 * F);
    switch (v) {
        case 1: return launch<256, 256, 4, 2, true, true, true>(a, w, act, M, 2 * F, K, s);
        case 2: return launch<256, 128, 4, 2, true, true>(a, w, act, M, 2 * F, K, s);
        case 4: return launch<128, 256, 2, 4, true, true>(a, w, act, M, 2 * F, K, s);
        case 6: return (sk && sk->base) ? launch_sk<true>(a, w, act, M, 2 * F, K, sk, s) : hipErrorInvalidValue;
        default: return launch<128, 128, 2, 2, true, true>(a, w, act, M, 2 * F, K, s);
    }
}
