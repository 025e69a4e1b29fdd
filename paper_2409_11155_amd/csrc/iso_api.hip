// C ABI of libiso: argument validation, context, and the two-stream ISO schedule.
//
// Schedule (paper Section 1, Figure 1(d); Section 3.1).  A layer is two blocks per chunk: the attention
// block A (norm, QKV, RoPE + cache write, attention, o_proj) and the MLP block M (residual + norm,
// gate/up, SwiGLU, down), each ending in a communication point X.  Chunk c's kernels AND its two copies
// are enqueued on stream c, so "the consumer of a collective waits for it" is plain stream order, and
// while stream c is inside a copy the other stream's kernels own the compute units.  The single
// cross-stream dependency is the event "chunk 0 has written its K/V rows", awaited by chunk 1 right
// before its attention (Section 3.1).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "iso_internal.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return fail(ISO_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));    \
    } while (0)

size_t elt_size(int dtype) { return dtype == ISO_F32 ? 4 : 2; }
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int n_qkv(const iso_cfg &c) { return (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim; }

struct WsLayout {
    size_t y, qkv, attn, part, part_m, gu, act, q8, a8, a8s, a8_pitch, total;
};

WsLayout ws_layout(const iso_cfg &c) {
    const size_t e = elt_size(c.dtype), t = (size_t)c.max_seq;
    WsLayout l;
    size_t off = 0;
    auto take = [&](size_t elems) { size_t o = off; off = align_up(off + elems * e, 256); return o; };
    l.y = take(t * c.hidden);
    l.qkv = take(t * n_qkv(c));
    l.attn = take(t * c.n_q_heads * c.head_dim);
    l.part = take(t * c.hidden);
    l.part_m = take(t * c.hidden);
    l.gu = take(t * 2 * c.ffn);
    l.act = take(t * c.ffn);
    l.q8 = take((t * (c.hidden + 16) + e - 1) / e);
    size_t kmax = (size_t)c.hidden;
    if ((size_t)c.n_q_heads * c.head_dim > kmax) kmax = (size_t)c.n_q_heads * c.head_dim;
    if ((size_t)c.ffn > kmax) kmax = (size_t)c.ffn;
    l.a8_pitch = kmax;
    l.a8 = take(c.dtype == ISO_BF16 ? (t * kmax + e - 1) / e : 0);
    l.a8s = take(c.dtype == ISO_BF16 ? t * 2 : 0);               // fp32 = two bf16 slots
    l.total = off;
    return l;
}

int check_cfg(const iso_cfg *c) {
    if (!c) return fail(ISO_ERR_NULL, "cfg is NULL");
    if (c->dtype != ISO_F32 && c->dtype != ISO_BF16) return fail(ISO_ERR_DTYPE, "dtype %d is not ISO_F32/ISO_BF16", c->dtype);
    if (c->hidden < 8 || c->hidden % 8) return fail(ISO_ERR_SHAPE, "hidden=%d must be a positive multiple of 8", c->hidden);
    if (c->ffn < 8 || c->ffn % 8) return fail(ISO_ERR_SHAPE, "ffn=%d must be a positive multiple of 8", c->ffn);
    if (c->head_dim != 64 && c->head_dim != 128) return fail(ISO_ERR_SHAPE, "head_dim=%d must be 64 or 128", c->head_dim);
    if (c->n_q_heads < 1 || c->n_kv_heads < 1) return fail(ISO_ERR_SHAPE, "head counts must be positive");
    if (c->n_q_heads % c->n_kv_heads) return fail(ISO_ERR_SHAPE, "n_q_heads=%d is not a multiple of n_kv_heads=%d", c->n_q_heads, c->n_kv_heads);
    if (c->max_seq < 1) return fail(ISO_ERR_SHAPE, "max_seq=%d must be positive", c->max_seq);
    if (!(c->rms_eps >= 0.f)) return fail(ISO_ERR_SHAPE, "rms_eps must be >= 0");
    if (!(c->rope_base > 1.f)) return fail(ISO_ERR_SHAPE, "rope_base must be > 1");
    return ISO_OK;
}

// True while `s` is recording into a HIP graph (or when that cannot be told).
bool capturing(hipStream_t s) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    return hipStreamIsCapturing(s, &st) != hipSuccess || st != hipStreamCaptureStatusNone;
}

// Brackets one launch with a pair of events in the launch's own stream when timing is on (never inside a graph
// capture: the events of a replayed graph have no elapsed time to read).
struct Timed {
    iso_ctx *c;
    int idx;
    hipStream_t s;
    Timed(iso_ctx *ctx, int kind, hipStream_t stream) : c(ctx), idx(-1), s(stream) {
        if (!c->timing || c->n_tev >= ISO_MAX_TIMED || capturing(stream)) return;
        if (c->n_tev == c->n_tev_created) {
            if (hipEventCreate(&c->tev0[c->n_tev]) != hipSuccess) return;
            if (hipEventCreate(&c->tev1[c->n_tev]) != hipSuccess) { (void)hipEventDestroy(c->tev0[c->n_tev]); return; }
            c->n_tev_created++;
        }
        idx = c->n_tev++;
        c->tkind[idx] = kind;
        (void)hipEventRecord(c->tev0[idx], s);
    }
    ~Timed() {
        if (idx >= 0) (void)hipEventRecord(c->tev1[idx], s);
    }
};

inline char *at(void *base, size_t row, size_t width, size_t e) { return (char *)base + row * width * e; }
inline const char *at(const void *base, size_t row, size_t width, size_t e) { return (const char *)base + row * width * e; }

// Stream-K workspace for a launch on stream s: the context owns one per stream of its own, so launches that share
// a workspace are ordered; a foreign stream gets none and takes the plain kernels.  Neither does a stream that is
// recording into a HIP graph: every stream-K launch carries its own sequence number (the flags of the workspace are
// never reset), and a replayed graph would present the number of its first run again.
iso_sk_ws *sk_for(iso_ctx *ctx, hipStream_t s) {
    if (((ctx->flags & ISO_FLAG_NO_STREAMK) || ctx->sk_hold) && ((ctx->flags >> 8) & 7) != 6) return nullptr;
    if (capturing(s)) return nullptr;
    if (s == ctx->stream[0] && ctx->sk[0].base) return &ctx->sk[0];
    if (s == ctx->stream[1] && ctx->sk[1].base) return &ctx->sk[1];
    return nullptr;
}

// Key-split attention workspace for a launch on stream s: one per stream of the context's own, none for others.
constexpr int ATTN_SLOTS = 512, ATTN_BLOCKS = 512;

const iso_attn_ws *attn_ws_for(const iso_ctx *ctx, hipStream_t s) {
    if (s == ctx->stream[0] && ctx->aws[0].part) return &ctx->aws[0];
    if (s == ctx->stream[1] && ctx->aws[1].part) return &ctx->aws[1];
    for (int k = 2; k < ISO_MAX_CHUNKS; ++k)
        if (ctx->xstream[k] && s == ctx->xstream[k] && ctx->aws[k].part) return &ctx->aws[k];
    return nullptr;
}

// Allocates one key-split attention workspace (counters zeroed; the caller synchronises the device afterwards).
hipError_t attn_ws_create(iso_attn_ws *ws) {
    ws->max_slots = ATTN_SLOTS;
    ws->max_blocks = ATTN_BLOCKS;
    hipError_t e = hipMalloc((void **)&ws->part, (size_t)ATTN_SLOTS * iso_attn_part_bytes());
    if (e == hipSuccess) e = hipMalloc((void **)&ws->cnt, ATTN_BLOCKS * sizeof(unsigned));
    if (e == hipSuccess) e = hipMemset(ws->cnt, 0, ATTN_BLOCKS * sizeof(unsigned));
    if (e != hipSuccess) {       // all or nothing: a workspace with one of its two buffers must never reach a launch
        if (ws->part) (void)hipFree(ws->part);
        if (ws->cnt) (void)hipFree(ws->cnt);
        ws->part = nullptr;
        ws->cnt = nullptr;
    }
    return e;
}

// Row ranges of a GEMM cut into ctx->gemm_segments launches (Section 3.2: several launches per matrix product,
// so that compute units given back by a finishing transfer are picked up at the next launch).  Segments are
// multiples of 256 rows; a product with fewer than 256 rows per segment is not cut.
template <typename F> int for_segments(const iso_ctx *ctx, int M, F &&launch) {
    int segs = ctx->gemm_segments > 1 ? ctx->gemm_segments : 1;
    if (M < 256 * segs) segs = 1;
    const int per = ((M + segs - 1) / segs + 255) / 256 * 256;
    for (int lo = 0; lo < M; lo += per) {
        const int rc = launch(lo, M - lo < per ? M - lo : per);
        if (rc != ISO_OK) return rc;
    }
    return ISO_OK;
}

#define LAUNCH_TRY(kind, stream, expr, what)                                                       \
    do {                                                                                           \
        Timed t_(ctx, kind, stream);                                                               \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return fail(ISO_ERR_HIP, "%s launch: %s", what, hipGetErrorString(e_)); \
    } while (0)

// FP8 operands of one projection of the layer: the FP8 weight and its scales, and the token row the activation
// rows start at (their FP8 copy goes to that chunk's own region of the workspace).  w8 == NULL: bf16 path.
struct F8Arg {
    const void *w8 = nullptr;
    const float *sw = nullptr;
    int row0 = 0;
    bool prequant = false;   // the producer of the activation has already left its FP8 codes and scales there
};

bool use_fp8(const iso_ctx *ctx, const F8Arg &f8, int M, int N, int K) {
    return (ctx->flags & ISO_FLAG_FP8_GEMM) && ctx->cfg.dtype == ISO_BF16 && f8.w8 && f8.sw &&
           iso_gemm_fp8_supported(M, N, K);
}

int gemm(iso_ctx *ctx, int kind, const void *a, const void *w, void *c, int M, int N, int K, hipStream_t s,
         const F8Arg &f8 = F8Arg()) {
    const size_t e_ = ctx->elt;
    if (use_fp8(ctx, f8, M, N, K)) {
        unsigned char *a8 = ctx->a8 + (size_t)f8.row0 * ctx->a8_pitch;
        float *sa = ctx->a8s + f8.row0;
        if (!f8.prequant)
            LAUNCH_TRY(ISO_K_QUANT, s, iso_launch_quant_rows_fp8(a, a8, sa, M, K, s), "fp8 row quantiser");
        Timed t_(ctx, kind, s);
        return for_segments(ctx, M, [&](int lo, int n) {
            hipError_t e = iso_launch_gemm_fp8(a8 + (size_t)lo * K, sa + lo, f8.w8, f8.sw, (char *)c + (size_t)lo * N * e_,
                                               n, N, K, (ctx->flags >> 8) & 15, sk_for(ctx, s), s);
            if (e != hipSuccess) return fail(ISO_ERR_HIP, "fp8 gemm launch (M=%d N=%d K=%d): %s", n, N, K, hipGetErrorString(e));
            return (int)ISO_OK;
        });
    }
    Timed t_(ctx, kind, s);
    return for_segments(ctx, M, [&](int lo, int n) {
        const void *ar = (const char *)a + (size_t)lo * K * e_;
        void *cr = (char *)c + (size_t)lo * N * e_;
        hipError_t e;
        const bool mfma = ctx->cfg.dtype == ISO_BF16 && !(ctx->flags & ISO_FLAG_SIMPLE_GEMM);
        if (mfma && !(ctx->flags & ISO_FLAG_GEMM_STAGED) && iso_gemm_bf16_dtl_supported(n, N, K))
            e = iso_launch_gemm_bf16_dtl(ar, w, cr, n, N, K, (ctx->flags >> 8) & 15, sk_for(ctx, s), s);
        else if (mfma && iso_gemm_bf16_mfma_supported(n, N, K))
            e = iso_launch_gemm_bf16_mfma(ar, w, cr, n, N, K, s);
        else
            e = iso_launch_gemm_simple(ctx->cfg.dtype, ar, w, cr, n, N, K, s);
        if (e != hipSuccess)
            return fail(ISO_ERR_HIP, "gemm launch (M=%d N=%d K=%d): %s", n, N, K, hipGetErrorString(e));
        return (int)ISO_OK;
    });
}

int attention(iso_ctx *ctx, const void *q, int q_stride, const void *kc, const void *vc, void *out, int Tc,
              int q_offset, int kv_len, hipStream_t s) {
    const iso_cfg &c = ctx->cfg;
    Timed t_(ctx, ISO_K_ATTN, s);
    hipError_t e;
    const bool mfma = c.dtype == ISO_BF16 && !(ctx->flags & ISO_FLAG_SIMPLE_ATTN);
    if (mfma && !(ctx->flags & ISO_FLAG_ATTN_STAGED) && iso_attn_bf16_dtl_supported(c.head_dim, kv_len, c.n_kv_heads))
        e = iso_launch_attn_bf16_dtl(q, kc, vc, out, Tc, q_offset, kv_len, c.n_q_heads, c.n_kv_heads, c.head_dim, q_stride,
                                     (ctx->flags >> 12) & 3, (ctx->flags >> 14) & 7, attn_ws_for(ctx, s), s);
    else if (mfma && iso_attn_bf16_mfma_supported(c.head_dim))
        e = iso_launch_attn_bf16_mfma(q, kc, vc, out, Tc, q_offset, kv_len, c.n_q_heads, c.n_kv_heads, c.head_dim, q_stride, s);
    else
        e = iso_launch_attn_simple(c.dtype, q, kc, vc, out, Tc, q_offset, kv_len, c.n_q_heads, c.n_kv_heads, c.head_dim, q_stride, s);
    if (e != hipSuccess) return fail(ISO_ERR_HIP, "attention launch: %s", hipGetErrorString(e));
    return ISO_OK;
}

#define ISO_TRY(expr)              \
    do {                           \
        int r_ = (expr);           \
        if (r_ != ISO_OK) return r_; \
    } while (0)

// The stream-K GEMM reports a wait that ran out through a pinned host word.  It stays set until iso_sync has
// returned the error: the layer, attention and projection entry points look at it before they enqueue anything, so
// that a pass whose results are invalid is not followed by hundreds of launches that build on them.
int sk_status(const iso_ctx *ctx) {
    if (ctx->sk[0].err && *(volatile unsigned *)ctx->sk[0].err)
        return fail(ISO_ERR_HIP, "stream-K GEMM: a wait for a partial tile ran out in an earlier launch; results since "
                                 "the last iso_sync are invalid (iso_sync reports and clears this)");
    return ISO_OK;
}


// Communication point of one chunk: nothing, the [n, H] partial as it is, or its int8 codes + row scales.
// `which` = 0 after o_proj, 1 after down; the host sink keeps the two points apart.
int comm_point(iso_ctx *ctx, int comm, int which, int lo, int n, hipStream_t s) {
    const iso_cfg &c = ctx->cfg;
    const size_t e = ctx->elt, H = (size_t)c.hidden;
    char *partr = (char *)(which ? ctx->part_m : ctx->part) + (size_t)lo * H * e;
    char *sink = (char *)ctx->host_sink + (size_t)which * c.max_seq * H * e;
    if (comm == ISO_COMM_D2H) {
        Timed t_(ctx, ISO_K_COMM, s);
        HIP_TRY(hipMemcpyAsync(sink + (size_t)lo * H * e, partr, (size_t)n * H * e, hipMemcpyDeviceToHost, s));
    } else if (comm == ISO_COMM_D2H_INT8) {
        signed char *q = ctx->q8 + (size_t)lo * (H + 16);
        LAUNCH_TRY(ISO_K_QUANT, s, iso_launch_quant_rows(c.dtype, partr, q, n, (int)H, s), "quantise");
        Timed t_(ctx, ISO_K_COMM, s);
        HIP_TRY(hipMemcpyAsync(sink + (size_t)lo * (H + 16), q, (size_t)n * (H + 16), hipMemcpyDeviceToHost, s));
    }
    return ISO_OK;
}

// One chunk = token rows [lo, lo + n).
struct Chunk {
    int lo, n;
    hipStream_t s;
};

// Attention block of one chunk.  `first_norm_delta`: when not NULL the block starts with the residual add
// left over from the previous layer's MLP block (x += delta) fused into this norm.
int attn_block_head(iso_ctx *ctx, const iso_weights *w, void *x, void *kc, void *vc, const Chunk &ck,
                    bool add_prev_partial) {
    const iso_cfg &c = ctx->cfg;
    const size_t e = ctx->elt;
    const int H = c.hidden, NQKV = n_qkv(c);
    char *xr = at(x, ck.lo, H, e);
    char *yr = at(ctx->y, ck.lo, H, e);
    char *qkvr = at(ctx->qkv, ck.lo, NQKV, e);
    // 8-bit projection: the norm writes the FP8 codes and row scales of y itself, y is never stored
    F8Arg f8{w->w_qkv_f8, w->s_qkv, ck.lo};
    f8.prequant = use_fp8(ctx, f8, ck.n, NQKV, H) && iso_rmsnorm_fp8_supported(H);
    unsigned char *a8 = ctx->a8 + (size_t)ck.lo * ctx->a8_pitch;
    float *sa = ctx->a8s + ck.lo;
    if (add_prev_partial) {   // x = (x + previous layer's attention partial) + its MLP partial, y = norm(x)
        const char *pa = at(ctx->part, ck.lo, H, e), *pm = at(ctx->part_m, ck.lo, H, e);
        if (f8.prequant)
            LAUNCH_TRY(ISO_K_RESID_NORM, ck.s, iso_launch_rmsnorm_fp8(xr, pa, pm, xr, w->g_attn, a8, sa, ck.n, H, c.rms_eps, ck.s),
                       "residual+rmsnorm+fp8");
        else
            LAUNCH_TRY(ISO_K_RESID_NORM, ck.s, iso_launch_rmsnorm(c.dtype, xr, pa, pm, xr, w->g_attn, yr, ck.n, H, c.rms_eps, ck.s),
                       "residual+rmsnorm");
    } else if (f8.prequant) {
        LAUNCH_TRY(ISO_K_RMSNORM, ck.s, iso_launch_rmsnorm_fp8(xr, nullptr, nullptr, nullptr, w->g_attn, a8, sa, ck.n, H, c.rms_eps, ck.s),
                   "rmsnorm+fp8");
    } else {
        LAUNCH_TRY(ISO_K_RMSNORM, ck.s, iso_launch_rmsnorm(c.dtype, xr, nullptr, nullptr, nullptr, w->g_attn, yr, ck.n, H, c.rms_eps, ck.s), "rmsnorm");
    }
    // bf16 layers with head_dim 128: rotary embedding and KV-cache write ride in the projection's epilogue whenever
    // the launch rule picks a kernel whose waves own whole heads (the 256-wide tile or its stream-K launch)
    const bool dtl = c.dtype == ISO_BF16 && c.head_dim == 128 && !use_fp8(ctx, f8, ck.n, NQKV, H) &&
                     !(ctx->flags & (ISO_FLAG_SIMPLE_GEMM | ISO_FLAG_GEMM_STAGED | ISO_FLAG_NO_FUSE)) &&
                     iso_gemm_bf16_dtl_supported(ck.n, NQKV, H);
    if (dtl) {
        const int segs = (ctx->gemm_segments > 1 && ck.n >= 256 * ctx->gemm_segments) ? ctx->gemm_segments : 1;
        const int per = ((ck.n + segs - 1) / segs + 255) / 256 * 256;
        bool all_fusable = true;                    // every segment must resolve to a head-owning variant
        for (int lo = 0; lo < ck.n; lo += per) {
            const int v = iso_gemm_bf16_dtl_resolve(std::min(per, ck.n - lo), NQKV, H, (ctx->flags >> 8) & 15, sk_for(ctx, ck.s));
            all_fusable = all_fusable && (v == 1 || v == 6);
        }
        if (all_fusable) {
            Timed t_(ctx, ISO_K_GEMM_QKV, ck.s);
            return for_segments(ctx, ck.n, [&](int lo, int n) {
                iso_sk_ws *sk = sk_for(ctx, ck.s);
                const int v = iso_gemm_bf16_dtl_resolve(n, NQKV, H, (ctx->flags >> 8) & 15, sk);
                hipError_t e_ = iso_launch_gemm_qkv_rope_bf16(yr + (size_t)lo * H * e, w->w_qkv, qkvr + (size_t)lo * NQKV * e, n,
                                                              NQKV, H, v, sk, ctx->rope_cos, ctx->rope_sin, kc, vc, ck.lo + lo,
                                                              c.n_q_heads, c.n_kv_heads, ck.s);
                if (e_ != hipSuccess) return fail(ISO_ERR_HIP, "qkv+rope launch: %s", hipGetErrorString(e_));
                return (int)ISO_OK;
            });
        }
    }
    ISO_TRY(gemm(ctx, ISO_K_GEMM_QKV, yr, w->w_qkv, qkvr, ck.n, NQKV, H, ck.s, f8));
    LAUNCH_TRY(ISO_K_ROPE_KV, ck.s, iso_launch_rope_kv(c.dtype, qkvr, kc, vc, ctx->rope_cos, ctx->rope_sin, ck.n, ck.lo, c.n_q_heads,
                                  c.n_kv_heads, c.head_dim, ck.s), "rope+kv");
    return ISO_OK;
}

int attn_block_tail(iso_ctx *ctx, const iso_weights *w, void *kc, void *vc, const Chunk &ck, int comm,
                    hipEvent_t after_compute) {
    const iso_cfg &c = ctx->cfg;
    const size_t e = ctx->elt;
    const int H = c.hidden, NQKV = n_qkv(c), NQD = c.n_q_heads * c.head_dim;
    char *qkvr = at(ctx->qkv, ck.lo, NQKV, e);
    char *attnr = at(ctx->attn, ck.lo, NQD, e);
    char *partr = at(ctx->part, ck.lo, H, e);
    ISO_TRY(attention(ctx, qkvr, NQKV, kc, vc, attnr, ck.n, ck.lo, ck.lo + ck.n, ck.s));
    ISO_TRY(gemm(ctx, ISO_K_GEMM_O, attnr, w->w_o, partr, ck.n, H, NQD, ck.s, F8Arg{w->w_o_f8, w->s_o, ck.lo}));
    if (after_compute) HIP_TRY(hipEventRecord(after_compute, ck.s));
    return comm_point(ctx, comm, 0, ck.lo, ck.n, ck.s);
}

int mlp_block(iso_ctx *ctx, const iso_weights *w, void *x, const Chunk &ck, int comm) {
    const iso_cfg &c = ctx->cfg;
    const size_t e = ctx->elt;
    const int H = c.hidden, F = c.ffn;
    char *xr = at(x, ck.lo, H, e);
    char *yr = at(ctx->y, ck.lo, H, e);
    const char *pa = at(ctx->part, ck.lo, H, e);
    char *partr = at(ctx->part_m, ck.lo, H, e);
    char *gur = at(ctx->gu, ck.lo, 2 * (size_t)F, e);
    char *actr = at(ctx->act, ck.lo, F, e);
    // y = norm(x1), x1 = x + (attention partial) held in registers only: the kernel that closes the layer rebuilds
    // it from the same two tensors, so the mid-layer residual is never rounded and never stored.
    // With an 8-bit gate/up projection the norm leaves the FP8 codes and row scales of y instead of y.
    F8Arg f8gu{w->w_gate_up_f8, w->s_gate_up, ck.lo};
    f8gu.prequant = use_fp8(ctx, f8gu, ck.n, 2 * F, H) && iso_rmsnorm_fp8_supported(H);
    unsigned char *a8 = ctx->a8 + (size_t)ck.lo * ctx->a8_pitch;
    float *sa = ctx->a8s + ck.lo;
    if (f8gu.prequant)
        LAUNCH_TRY(ISO_K_RESID_NORM, ck.s, iso_launch_rmsnorm_fp8(xr, pa, nullptr, nullptr, w->g_mlp, a8, sa, ck.n, H, c.rms_eps, ck.s),
                   "residual+rmsnorm+fp8");
    else
        LAUNCH_TRY(ISO_K_RESID_NORM, ck.s, iso_launch_rmsnorm(c.dtype, xr, pa, nullptr, nullptr, w->g_mlp, yr, ck.n, H, c.rms_eps, ck.s),
                   "residual+rmsnorm");
    const bool fused = c.dtype == ISO_BF16 && !(ctx->flags & (ISO_FLAG_SIMPLE_GEMM | ISO_FLAG_GEMM_STAGED | ISO_FLAG_NO_FUSE)) &&
                       iso_gemm_swiglu_bf16_supported(ck.n, F, H);
    if (fused && use_fp8(ctx, f8gu, ck.n, 2 * F, H)) {
        if (!f8gu.prequant)
            LAUNCH_TRY(ISO_K_QUANT, ck.s, iso_launch_quant_rows_fp8(yr, a8, sa, ck.n, H, ck.s), "fp8 row quantiser");
        Timed t_(ctx, ISO_K_GEMM_GATE_UP, ck.s);
        ISO_TRY(for_segments(ctx, ck.n, [&](int lo, int n) {
            hipError_t e_ = iso_launch_gemm_swiglu_fp8(a8 + (size_t)lo * H, sa + lo, f8gu.w8, f8gu.sw, actr + (size_t)lo * F * e,
                                                       n, F, H, (ctx->flags >> 8) & 15, sk_for(ctx, ck.s), ck.s);
            if (e_ != hipSuccess) return fail(ISO_ERR_HIP, "fp8 gate/up+swiglu launch: %s", hipGetErrorString(e_));
            return (int)ISO_OK;
        }));
    } else if (fused) {   // gate/up projection with the activation in its epilogue: the [Tc, 2F] tensor never exists
        Timed t_(ctx, ISO_K_GEMM_GATE_UP, ck.s);
        ISO_TRY(for_segments(ctx, ck.n, [&](int lo, int n) {
            hipError_t e_ = iso_launch_gemm_swiglu_bf16(yr + (size_t)lo * H * e, w->w_gate_up, actr + (size_t)lo * F * e, n, F, H,
                                                        (ctx->flags >> 8) & 15, sk_for(ctx, ck.s), ck.s);
            if (e_ != hipSuccess) return fail(ISO_ERR_HIP, "gate/up+swiglu launch: %s", hipGetErrorString(e_));
            return (int)ISO_OK;
        }));
    } else {
        ISO_TRY(gemm(ctx, ISO_K_GEMM_GATE_UP, yr, w->w_gate_up, gur, ck.n, 2 * F, H, ck.s, f8gu));
        LAUNCH_TRY(ISO_K_SWIGLU, ck.s, iso_launch_swiglu(c.dtype, gur, actr, ck.n, F, ck.s), "swiglu");
    }
    ISO_TRY(gemm(ctx, ISO_K_GEMM_DOWN, actr, w->w_down, partr, ck.n, H, F, ck.s, F8Arg{w->w_down_f8, w->s_down, ck.lo}));
    return comm_point(ctx, comm, 1, ck.lo, ck.n, ck.s);
}

int final_residual(iso_ctx *ctx, void *x, const Chunk &ck) {
    const iso_cfg &c = ctx->cfg;
    const size_t e = ctx->elt;
    char *xr = at(x, ck.lo, c.hidden, e);
    LAUNCH_TRY(ISO_K_RESIDUAL, ck.s, iso_launch_rmsnorm(c.dtype, xr, at(ctx->part, ck.lo, c.hidden, e), at(ctx->part_m, ck.lo, c.hidden, e),
               xr, nullptr, nullptr, ck.n, c.hidden, c.rms_eps, ck.s), "residual");
    return ISO_OK;
}

int check_layer_args(iso_ctx *ctx, const iso_weights *layers, int n_layers, void *x, void *kc, void *vc, int T,
                     int split, int comm, int sched) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!layers || !x || !kc || !vc) return fail(ISO_ERR_NULL, "weights, x, k_cache and v_cache must be non-NULL");
    if (n_layers < 1) return fail(ISO_ERR_SHAPE, "n_layers=%d must be positive", n_layers);
    for (int l = 0; l < n_layers; ++l) {
        const iso_weights &w = layers[l];
        if (!w.w_qkv || !w.w_o || !w.w_gate_up || !w.w_down || !w.g_attn || !w.g_mlp)
            return fail(ISO_ERR_NULL, "layer %d has a NULL weight pointer", l);
    }
    if (T < 1) return fail(ISO_ERR_SHAPE, "T=%d must be positive", T);
    if (T > ctx->cfg.max_seq) return fail(ISO_ERR_WORKSPACE, "T=%d exceeds max_seq=%d", T, ctx->cfg.max_seq);
    if (split < 0 || split > T) return fail(ISO_ERR_SPLIT, "split=%d outside [0, %d]", split, T);
    if (comm != ISO_COMM_NONE && comm != ISO_COMM_D2H && comm != ISO_COMM_D2H_INT8)
        return fail(ISO_ERR_SHAPE, "unknown comm mode %d", comm);
    if (sched != ISO_SCHED_OVERLAP && sched != ISO_SCHED_SERIAL && sched != ISO_SCHED_STREAM_PER_CHUNK)
        return fail(ISO_ERR_SHAPE, "unknown schedule %d", sched);
    return sk_status(ctx);
}

// Extra streams for ISO_SCHED_STREAM_PER_CHUNK, created on first use (default priority, like every stream here).
int chunk_streams(iso_ctx *ctx, int nc, hipStream_t *out) {
    out[0] = ctx->stream[0];
    out[1] = ctx->stream[1];
    for (int k = 2; k < nc; ++k) {
        if (!ctx->xstream[k]) {
            HIP_TRY(hipStreamCreateWithFlags(&ctx->xstream[k], hipStreamNonBlocking));
            if (ctx->cfg.dtype == ISO_BF16 && !ctx->aws[k].part) {   // same launch choices as on the caller's streams
                HIP_TRY(attn_ws_create(&ctx->aws[k]));
                HIP_TRY(hipDeviceSynchronize());
            }
        }
        out[k] = ctx->xstream[k];
    }
    return ISO_OK;
}

// edges[0..nc]: chunk c is rows [edges[c], edges[c+1]).
int run_stack(iso_ctx *ctx, const iso_weights *layers, int n_layers, void *x, void *k_caches, void *v_caches,
              const int *edges, int nc, int comm, int sched) {
    const iso_cfg &c = ctx->cfg;
    const size_t cache_bytes = (size_t)c.max_seq * c.n_kv_heads * c.head_dim * ctx->elt;
    const bool overlap = nc > 1 && sched != ISO_SCHED_SERIAL && ctx->stream[1] != ctx->stream[0];
    const bool per_chunk = overlap && sched == ISO_SCHED_STREAM_PER_CHUNK;
    hipStream_t st[ISO_MAX_CHUNKS];
    for (int k = 0; k < ISO_MAX_CHUNKS; ++k) st[k] = ctx->stream[0];
    if (per_chunk) ISO_TRY(chunk_streams(ctx, nc, st));
    else if (overlap) for (int k = 0; k < nc; ++k) st[k] = ctx->stream[k & 1];
    const int n_streams = per_chunk ? nc : (overlap ? 2 : 1);
    Chunk ch[ISO_MAX_CHUNKS];
    for (int k = 0; k < nc; ++k) ch[k] = Chunk{edges[k], edges[k + 1] - edges[k], st[k]};

    // Stream-K takes every compute unit for one GEMM.  That pays while the other chunk's stream mostly waits for
    // its bf16 transfers; when two chunks compute side by side most of the time (no transfers, or the halved int8
    // ones) the tile-per-workgroup launches share the chip better (measured: 4-7 % either way).
    struct SkHold {
        iso_ctx *c;
        ~SkHold() { c->sk_hold = 0; }
    } sk_hold_{ctx};
    ctx->sk_hold = overlap && comm != ISO_COMM_D2H;
    // With transfers to hide and chunks long enough to fill the chip on their own (measured: from about 1024 rows),
    // the attention blocks are chained whole; otherwise the chunks' independent front parts run side by side.
    int min_rows = edges[1] - edges[0];
    for (int k = 1; k < nc; ++k) min_rows = std::min(min_rows, edges[k + 1] - edges[k]);
    const bool chain_blocks = overlap && comm != ISO_COMM_NONE && min_rows >= 1024;
    if (overlap) {   // fork: the other streams start after whatever produced x in stream0
        HIP_TRY(hipEventRecord(ctx->ev_fork, st[0]));
        for (int k = 1; k < n_streams; ++k) HIP_TRY(hipStreamWaitEvent(st[k], ctx->ev_fork, 0));
    }
    for (int l = 0; l < n_layers; ++l) {
        const iso_weights *w = &layers[l];
        void *kc = (char *)k_caches + (size_t)l * cache_bytes;
        void *vc = (char *)v_caches + (size_t)l * cache_bytes;
        if (chain_blocks) {
            // Whole attention blocks one after the other in chunk order: chunk k starts once chunk k-1's output
            // projection has been issued to the matrix cores, so chunk 0 has the chip to itself, its transfer starts
            // as early as it can and runs under chunk 1's block (the order of the paper's Figure 1(d)).
            for (int k = 0; k < nc; ++k) {
                if (k > 0) HIP_TRY(hipStreamWaitEvent(ch[k].s, ctx->ev_kv[k - 1], 0));
                ISO_TRY(attn_block_head(ctx, w, x, kc, vc, ch[k], l > 0));
                ISO_TRY(attn_block_tail(ctx, w, kc, vc, ch[k], comm, k + 1 < nc ? ctx->ev_kv[k] : nullptr));
            }
        } else {
            // Heads first: the norm/QKV/RoPE of a chunk do not depend on any other chunk.  A chunk's attention then
            // waits for an event of its predecessor, and through it for every earlier chunk:
            //  * two streams: the event says the predecessor's K/V rows are in the cache; the predecessor sits on
            //    the other stream, behind ITS predecessor's head on this one;
            //  * one stream per chunk: the event follows the predecessor's output projection, so the attention
            //    kernels run one after the other in chunk order.
            for (int k = 0; k < nc; ++k) {
                ISO_TRY(attn_block_head(ctx, w, x, kc, vc, ch[k], l > 0));
                if (overlap && !per_chunk && k + 1 < nc) HIP_TRY(hipEventRecord(ctx->ev_kv[k], ch[k].s));
            }
            for (int k = 0; k < nc; ++k) {
                if (overlap && k > 0) HIP_TRY(hipStreamWaitEvent(ch[k].s, ctx->ev_kv[k - 1], 0));
                ISO_TRY(attn_block_tail(ctx, w, kc, vc, ch[k], comm, (per_chunk && k + 1 < nc) ? ctx->ev_kv[k] : nullptr));
            }
        }
        for (int k = 0; k < nc; ++k) ISO_TRY(mlp_block(ctx, w, x, ch[k], comm));
    }
    for (int k = 0; k < nc; ++k) ISO_TRY(final_residual(ctx, x, ch[k]));
    if (overlap) {   // join: later work in stream0 sees every chunk
        for (int k = 1; k < n_streams; ++k) {
            HIP_TRY(hipEventRecord(ctx->ev_join[k], st[k]));
            HIP_TRY(hipStreamWaitEvent(st[0], ctx->ev_join[k], 0));
        }
    }
    return ISO_OK;
}

int run_split(iso_ctx *ctx, const iso_weights *layers, int n_layers, void *x, void *k_caches, void *v_caches, int T,
              int split, int comm, int sched) {
    const bool two = split > 0 && split < T;
    const int edges[3] = {0, two ? split : T, T};
    return run_stack(ctx, layers, n_layers, x, k_caches, v_caches, edges, two ? 2 : 1, comm, sched);
}

}  // namespace

extern "C" {

const char *iso_last_error(void) { return g_err; }

int iso_validate_cfg(const iso_cfg *cfg) { return check_cfg(cfg); }

int iso_plan_chunks(const iso_cfg *cfg, int T, int split, iso_plan *out) {
    ISO_TRY(check_cfg(cfg));
    if (!out) return fail(ISO_ERR_NULL, "out is NULL");
    if (T < 1) return fail(ISO_ERR_SHAPE, "T=%d must be positive", T);
    if (T > cfg->max_seq) return fail(ISO_ERR_WORKSPACE, "T=%d exceeds max_seq=%d", T, cfg->max_seq);
    if (split < 0 || split > T) return fail(ISO_ERR_SPLIT, "split=%d outside [0, %d]", split, T);
    memset(out, 0, sizeof(*out));
    const bool two = split > 0 && split < T;
    out->n_chunks = two ? 2 : 1;
    out->q_offset[0] = 0;
    out->n_tokens[0] = two ? split : T;
    out->kv_len[0] = out->n_tokens[0];
    if (two) {
        out->q_offset[1] = split;
        out->n_tokens[1] = T - split;
        out->kv_len[1] = T;
    }
    for (int k = 0; k < out->n_chunks; ++k)
        out->comm_bytes[k] = (size_t)out->n_tokens[k] * cfg->hidden * elt_size(cfg->dtype);
    out->workspace_bytes = ws_layout(*cfg).total;
    return ISO_OK;
}

int iso_plan_chunk_count(const iso_cfg *cfg, int T, int *n_chunks) {
    ISO_TRY(check_cfg(cfg));
    if (!n_chunks) return fail(ISO_ERR_NULL, "n_chunks is NULL");
    if (T < 1) return fail(ISO_ERR_SHAPE, "T=%d must be positive", T);
    if (T > cfg->max_seq) return fail(ISO_ERR_WORKSPACE, "T=%d exceeds max_seq=%d", T, cfg->max_seq);
    int n = T / 2048;
    if (n < 2) n = 2;
    if (n > ISO_MAX_CHUNKS) n = ISO_MAX_CHUNKS;
    if (T < 512) n = 1;
    *n_chunks = n;
    return ISO_OK;
}

int iso_plan_split(const iso_cfg *cfg, int T, int n_chunks, double attn_flop_cost, int *bounds) {
    ISO_TRY(check_cfg(cfg));
    if (T < 1) return fail(ISO_ERR_SHAPE, "T=%d must be positive", T);
    if (T > cfg->max_seq) return fail(ISO_ERR_WORKSPACE, "T=%d exceeds max_seq=%d", T, cfg->max_seq);
    if (n_chunks < 1 || n_chunks > ISO_MAX_CHUNKS || n_chunks > T)
        return fail(ISO_ERR_SHAPE, "n_chunks=%d outside [1, min(T, %d)]", n_chunks, ISO_MAX_CHUNKS);
    if (n_chunks > 1 && !bounds) return fail(ISO_ERR_NULL, "bounds is NULL");
    const double r = attn_flop_cost > 0.0 ? attn_flop_cost : 3.0;
    const double nq = cfg->n_q_heads, nkv = cfg->n_kv_heads, d = cfg->head_dim, H = cfg->hidden, F = cfg->ffn;
    // cumulative cost of the first t positions: proj * t + a * t * (t + 1), a = r * 2 * nq * d
    const double proj = 2.0 * H * (nq + 2.0 * nkv) * d + 2.0 * H * nq * d + 6.0 * H * F;
    const double a = r * 2.0 * nq * d;
    const double total = proj * T + a * (double)T * (T + 1.0);
    const int align = T >= 256 * n_chunks ? 128 : 1;
    int prev = 0;
    for (int j = 1; j < n_chunks; ++j) {
        const double target = total * j / n_chunks;
        const double b = proj + a;
        const double t = (sqrt(b * b + 4.0 * a * target) - b) / (2.0 * a);    // a > 0 for every valid cfg
        long cut = lround(t / align) * align;
        if (cut <= prev) cut = prev + align;              // at least one (aligned) step per chunk ...
        const long last = (long)T - (long)(n_chunks - j);
        if (cut > last) cut = last;                       // ... and room for the chunks behind
        if (cut <= prev) cut = prev + 1;
        bounds[j - 1] = (int)cut;
        prev = (int)cut;
    }
    return ISO_OK;
}

int iso_create(iso_ctx **out, const iso_cfg *cfg, void *stream0, void *stream1) {
    if (!out) return fail(ISO_ERR_NULL, "out is NULL");
    *out = nullptr;
    ISO_TRY(check_cfg(cfg));
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    iso_ctx *ctx = new iso_ctx();
    memset(ctx, 0, sizeof(*ctx));
    ctx->cfg = *cfg;
    ctx->device = dev;
    ctx->stream[0] = (hipStream_t)stream0;
    ctx->stream[1] = (hipStream_t)stream1;
    ctx->elt = elt_size(cfg->dtype);
    ctx->tev0 = new hipEvent_t[ISO_MAX_TIMED]();
    ctx->tev1 = new hipEvent_t[ISO_MAX_TIMED]();
    ctx->tkind = new int[ISO_MAX_TIMED]();
    const WsLayout l = ws_layout(*cfg);
    const size_t half = (size_t)cfg->head_dim / 2;
    const size_t table = (size_t)cfg->max_seq * half;
    int rc = ISO_OK;
    auto hip_ok = [&](hipError_t e, const char *what) {
        if (e != hipSuccess && rc == ISO_OK) rc = fail(ISO_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
        return e == hipSuccess;
    };
    do {
        if (!hip_ok(hipMalloc(&ctx->ws, l.total), "hipMalloc(workspace)")) break;
        ctx->ws_bytes = l.total;
        char *b = (char *)ctx->ws;
        ctx->y = b + l.y; ctx->qkv = b + l.qkv; ctx->attn = b + l.attn;
        ctx->part = b + l.part; ctx->part_m = b + l.part_m; ctx->gu = b + l.gu; ctx->act = b + l.act;
        ctx->q8 = (signed char *)(b + l.q8);
        ctx->a8 = (unsigned char *)(b + l.a8);
        ctx->a8s = (float *)(b + l.a8s);
        ctx->a8_pitch = l.a8_pitch;
        if (!hip_ok(hipMalloc((void **)&ctx->rope_cos, table * sizeof(float)), "hipMalloc(rope cos)")) break;
        if (!hip_ok(hipMalloc((void **)&ctx->rope_sin, table * sizeof(float)), "hipMalloc(rope sin)")) break;
        {   // rotary table: angles in double on the host, stored as fp32
            std::vector<float> hc(table), hs(table);
            for (size_t i = 0; i < half; ++i) {
                const double inv_freq = pow((double)cfg->rope_base, -2.0 * (double)i / (double)cfg->head_dim);
                for (size_t p = 0; p < (size_t)cfg->max_seq; ++p) {
                    const double ang = (double)p * inv_freq;
                    hc[p * half + i] = (float)cos(ang);
                    hs[p * half + i] = (float)sin(ang);
                }
            }
            if (!hip_ok(hipMemcpy(ctx->rope_cos, hc.data(), table * sizeof(float), hipMemcpyHostToDevice), "copy rope cos")) break;
            if (!hip_ok(hipMemcpy(ctx->rope_sin, hs.data(), table * sizeof(float), hipMemcpyHostToDevice), "copy rope sin")) break;
        }
        if (!hip_ok(hipHostMalloc(&ctx->host_sink, 2 * (size_t)cfg->max_seq * cfg->hidden * ctx->elt, hipHostMallocDefault),
                    "hipHostMalloc(sink)")) break;
        if (cfg->dtype == ISO_BF16) {   // stream-K GEMM workspaces: one per stream, one shared error word
            int cus = 0;
            if (!hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev), "device attribute")) break;
            if (cus > iso_gemm_sk_max_wg()) cus = iso_gemm_sk_max_wg();
            unsigned *err = nullptr;
            if (!hip_ok(hipHostMalloc((void **)&err, 64, hipHostMallocDefault), "hipHostMalloc(stream-K status)")) break;
            *err = 0;
            ctx->sk[0].err = ctx->sk[1].err = err;
            const size_t bytes = iso_gemm_sk_ws_bytes(cus);
            bool ok = true;
            for (int i = 0; i < 2 && ok; ++i) {
                ctx->sk[i].num_wg = cus;
                ctx->sk[i].epoch = 0;
                ok = hip_ok(hipMalloc(&ctx->sk[i].base, bytes), "hipMalloc(stream-K workspace)") &&
                     hip_ok(hipMemset(ctx->sk[i].base, 0, 4096), "hipMemset(stream-K flags)");
            }
            if (!ok) break;
            // key-split attention workspaces: one per stream (both streams may run an attention launch at once)
            for (int i = 0; i < 2 && ok; ++i) ok = hip_ok(attn_ws_create(&ctx->aws[i]), "attention key-split workspace");
            if (!ok) break;
            // the memsets ran on the null stream, which the library's non-blocking streams do not wait for
            if (!hip_ok(hipDeviceSynchronize(), "hipDeviceSynchronize")) break;
            // static workspace of iso_gemm_rowpar_static: address on this device, kernel attributes
            if (!hip_ok(iso_gemm_static_setup(), "static stream-K workspace")) break;
        }
        if (!hip_ok(hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming), "event")) break;
        {
            bool ok = true;
            for (int k = 0; k < ISO_MAX_CHUNKS && ok; ++k)
                ok = hip_ok(hipEventCreateWithFlags(&ctx->ev_join[k], hipEventDisableTiming), "event") &&
                     hip_ok(hipEventCreateWithFlags(&ctx->ev_kv[k], hipEventDisableTiming), "event");
            if (!ok) break;
        }
    } while (0);
    if (rc != ISO_OK) {
        char keep[sizeof(g_err)];
        memcpy(keep, g_err, sizeof(keep));
        iso_destroy(ctx);
        memcpy(g_err, keep, sizeof(keep));
        return rc;
    }
    *out = ctx;
    return ISO_OK;
}

int iso_sync(iso_ctx *ctx) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    HIP_TRY(hipStreamSynchronize(ctx->stream[0]));
    if (ctx->stream[1] != ctx->stream[0]) HIP_TRY(hipStreamSynchronize(ctx->stream[1]));
    if (ctx->sk[0].err && *ctx->sk[0].err) {
        *ctx->sk[0].err = 0;
        return fail(ISO_ERR_HIP, "stream-K GEMM: a wait for a partial tile ran out; results of this pass are invalid");
    }
    return ISO_OK;
}

int iso_destroy(iso_ctx *ctx) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (ctx->ws) {   // only a fully or partly built context has device state to drain
        (void)hipStreamSynchronize(ctx->stream[0]);
        if (ctx->stream[1] != ctx->stream[0]) (void)hipStreamSynchronize(ctx->stream[1]);
        for (int k = 0; k < ISO_MAX_CHUNKS; ++k)
            if (ctx->xstream[k]) (void)hipStreamSynchronize(ctx->xstream[k]);
    }
    // everything is freed either way; the return value says whether the last pass before the teardown was valid
    const int rc = ctx->sk[0].err ? sk_status(ctx) : (int)ISO_OK;
    for (int i = 0; i < ctx->n_tev_created; ++i) {
        (void)hipEventDestroy(ctx->tev0[i]);
        (void)hipEventDestroy(ctx->tev1[i]);
    }
    delete[] ctx->tev0;
    delete[] ctx->tev1;
    delete[] ctx->tkind;
    if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
    for (int k = 0; k < ISO_MAX_CHUNKS; ++k) {
        if (ctx->ev_join[k]) (void)hipEventDestroy(ctx->ev_join[k]);
        if (ctx->ev_kv[k]) (void)hipEventDestroy(ctx->ev_kv[k]);
        if (ctx->xstream[k]) (void)hipStreamDestroy(ctx->xstream[k]);
    }
    if (ctx->sk[0].err) (void)hipHostFree(ctx->sk[0].err);
    for (int i = 0; i < 2; ++i)
        if (ctx->sk[i].base) (void)hipFree(ctx->sk[i].base);
    for (int i = 0; i < ISO_MAX_CHUNKS; ++i) {
        if (ctx->aws[i].part) (void)hipFree(ctx->aws[i].part);
        if (ctx->aws[i].cnt) (void)hipFree(ctx->aws[i].cnt);
    }
    if (ctx->host_sink) (void)hipHostFree(ctx->host_sink);
    if (ctx->rope_cos) (void)hipFree(ctx->rope_cos);
    if (ctx->rope_sin) (void)hipFree(ctx->rope_sin);
    if (ctx->ws) (void)hipFree(ctx->ws);
    delete ctx;
    return rc;
}

int iso_gemm_launch_plan(int M, int N, int K, int num_cu, int *kind, int *team, int *grid) {
    if (!kind || !team || !grid) return fail(ISO_ERR_NULL, "kind, team and grid must be non-NULL");
    if (M < 1 || N < 1 || K < 1 || num_cu < 0) return fail(ISO_ERR_SHAPE, "M=%d N=%d K=%d num_cu=%d", M, N, K, num_cu);
    if (!iso_gemm_bf16_dtl_supported(M, N, K)) {
        *kind = iso_gemm_bf16_mfma_supported(M, N, K) ? ISO_GEMM_STAGED : ISO_GEMM_SIMPLE;
        *team = 1;
        *grid = 0;
        return ISO_OK;
    }
    iso_gemm_bf16_dtl_plan(M, N, K, num_cu, kind, team, grid);
    return ISO_OK;
}

int iso_quantize_rows_fp8(iso_ctx *ctx, const void *x, int rows, int cols, void *q, float *scale, void *stream) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!x || !q || !scale) return fail(ISO_ERR_NULL, "x, q and scale must be non-NULL");
    if (ctx->cfg.dtype != ISO_BF16) return fail(ISO_ERR_DTYPE, "FP8 quantisation takes bf16 input");
    if (rows < 1 || cols < 8 || cols % 8) return fail(ISO_ERR_SHAPE, "rows=%d cols=%d: need rows >= 1, cols a positive multiple of 8", rows, cols);
    hipError_t e = iso_launch_quant_rows_fp8(x, q, scale, rows, cols, (hipStream_t)stream);
    if (e != hipSuccess) return fail(ISO_ERR_HIP, "fp8 row quantiser launch: %s", hipGetErrorString(e));
    return ISO_OK;
}

int iso_rmsnorm_fp8(iso_ctx *ctx, void *x, const void *delta, const void *g, void *q, float *scale, int T, void *stream) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!x || !g || !q || !scale) return fail(ISO_ERR_NULL, "x, g, q and scale must be non-NULL");
    if (ctx->cfg.dtype != ISO_BF16) return fail(ISO_ERR_DTYPE, "the fused norm + FP8 quantiser takes bf16 rows");
    if (T < 1) return fail(ISO_ERR_SHAPE, "T=%d must be positive", T);
    if (!iso_rmsnorm_fp8_supported(ctx->cfg.hidden))
        return fail(ISO_ERR_SHAPE, "hidden=%d: the fused norm + FP8 quantiser takes rows of at most 8192 elements", ctx->cfg.hidden);
    LAUNCH_TRY(delta ? ISO_K_RESID_NORM : ISO_K_RMSNORM, (hipStream_t)stream,
               iso_launch_rmsnorm_fp8(x, delta, nullptr, delta ? x : nullptr, g, q, scale, T, ctx->cfg.hidden, ctx->cfg.rms_eps,
                                      (hipStream_t)stream), "rmsnorm+fp8");
    return ISO_OK;
}

int iso_gemm_fp8(iso_ctx *ctx, const void *a8, const float *sa, const void *w8, const float *sw, void *c, int M, int N,
                 int K, void *stream) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!a8 || !sa || !w8 || !sw || !c) return fail(ISO_ERR_NULL, "operands, scales and c must be non-NULL");
    if (ctx->cfg.dtype != ISO_BF16) return fail(ISO_ERR_DTYPE, "the FP8 GEMM writes bf16");
    if (!iso_gemm_fp8_supported(M, N, K)) return fail(ISO_ERR_SHAPE, "M=%d N=%d K=%d: need M >= 1, N %% 8 == 0, K %% 128 == 0", M, N, K);
    ISO_TRY(sk_status(ctx));
    Timed t_(ctx, ISO_K_GEMM_O, (hipStream_t)stream);
    hipError_t e = iso_launch_gemm_fp8(a8, sa, w8, sw, c, M, N, K, (ctx->flags >> 8) & 15, sk_for(ctx, (hipStream_t)stream),
                                       (hipStream_t)stream);
    if (e != hipSuccess) return fail(ISO_ERR_HIP, "fp8 gemm launch: %s", hipGetErrorString(e));
    return ISO_OK;
}

int iso_set_gemm_segments(iso_ctx *ctx, int n) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (n < 1 || n > 16) return fail(ISO_ERR_SHAPE, "segments=%d outside [1, 16]", n);
    ctx->gemm_segments = n;
    return ISO_OK;
}

int iso_copy_d2h_async(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src) return fail(ISO_ERR_NULL, "dst and src must be non-NULL");
    HIP_TRY(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, (hipStream_t)stream));
    return ISO_OK;
}

int iso_set_flags(iso_ctx *ctx, int flags) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    ctx->flags = flags;
    return ISO_OK;
}

int iso_timing_enable(iso_ctx *ctx, int on) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    ctx->timing = on ? 1 : 0;
    ctx->n_tev = 0;
    return ISO_OK;
}

int iso_timing_read(iso_ctx *ctx, int kind, double *total_ms, int *launches) {
    if (!ctx || !total_ms || !launches) return fail(ISO_ERR_NULL, "ctx, total_ms and launches must be non-NULL");
    if (kind < 0 || kind >= ISO_K_COUNT) return fail(ISO_ERR_SHAPE, "unknown kernel kind %d", kind);
    ISO_TRY(iso_sync(ctx));
    double sum = 0.0;
    int n = 0;
    for (int i = 0; i < ctx->n_tev; ++i) {
        if (ctx->tkind[i] != kind) continue;
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, ctx->tev0[i], ctx->tev1[i]));
        sum += ms;
        ++n;
    }
    *total_ms = sum;
    *launches = n;
    return ISO_OK;
}

int iso_device_count(int *count) {
    if (!count) return fail(ISO_ERR_NULL, "count is NULL");
    *count = 0;
    hipError_t e = hipGetDeviceCount(count);
    if (e == hipErrorNoDevice || e == hipErrorInsufficientDriver) { *count = 0; (void)hipGetLastError(); return ISO_OK; }
    if (e != hipSuccess) { *count = 0; return fail(ISO_ERR_HIP, "hipGetDeviceCount: %s", hipGetErrorString(e)); }
    return ISO_OK;
}
int iso_device_sync(void) { HIP_TRY(hipDeviceSynchronize()); return ISO_OK; }
int iso_dev_alloc(void **ptr, size_t bytes) {
    if (!ptr) return fail(ISO_ERR_NULL, "ptr is NULL");
    *ptr = nullptr;
    HIP_TRY(hipMalloc(ptr, bytes ? bytes : 1));
    return ISO_OK;
}
int iso_dev_free(void *ptr) { if (ptr) HIP_TRY(hipFree(ptr)); return ISO_OK; }
int iso_dev_fill(void *ptr, int byte_value, size_t bytes) {
    if (!ptr) return fail(ISO_ERR_NULL, "ptr is NULL");
    HIP_TRY(hipMemset(ptr, byte_value, bytes));
    HIP_TRY(hipDeviceSynchronize());
    return ISO_OK;
}
int iso_host_alloc(void **ptr, size_t bytes) {
    if (!ptr) return fail(ISO_ERR_NULL, "ptr is NULL");
    *ptr = nullptr;
    HIP_TRY(hipHostMalloc(ptr, bytes ? bytes : 1, hipHostMallocDefault));
    return ISO_OK;
}
int iso_host_free(void *ptr) { if (ptr) HIP_TRY(hipHostFree(ptr)); return ISO_OK; }
int iso_copy_h2d(void *dst, const void *src, size_t bytes) {
    if (!dst || !src) return fail(ISO_ERR_NULL, "dst and src must be non-NULL");
    HIP_TRY(hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice));
    return ISO_OK;
}
int iso_copy_d2h(void *dst, const void *src, size_t bytes) {
    if (!dst || !src) return fail(ISO_ERR_NULL, "dst and src must be non-NULL");
    HIP_TRY(hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost));
    return ISO_OK;
}
int iso_copy_d2d(void *dst, const void *src, size_t bytes) {
    if (!dst || !src) return fail(ISO_ERR_NULL, "dst and src must be non-NULL");
    HIP_TRY(hipMemcpy(dst, src, bytes, hipMemcpyDeviceToDevice));
    HIP_TRY(hipDeviceSynchronize());   // a device-to-device hipMemcpy may return before the copy has run
    return ISO_OK;
}
int iso_stream_create(void **stream) {
    if (!stream) return fail(ISO_ERR_NULL, "stream is NULL");
    hipStream_t s = nullptr;
    HIP_TRY(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
    *stream = (void *)s;
    return ISO_OK;
}
int iso_stream_destroy(void *stream) {
    if (stream) HIP_TRY(hipStreamDestroy((hipStream_t)stream));
    return ISO_OK;
}

void *iso_host_sink(iso_ctx *ctx) { return ctx ? ctx->host_sink : nullptr; }

int iso_layer_prefill(iso_ctx *ctx, const iso_weights *w, void *x, void *k_cache, void *v_cache, int T, int split,
                      int comm, int sched) {
    ISO_TRY(check_layer_args(ctx, w, 1, x, k_cache, v_cache, T, split, comm, sched));
    return run_split(ctx, w, 1, x, k_cache, v_cache, T, split, comm, sched);
}

int iso_stack_prefill(iso_ctx *ctx, const iso_weights *layers, int n_layers, void *x, void *k_caches, void *v_caches,
                      int T, int split, int comm, int sched) {
    ISO_TRY(check_layer_args(ctx, layers, n_layers, x, k_caches, v_caches, T, split, comm, sched));
    return run_split(ctx, layers, n_layers, x, k_caches, v_caches, T, split, comm, sched);
}

int iso_stack_prefill_chunks(iso_ctx *ctx, const iso_weights *layers, int n_layers, void *x, void *k_caches,
                             void *v_caches, int T, const int *bounds, int n_chunks, int comm, int sched) {
    ISO_TRY(check_layer_args(ctx, layers, n_layers, x, k_caches, v_caches, T, 0, comm, sched));
    if (n_chunks < 1 || n_chunks > ISO_MAX_CHUNKS)
        return fail(ISO_ERR_SHAPE, "n_chunks=%d outside [1, %d]", n_chunks, ISO_MAX_CHUNKS);
    if (n_chunks > 1 && !bounds) return fail(ISO_ERR_NULL, "bounds is NULL");
    int edges[ISO_MAX_CHUNKS + 1];
    edges[0] = 0;
    for (int k = 1; k < n_chunks; ++k) {
        edges[k] = bounds[k - 1];
        if (edges[k] <= edges[k - 1] || edges[k] >= T)
            return fail(ISO_ERR_SPLIT, "bounds[%d]=%d must lie in (%d, %d)", k - 1, edges[k], edges[k - 1], T);
    }
    edges[n_chunks] = T;
    return run_stack(ctx, layers, n_layers, x, k_caches, v_caches, edges, n_chunks, comm, sched);
}

int iso_attn_chunk(iso_ctx *ctx, const void *q, const void *k_cache, const void *v_cache, void *out, int Tc,
                   int q_offset, int kv_len, void *stream) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!q || !k_cache || !v_cache || !out) return fail(ISO_ERR_NULL, "q, k_cache, v_cache and out must be non-NULL");
    if (Tc < 1) return fail(ISO_ERR_SHAPE, "Tc=%d must be positive", Tc);
    if (q_offset < 0) return fail(ISO_ERR_SHAPE, "q_offset=%d must be >= 0", q_offset);
    if (kv_len < 1) return fail(ISO_ERR_SHAPE, "kv_len=%d must be positive", kv_len);
    if (kv_len > ctx->cfg.max_seq) return fail(ISO_ERR_WORKSPACE, "kv_len=%d exceeds max_seq=%d", kv_len, ctx->cfg.max_seq);
    if (Tc > ctx->cfg.max_seq) return fail(ISO_ERR_WORKSPACE, "Tc=%d exceeds max_seq=%d", Tc, ctx->cfg.max_seq);
    ISO_TRY(sk_status(ctx));
    return attention(ctx, q, ctx->cfg.n_q_heads * ctx->cfg.head_dim, k_cache, v_cache, out, Tc, q_offset, kv_len,
                     (hipStream_t)stream);
}

int iso_gemm_rowpar(iso_ctx *ctx, const void *a, const void *w, void *c, int M, int N, int K, void *stream,
                    void *host_sink) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!a || !w || !c) return fail(ISO_ERR_NULL, "a, w and c must be non-NULL");
    if (M < 1 || N < 1 || K < 1) return fail(ISO_ERR_SHAPE, "M=%d N=%d K=%d must be positive", M, N, K);
    if (ctx->cfg.dtype == ISO_BF16 && (K % 8)) return fail(ISO_ERR_SHAPE, "K=%d must be a multiple of 8 for bf16", K);
    ISO_TRY(sk_status(ctx));
    ISO_TRY(gemm(ctx, ISO_K_GEMM_O, a, w, c, M, N, K, (hipStream_t)stream));
    if (host_sink) {
        Timed t_(ctx, ISO_K_COMM, (hipStream_t)stream);
        HIP_TRY(hipMemcpyAsync(host_sink, c, (size_t)M * N * ctx->elt, hipMemcpyDeviceToHost, (hipStream_t)stream));
    }
    return ISO_OK;
}

int iso_gemm_rowpar_static(iso_ctx *ctx, const void *a, const void *w, void *c, int M, int N, int K, void *stream) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!a || !w || !c) return fail(ISO_ERR_NULL, "a, w and c must be non-NULL");
    if (ctx->cfg.dtype != ISO_BF16) return fail(ISO_ERR_DTYPE, "the static-workspace GEMM takes bf16 operands");
    if (M < 1 || N < 1 || K < 1) return fail(ISO_ERR_SHAPE, "M=%d N=%d K=%d must be positive", M, N, K);
    if (!iso_gemm_bf16_dtl_supported(M, N, K))
        return fail(ISO_ERR_SHAPE, "M=%d N=%d K=%d is beyond what the static-workspace GEMM takes: K a multiple of 64, "
                                   "N a multiple of 8, M*K and N*K below 2^31 elements", M, N, K);
    ISO_TRY(sk_status(ctx));
    hipError_t e = iso_launch_gemm_bf16_sk_static(a, w, c, M, N, K, ctx->sk[0].err, (hipStream_t)stream);
    if (e == hipErrorNotReady) return fail(ISO_ERR_HIP, "no context has been created on the current device");
    if (e != hipSuccess) return fail(ISO_ERR_HIP, "static-workspace gemm launch (M=%d N=%d K=%d): %s", M, N, K, hipGetErrorString(e));
    return ISO_OK;
}

unsigned *iso_streamk_status_word(iso_ctx *ctx) { return ctx ? ctx->sk[0].err : nullptr; }

int iso_rmsnorm(iso_ctx *ctx, const void *x, const void *g, void *y, int T, void *stream) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!x || !g || !y) return fail(ISO_ERR_NULL, "x, g and y must be non-NULL");
    if (T < 1) return fail(ISO_ERR_SHAPE, "T=%d must be positive", T);
    LAUNCH_TRY(ISO_K_RMSNORM, (hipStream_t)stream, iso_launch_rmsnorm(ctx->cfg.dtype, x, nullptr, nullptr, nullptr, g, y, T, ctx->cfg.hidden, ctx->cfg.rms_eps,
                                  (hipStream_t)stream), "rmsnorm");
    return ISO_OK;
}

int iso_residual_rmsnorm(iso_ctx *ctx, void *x, const void *delta, const void *g, void *y, int T, void *stream) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!x || !delta) return fail(ISO_ERR_NULL, "x and delta must be non-NULL");
    if ((y != nullptr) != (g != nullptr)) return fail(ISO_ERR_NULL, "g and y must both be given or both be NULL");
    if (T < 1) return fail(ISO_ERR_SHAPE, "T=%d must be positive", T);
    LAUNCH_TRY(y ? ISO_K_RESID_NORM : ISO_K_RESIDUAL, (hipStream_t)stream, iso_launch_rmsnorm(ctx->cfg.dtype, x, delta, nullptr, x, g, y, T, ctx->cfg.hidden, ctx->cfg.rms_eps,
                                  (hipStream_t)stream), "residual+rmsnorm");
    return ISO_OK;
}

int iso_rope_kv_write(iso_ctx *ctx, void *qkv, void *k_cache, void *v_cache, int Tc, int q_offset, void *stream) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!qkv || !k_cache || !v_cache) return fail(ISO_ERR_NULL, "qkv, k_cache and v_cache must be non-NULL");
    if (Tc < 1 || q_offset < 0) return fail(ISO_ERR_SHAPE, "Tc=%d must be positive and q_offset=%d >= 0", Tc, q_offset);
    if ((long long)q_offset + Tc > ctx->cfg.max_seq)
        return fail(ISO_ERR_WORKSPACE, "q_offset+Tc=%lld exceeds max_seq=%d", (long long)q_offset + Tc, ctx->cfg.max_seq);
    const iso_cfg &c = ctx->cfg;
    LAUNCH_TRY(ISO_K_ROPE_KV, (hipStream_t)stream, iso_launch_rope_kv(c.dtype, qkv, k_cache, v_cache, ctx->rope_cos, ctx->rope_sin, Tc, q_offset,
                                  c.n_q_heads, c.n_kv_heads, c.head_dim, (hipStream_t)stream), "rope+kv");
    return ISO_OK;
}

int iso_swiglu(iso_ctx *ctx, const void *gu, void *a, int T, void *stream) {
    if (!ctx) return fail(ISO_ERR_NULL, "ctx is NULL");
    if (!gu || !a) return fail(ISO_ERR_NULL, "gu and a must be non-NULL");
    if (T < 1) return fail(ISO_ERR_SHAPE, "T=%d must be positive", T);
    LAUNCH_TRY(ISO_K_SWIGLU, (hipStream_t)stream, iso_launch_swiglu(ctx->cfg.dtype, gu, a, T, ctx->cfg.ffn, (hipStream_t)stream), "swiglu");
    return ISO_OK;
}

}  // extern "C"
