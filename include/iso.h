/*
 * iso.h -- C ABI of the ISO (intra-sequence overlap) layer-shard prefill for MI355X (gfx950).
 *
 * One GPU's tensor-parallel shard of a decoder layer is run over one prompt that is cut into two
 * chunks along the sequence (paper, Section 1 and Section 3.1).  The attention of chunk 1 reads the
 * K/V rows that chunk 0 wrote to the cache; that is the only ordering constraint between the chunks
 * (Section 3.1).  Everything else is per token and is issued per chunk on two HIP streams, so the
 * communication point that ends each block (Section 2.2: the collective after o_proj and after the
 * down matrix) overlaps with the other chunk's kernels.  On a single GPU the collective is replaced
 * by a device-to-host copy of the same byte count, placed in the chunk's stream.
 *
 * Conventions
 *   - All device buffers are caller-owned, row-major, token-major, 16-byte aligned.
 *   - "hidden" is the full model width; head counts and ffn are LOCAL to the shard (Section 2.1, TP).
 *   - Streams are hipStream_t handles passed as void*; every call is asynchronous with respect to the
 *     host and returns after enqueueing.  No entry point synchronises the device except iso_sync and
 *     iso_destroy.
 *   - Every function returns ISO_OK (0) or a negative iso_status.  Arguments are validated before any
 *     device work is enqueued; nothing throws or aborts.  iso_last_error() describes the last failure
 *     of the calling thread.
 *   - The sum over tensor-parallel ranks is over a world of one rank: the shard's partial output is
 *     what is added to the residual stream.
 *   - The compute entry points may be recorded into a HIP graph (stream capture on stream0; the
 *     library's other streams join through its events) once the same call has run eagerly, so that
 *     streams, events and kernel attributes exist.  While a stream is capturing, the stream-K GEMM
 *     launch is not used (its launches are numbered, a replay would repeat a number) and per-launch
 *     timing is off.
 */
#ifndef ISO_H_
#define ISO_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ISO_OK = 0,
    ISO_ERR_NULL = -1,      /* a required pointer is NULL                               */
    ISO_ERR_SHAPE = -2,     /* a size is non-positive, misaligned or inconsistent       */
    ISO_ERR_DTYPE = -3,     /* unknown element type                                     */
    ISO_ERR_SPLIT = -4,     /* split point outside [0, T]                               */
    ISO_ERR_WORKSPACE = -5, /* T (or kv_len, M) exceeds what the context was created for */
    ISO_ERR_HIP = -6        /* a HIP runtime call failed (no device, out of memory, ...) */
} iso_status;

typedef enum { ISO_F32 = 0, ISO_BF16 = 1 } iso_dtype;

/* What stands at the two communication points of a layer (after o_proj, after down). */
typedef enum {
    ISO_COMM_NONE = 0, /* nothing: compute only                                                      */
    ISO_COMM_D2H = 1,  /* copy the [Tc, hidden] partial to pinned host memory in the chunk's stream;  */
                       /* the consumer kernel is behind the copy in stream order                      */
    ISO_COMM_D2H_INT8 = 2 /* Section 3.2 (communication dominates): quantise the partial to int8 first.   */
                       /* Per token row: scale = max|p|/127 (1 for a zero row), code = nearest-even(p/scale)   */
                       /* clipped to +-127.  The copy moves Tc rows of hidden codes + the fp32 scale (row     */
                       /* pitch hidden + 16 bytes); the layer continues with code*scale, the value a receiver */
                       /* of the quantised payload would add to its residual stream.                          */
} iso_comm;

/* How the two chunks are issued (Section 1, Figure 1 (a) versus (d)). */
typedef enum {
    ISO_SCHED_OVERLAP = 0, /* chunk 0 on stream0, chunk 1 on stream1; one event per layer orders them: with transfers
                              and chunks of >= 1024 rows chunk 1's attention block starts when chunk 0's has been
                              issued, otherwise chunk 1's attention starts when chunk 0's K/V rows are written */
    ISO_SCHED_SERIAL = 1,  /* every chunk on stream0, one block after the other, copies in line        */
    ISO_SCHED_STREAM_PER_CHUNK = 2 /* each chunk on a stream of its own (the context makes the extra ones), attention
                                      blocks chained in chunk order; meant for more than two chunks            */
} iso_sched;

typedef struct {
    int hidden;      /* H, multiple of 8                                         */
    int n_q_heads;   /* local query heads                                        */
    int n_kv_heads;  /* local key/value heads; divides n_q_heads                 */
    int head_dim;    /* 64 or 128                                                */
    int ffn;         /* local MLP width F, multiple of 8                         */
    float rms_eps;   /* RMSNorm epsilon (inside the square root)                 */
    float rope_base; /* rotary base; theta_i = base^(-2i/head_dim)               */
    int dtype;       /* iso_dtype of every activation, weight and cache tensor   */
    int max_seq;     /* largest T (and kv_len) any later call may use            */
} iso_cfg;

/* Device pointers to one layer shard's weights, all of cfg.dtype.  y = x W^T for every matrix. */
typedef struct {
    const void *w_qkv;     /* [(nq + 2 nkv) * d, hidden]; rows: q heads, then k heads, then v heads */
    const void *w_o;       /* [hidden, nq * d]                                                      */
    const void *w_gate_up; /* [2 * ffn, hidden]; rows: gate, then up                                */
    const void *w_down;    /* [hidden, ffn]                                                         */
    const void *g_attn;    /* [hidden] RMSNorm gain before the attention block                      */
    const void *g_mlp;     /* [hidden] RMSNorm gain before the MLP block                            */
    /* Optional FP8 (E4M3) copies of the four matrices, same shapes, one byte per element, each with one fp32
     * scale per row (= output channel): matrix row = fp8 row * scale.  Made by iso_quantize_rows_fp8.  Read only
     * when ISO_FLAG_FP8_GEMM is set and all eight pointers are non-NULL; NULL otherwise. */
    const void *w_qkv_f8, *w_o_f8, *w_gate_up_f8, *w_down_f8;
    const float *s_qkv, *s_o, *s_gate_up, *s_down;
} iso_weights;

typedef struct iso_ctx iso_ctx;

/* Chunk ranges and buffer sizes derived on the host (no device needed). */
typedef struct {
    int n_chunks;             /* 1 (unsplit) or 2                                   */
    int q_offset[2];          /* first token of each chunk                          */
    int n_tokens[2];          /* tokens of each chunk                               */
    int kv_len[2];            /* keys visible to each chunk = q_offset + n_tokens   */
    size_t comm_bytes[2];     /* bytes moved at EACH communication point of a chunk */
    size_t workspace_bytes;   /* device workspace a context for cfg.max_seq holds   */
} iso_plan;

#define ISO_MAX_CHUNKS 8      /* most chunks one prompt may be cut into */

/* Checks a configuration; returns ISO_OK or the error iso_create would return for it.  Host only. */
int iso_validate_cfg(const iso_cfg *cfg);

/* Fills `out` with the chunk ranges for a prompt of T tokens cut at `split` (Section 3.1; an unequal
 * cut is the remedy of Section 6 for the dearer second half).  split == 0 or split == T means one
 * chunk.  Host only.  Errors: NULL, bad cfg, T < 1, T > max_seq (ISO_ERR_WORKSPACE), split outside
 * [0, T] (ISO_ERR_SPLIT). */
int iso_plan_chunks(const iso_cfg *cfg, int T, int split, iso_plan *out);

/* Cut points for n_chunks chunks of equal estimated cost instead of equal length (Section 6: the later part of
 * the sequence is dearer, so the first chunk should be longer; finer cuts than two).  The cost of position i is
 * the layer's projection flops per token plus attn_flop_cost * 4 * nq * d * (i + 1) for its attention over
 * i + 1 keys; attn_flop_cost says how much dearer an attention flop is than a projection flop on the machine
 * (<= 0 selects 3.0, the ratio measured on MI355X at these shapes).  bounds[0 .. n_chunks-2] receives the
 * ascending cut points, each a multiple of 128 when T >= 256 * n_chunks.  Host only.
 * Errors: NULL, bad cfg, T < 1 or n_chunks outside [1, min(T, ISO_MAX_CHUNKS)] (ISO_ERR_SHAPE),
 * T > max_seq (ISO_ERR_WORKSPACE). */
int iso_plan_split(const iso_cfg *cfg, int T, int n_chunks, double attn_flop_cost, int *bounds);

/* How many chunks to cut a prompt of T tokens into for ISO_SCHED_STREAM_PER_CHUNK: chunks of about 2048 tokens, at
 * least 2 and at most ISO_MAX_CHUNKS (1 for prompts shorter than 512 tokens, where the projections of half a prompt no
 * longer fill the matrix cores).  Rule read off the chunk-count sweeps on MI355X (2k: 2-3, 8k: 4, 32k-128k: 8); more
 * chunks shorten the unoverlapped ends of the pipeline, fewer keep the GEMMs large.  Host only.
 * Errors: NULL, bad cfg, T < 1 (ISO_ERR_SHAPE), T > max_seq (ISO_ERR_WORKSPACE). */
int iso_plan_chunk_count(const iso_cfg *cfg, int T, int *n_chunks);

/* Creates a context on the current HIP device: workspace for max_seq tokens, the rotary table
 * (computed on the host in double, stored fp32), one event pair, and pinned host memory for the
 * copy stand-in.  stream0/stream1 are the caller's two streams (stream1 may equal stream0; NULL is
 * the default stream).  On failure *out is NULL. */
int iso_create(iso_ctx **out, const iso_cfg *cfg, void *stream0, void *stream1);
/* iso_sync waits for both streams.  iso_destroy synchronises the streams and frees everything the context owns.
 * Both return ISO_ERR_HIP if a stream-K GEMM launched since the last iso_sync gave up a (bounded) wait for a
 * partial tile: every result of that pass is then invalid.  The condition stays set until iso_sync has reported
 * it; meanwhile the layer, attention and projection entry points refuse to enqueue further work (ISO_ERR_HIP). */
int iso_destroy(iso_ctx *ctx);
int iso_sync(iso_ctx *ctx);
/* Host address of the pinned word behind that condition (0 = fine), NULL for an fp32 context.  For tests of the
 * error path: a test writes 1 there instead of making a kernel time out. */
unsigned *iso_streamk_status_word(iso_ctx *ctx);
const char *iso_last_error(void);         /* message for the calling thread's last failure        */

/* One decoder-layer shard over a prompt of T tokens (Section 2.2 for the block structure, Section 3.1
 * for the chunking):
 *     x1 = x + o_proj(attention(rope(qkv(rmsnorm(x; g_attn)))));  x = x1 + down(swiglu(gate_up(rmsnorm(x1; g_mlp))))
 * x        [T, hidden] device, read and overwritten with the layer output.
 * k_cache  [max_seq, nkv, d] device; rows 0..T-1 are written (keys after RoPE).
 * v_cache  [max_seq, nkv, d] device; rows 0..T-1 are written.
 * split    0 or T: one chunk on stream0.  1..T-1: two chunks [0,split) and [split,T).
 * comm     iso_comm; sched: iso_sched (ignored for one chunk).
 * On entry stream1 is made to wait for the work already in stream0; on return stream0 waits for
 * stream1, so the call behaves like one operation enqueued on stream0.
 * Errors: NULL, ISO_ERR_WORKSPACE if T > max_seq, ISO_ERR_SPLIT, ISO_ERR_SHAPE if T < 1. */
int iso_layer_prefill(iso_ctx *ctx, const iso_weights *w, void *x, void *k_cache, void *v_cache,
                      int T, int split, int comm, int sched);

/* A stack of n_layers such layers (Section 2.2: stacked transformer blocks).  layers[l] are the
 * weights of layer l; k_caches/v_caches hold n_layers consecutive caches of [max_seq, nkv, d].
 * The chunks stay on their streams across layers (no join between layers), so the communication
 * of layer l overlaps the attention block of layer l+1 of the other chunk. */
int iso_stack_prefill(iso_ctx *ctx, const iso_weights *layers, int n_layers, void *x,
                      void *k_caches, void *v_caches, int T, int split, int comm, int sched);

/* The same stack with the prompt cut into n_chunks chunks at bounds[0] < bounds[1] < ... (Section 6: finer
 * segmentation than two chunks; the figure that draws it is not available, this is the natural extension of the
 * two-chunk schedule).  Chunk c covers [bounds[c-1], bounds[c]) with bounds[-1] = 0 and bounds[n_chunks-1] = T,
 * runs on stream c % 2 in ISO_SCHED_OVERLAP (all on stream0 in ISO_SCHED_SERIAL), and its attention waits for
 * the K/V rows of chunk c-1 (hence of every earlier chunk).  More chunks shorten the two ends of the pipeline
 * that nothing overlaps (the first attention block and the last transfer) at the price of smaller GEMMs.
 * n_chunks == 1 ignores bounds (may be NULL).  n_chunks == 2 with bounds[0] == split is iso_stack_prefill.
 * Errors: as iso_stack_prefill; n_chunks outside [1, ISO_MAX_CHUNKS] (ISO_ERR_SHAPE); bounds NULL for
 * n_chunks > 1 (ISO_ERR_NULL); bounds not strictly ascending inside (0, T) (ISO_ERR_SPLIT). */
int iso_stack_prefill_chunks(iso_ctx *ctx, const iso_weights *layers, int n_layers, void *x,
                             void *k_caches, void *v_caches, int T, const int *bounds, int n_chunks,
                             int comm, int sched);

/* Attention of one chunk over the KV cache (Section 3.1; chunked prefill, Section 2.1).
 * q        [Tc, nq, d] device, rotary embedding already applied.
 * k_cache, v_cache  [>= kv_len, nkv, d] device.
 * out      [Tc, nq * d] device.
 * Key j is visible to local row i iff j <= q_offset + i and j < kv_len; softmax scale 1/sqrt(d);
 * query head h reads kv head h / (nq / nkv).
 * Errors: NULL, Tc < 1, q_offset < 0, kv_len < 1 (ISO_ERR_SHAPE), kv_len > max_seq or
 * Tc > max_seq (ISO_ERR_WORKSPACE). */
int iso_attn_chunk(iso_ctx *ctx, const void *q, const void *k_cache, const void *v_cache, void *out,
                   int Tc, int q_offset, int kv_len, void *stream);

/* Row-parallel projection and its communication point (Section 2.2: o_proj / down followed by a
 * collective):  c[M, N] = a[M, K] * w[N, K]^T, then, if host_sink != NULL, an asynchronous copy of c
 * (M*N elements) to host_sink in the same stream.  host_sink must be pinned host memory of at least
 * M*N*sizeof(element) bytes.  K must be a multiple of 8 for bf16.
 * Errors: NULL, non-positive or misaligned sizes (ISO_ERR_SHAPE). */
int iso_gemm_rowpar(iso_ctx *ctx, const void *a, const void *w, void *c, int M, int N, int K,
                    void *stream, void *host_sink);

/* iso_gemm_rowpar for callers that cannot allocate or record memset nodes: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  c[M, N] = a[M, K] * w[N, K]^T (bf16, no host copy) through the
 * stream-K kernel, whose flag words and fp32 partial tiles live in a static device array of 4 KiB + 256 * 256 KiB
 * (64 MiB + 4 KiB) that every GPU the library runs on holds until the process ends; its address on a device is
 * looked up when the first bf16 context is created there.  The call enqueues two kernels on `stream` (one clears the
 * flag words, then the product) and calls no allocating routine, no hipMemsetAsync and no event creation; it is not
 * part of the per-launch timing record.  Limits: bf16 context; K a multiple of 64, N a multiple of 8, M*K and N*K
 * below 2^31 elements (ISO_ERR_SHAPE otherwise); at most 256 workgroups are used whatever the device.  All calls on
 * one GPU share the array: calls that may overlap in time (different streams, different contexts, different host
 * threads) race on it and must be ordered by the caller; calls in one stream are ordered by the stream.  A wait that
 * runs out is reported as for every stream-K launch (iso_sync).
 * Errors: NULL, ISO_ERR_DTYPE (fp32 context), ISO_ERR_SHAPE, ISO_ERR_HIP. */
int iso_gemm_rowpar_static(iso_ctx *ctx, const void *a, const void *w, void *c, int M, int N, int K, void *stream);

/* The element-wise steps of the layer, exposed for parity tests and per-kernel measurement.
 * All pointers are device pointers of cfg.dtype; `stream` is a hipStream_t.                     */
/* y[t,:] = x[t,:] * rsqrt(mean(x[t,:]^2) + eps) * g */
int iso_rmsnorm(iso_ctx *ctx, const void *x, const void *g, void *y, int T, void *stream);
/* x[t,:] += delta[t,:] (in place); if y != NULL also y[t,:] = rmsnorm(x[t,:]; g) */
int iso_residual_rmsnorm(iso_ctx *ctx, void *x, const void *delta, const void *g, void *y, int T,
                         void *stream);
/* qkv [Tc, (nq+2nkv)*d]: rotates the q part in place at positions q_offset+i and writes rotated k
 * and plain v to rows q_offset+i of the caches (rotate-half pairs (i, i+d/2)). */
int iso_rope_kv_write(iso_ctx *ctx, void *qkv, void *k_cache, void *v_cache, int Tc, int q_offset,
                      void *stream);
/* a[t, f] = silu(gu[t, f]) * gu[t, ffn + f],  gu [T, 2*ffn] -> a [T, ffn] */
int iso_swiglu(iso_ctx *ctx, const void *gu, void *a, int T, void *stream);

/* Kernel selection, for tests and measurement.  Default 0 = the matrix-core kernels wherever the dtype
 * and shapes allow.  The forced alternatives are complete HIP kernels as well (they are the fp32 path). */
enum {
    ISO_FLAG_SIMPLE_GEMM = 1, /* SIMT tile GEMM instead of the MFMA GEMMs                  */
    ISO_FLAG_SIMPLE_ATTN = 2, /* one-wave-per-row attention instead of the MFMA attention  */
    ISO_FLAG_GEMM_STAGED = 4, /* register-staged 128x128 MFMA GEMM instead of the direct-to-LDS one */
    ISO_FLAG_NO_FUSE = 8,     /* no fused epilogues: gate/up projection and SwiGLU as two kernels, QKV projection
                                 and rotary embedding + KV-cache write as two kernels                  */
    ISO_FLAG_ATTN_STAGED = 16,/* register-staged MFMA attention instead of the direct-to-LDS one    */
    ISO_FLAG_NO_STREAMK = 32, /* never pick the stream-K launch of the direct-to-LDS GEMM by itself  */
    ISO_FLAG_FP8_GEMM = 64    /* bf16 layers: run the four projections on the FP8 matrix cores (needs the FP8
                                 weights in iso_weights; activations are quantised per token row on the fly) */
    /* bits 8..11: tile variant of the direct-to-LDS GEMM (0 = chosen from the shape; 6 = its stream-K launch, which
     * this value also forces for the FP8 GEMM) */
    /* bits 12..13: launch shape of the direct-to-LDS attention (0 = chosen from the size; 1 = key tiles split inside
     * the workgroup; 2 = that, and two row blocks (longest with shortest) per workgroup; 3 = one row block per
     * workgroup, two workgroups per compute unit) */
    /* bits 14..16: key split of the direct-to-LDS attention ACROSS workgroups (0 = chosen from the size: launches of at
     * most half as many workgroups as the device has compute units; 1 = never; 2, 3, 4 = that many shares) */
};
int iso_set_flags(iso_ctx *ctx, int flags);

/* Which kernel a bf16 projection of these sizes takes when nothing is forced, on a device with num_cu compute units
 * (num_cu == 0: as for a stream the context does not own, i.e. never stream-K).  Host only; for tests and tuning.
 * kind: ISO_GEMM_TILE_256 / ISO_GEMM_TILE_128 (one 256x256 / 128x128 tile per workgroup, *grid workgroups),
 * ISO_GEMM_STREAMK (*grid workgroups in teams of *team), ISO_GEMM_STAGED / ISO_GEMM_SIMPLE (the fallbacks for sizes
 * the direct-to-LDS kernel does not take; *grid is 0).  Errors: NULL, non-positive sizes (ISO_ERR_SHAPE). */
typedef enum {
    ISO_GEMM_TILE_256 = 1,
    ISO_GEMM_TILE_128 = 3,
    ISO_GEMM_STREAMK = 6,
    ISO_GEMM_STAGED = 100,
    ISO_GEMM_SIMPLE = 101
} iso_gemm_kind;
int iso_gemm_launch_plan(int M, int N, int K, int num_cu, int *kind, int *team, int *grid);

/* FP8 projections (the paper runs its matrix products in 8 bits, Section 4.1; FP8 E4M3 is the 8-bit type of the
 * CDNA4 matrix cores).  bf16 contexts only.
 * iso_quantize_rows_fp8: x [rows, cols] bf16 device -> q [rows, cols] E4M3 bytes + scale [rows] fp32, all device.
 *   Per row, in fp32: amax = max|x|, q = e4m3(x * (448 / amax)) rounded to nearest even, scale = amax / 448
 *   (an all-zero row gets scale 1).  cols % 8 == 0.  Used once per weight matrix and, inside the layer, per
 *   projection input.
 * iso_gemm_fp8: c [M, N] bf16 = (a8 [M, K] x w8 [N, K]^T) * sa[M] * sw[N], fp32 accumulation of the exact products.
 *   K % 128 == 0, N % 8 == 0.
 * iso_rmsnorm_fp8: the norm in front of an 8-bit projection with the quantiser in its tail.  x [T, hidden] bf16;
 *   delta (NULL or [T, hidden] bf16): x += delta in place first; then q [T, hidden] / scale [T] are exactly what
 *   iso_quantize_rows_fp8 gives for the bf16 output of iso_rmsnorm / iso_residual_rmsnorm, which is never stored.
 *   hidden <= 8192 (the row stays in registers), else ISO_ERR_SHAPE.  The layer entry points use it for the QKV
 *   and gate/up inputs under ISO_FLAG_FP8_GEMM.
 * Errors: NULL, ISO_ERR_SHAPE for sizes the kernels do not take, ISO_ERR_DTYPE for an fp32 context. */
int iso_rmsnorm_fp8(iso_ctx *ctx, void *x, const void *delta, const void *g, void *q, float *scale, int T,
                    void *stream);
int iso_quantize_rows_fp8(iso_ctx *ctx, const void *x, int rows, int cols, void *q, float *scale, void *stream);
int iso_gemm_fp8(iso_ctx *ctx, const void *a8, const float *sa, const void *w8, const float *sw, void *c,
                 int M, int N, int K, void *stream);

/* GEMM segmentation (Section 3.2, the remedy for the computation-dominated case): every projection of the layer
 * entry points is issued as n launches over consecutive row ranges (multiples of 256 rows; products with fewer
 * than 256 * n rows stay whole).  Results are the same bits as long as the segments take the same kernel variant
 * as the whole product (the launch rule looks at the tile count, so a segment may get the 128x128 tile or miss the
 * stream-K launch where the whole product does not; the sum order inside a tile then differs) and agree within
 * rounding otherwise.  n in [1, 16]; 1 (the default) is one launch.  Errors: NULL, ISO_ERR_SHAPE. */
int iso_set_gemm_segments(iso_ctx *ctx, int n);

/* Per-launch timing for measurement.  While enabled, every kernel launch and every copy the library
 * enqueues is bracketed by a pair of HIP events recorded in the stream of that launch (at most 65536
 * launches are kept; enabling clears the record).  iso_timing_read synchronises both streams and returns
 * the summed duration and the number of recorded launches of one kind. */
typedef enum {
    ISO_K_GEMM_QKV = 0, ISO_K_GEMM_O = 1, ISO_K_GEMM_GATE_UP = 2, ISO_K_GEMM_DOWN = 3, ISO_K_ATTN = 4,
    ISO_K_RMSNORM = 5, ISO_K_RESID_NORM = 6, ISO_K_RESIDUAL = 7, ISO_K_ROPE_KV = 8, ISO_K_SWIGLU = 9,
    ISO_K_COMM = 10, ISO_K_QUANT = 11, ISO_K_COUNT = 12
} iso_kernel_kind;
int iso_timing_enable(iso_ctx *ctx, int on);
int iso_timing_read(iso_ctx *ctx, int kind, double *total_ms, int *launches);

/* Device plumbing, so that callers need nothing but this library to hold buffers and streams.  All of
 * these act on the current HIP device of the calling thread; copies are synchronous (they return when
 * the bytes have arrived).  Errors: ISO_ERR_NULL, ISO_ERR_HIP. */
int iso_device_count(int *count);                         /* 0 devices is ISO_OK with *count == 0  */
int iso_device_sync(void);                                /* hipDeviceSynchronize                   */
int iso_dev_alloc(void **ptr, size_t bytes);              /* device memory, 256-byte aligned        */
int iso_dev_free(void *ptr);
int iso_dev_fill(void *ptr, int byte_value, size_t bytes);
int iso_host_alloc(void **ptr, size_t bytes);             /* pinned host memory                     */
int iso_host_free(void *ptr);
int iso_copy_h2d(void *dst_dev, const void *src_host, size_t bytes);
int iso_copy_d2h(void *dst_host, const void *src_dev, size_t bytes);
/* Asynchronous device-to-host copy in `stream` (dst_host pinned, e.g. from iso_host_alloc): the same call the
 * communication stand-in makes, exposed so that a caller can keep the copy engine busy beside a kernel. */
int iso_copy_d2h_async(void *dst_host, const void *src_dev, size_t bytes, void *stream);
int iso_copy_d2d(void *dst_dev, const void *src_dev, size_t bytes);
int iso_stream_create(void **stream);                     /* non-blocking stream, default priority  */
int iso_stream_destroy(void *stream);

/* Pinned host buffer of the communication stand-in, for tests: two regions of max_seq * hidden elements
 * (after o_proj, after down); with ISO_COMM_D2H_INT8 a region holds rows of hidden + 16 bytes. */
void *iso_host_sink(iso_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* ISO_H_ */
