// Internal declarations shared by the HIP sources of libiso (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "iso.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// Workspace of one stream-K GEMM in flight (flag words + one fp32 partial tile per workgroup).  Launches that
// share a workspace must be ordered (same stream); the context keeps one per stream of its own.
struct iso_sk_ws {
    void *base;        // device; flag words zeroed once at creation, never reset (each launch uses a new epoch)
    unsigned *err;     // pinned host word the kernel sets if a bounded wait ran out
    unsigned epoch;    // launch counter
    int num_wg;        // grid size = compute units of the device
};

// Workspace of the attention launches that split the keys of a row block across workgroups: partial states and one
// arrival counter per (row block, head).  Counters are zero between launches (the last arriver resets its own).
// Launches that share a workspace must be ordered (same stream); the context keeps one per stream of its own.
struct iso_attn_ws {
    unsigned char *part;   // device, max_slots * iso_attn_part_bytes()
    unsigned *cnt;         // device, max_blocks words, zeroed at creation
    int max_slots;         // (row block, head, share) triples a launch may use
    int max_blocks;        // (row block, head) pairs a launch may use
};

struct iso_ctx {
    iso_cfg cfg;
    int device;
    int flags;
    hipStream_t stream[2];
    hipStream_t xstream[ISO_MAX_CHUNKS];   // own streams for chunks 2.. of ISO_SCHED_STREAM_PER_CHUNK, made on first use
    hipEvent_t ev_fork, ev_join[ISO_MAX_CHUNKS], ev_kv[ISO_MAX_CHUNKS];
    size_t elt;        // bytes per element
    // device workspace, each sized for max_seq tokens; chunks use disjoint row ranges
    void *ws;          // one allocation
    size_t ws_bytes;
    void *y;           // [max_seq, hidden]   normed activations (both norms)
    void *qkv;         // [max_seq, n_qkv]
    void *attn;        // [max_seq, nq*d]
    void *part;        // [max_seq, hidden]   row-parallel partial of the attention block (o_proj)
    void *part_m;      // [max_seq, hidden]   row-parallel partial of the MLP block (down); both live until the layer closes
    void *gu;          // [max_seq, 2*ffn]
    void *act;         // [max_seq, ffn]
    signed char *q8;   // [max_seq, hidden + 16] int8 codes + fp32 scale per row (ISO_COMM_D2H_INT8)
    unsigned char *a8; // [max_seq, max(hidden, nq*d, ffn)] FP8 copy of the current projection input (bf16 contexts)
    float *a8s;        // [max_seq] its row scales
    size_t a8_pitch;   // bytes per token of a8
    float *rope_cos;   // [max_seq, d/2]
    float *rope_sin;   // [max_seq, d/2]
    int gemm_segments; // launches per projection GEMM along M (0 or 1: one launch)
    int sk_hold;       // set while a pass enqueues work for which stream-K is not to be picked
    iso_sk_ws sk[2];   // stream-K GEMM workspaces, one per caller stream (bf16 contexts only; base == null otherwise)
    iso_attn_ws aws[ISO_MAX_CHUNKS];   // key-split attention workspaces: [0], [1] for the caller's streams, [k] for xstream[k]
    void *host_sink;   // pinned, 2 * max_seq * hidden elements
    // optional per-launch timing (iso_timing_*): event pairs recorded around every launch, in its stream
    int timing;
    int n_tev, n_tev_created;
    hipEvent_t *tev0, *tev1;
    int *tkind;
};
constexpr int ISO_MAX_TIMED = 65536;

// ---- launchers; each validates nothing (callers do) and returns the launch status -------------
// x_new = x (+ delta (+ delta2)); x_out (may be x) receives it when given; y = rmsnorm(x_new) * g when given
hipError_t iso_launch_rmsnorm(int dtype, const void *x, const void *delta_or_null, const void *delta2_or_null,
                              void *x_out_or_null, const void *g, void *y_or_null, int T, int H, float eps, hipStream_t s);
hipError_t iso_launch_rope_kv(int dtype, void *qkv, void *k_cache, void *v_cache, const float *cos_t,
                              const float *sin_t, int Tc, int q_offset, int nq, int nkv, int d, hipStream_t s);
hipError_t iso_launch_quant_rows(int dtype, void *part, void *q8, int T, int H, hipStream_t s);
hipError_t iso_launch_swiglu(int dtype, const void *gu, void *a, int T, int F, hipStream_t s);
hipError_t iso_launch_gemm_simple(int dtype, const void *a, const void *w, void *c, int M, int N, int K,
                                  hipStream_t s);
hipError_t iso_launch_gemm_bf16_mfma(const void *a, const void *w, void *c, int M, int N, int K, hipStream_t s);
bool iso_gemm_bf16_mfma_supported(int M, int N, int K);
hipError_t iso_launch_gemm_bf16_dtl(const void *a, const void *w, void *c, int M, int N, int K, int variant,
                                    iso_sk_ws *sk_or_null, hipStream_t s);
bool iso_gemm_bf16_dtl_supported(int M, int N, int K);
// which variant (1..6; -1: none; +8: plain main loop) a launch with `variant` resolves to
int iso_gemm_bf16_dtl_resolve(int M, int N, int K, int variant, const iso_sk_ws *sk_or_null);
// QKV projection with rotary embedding + KV-cache write in the epilogue (head_dim 128; resolved variant 1 or 6)
hipError_t iso_launch_gemm_qkv_rope_bf16(const void *a, const void *w, void *qkv, int M, int N, int K, int resolved,
                                         iso_sk_ws *sk_or_null, const float *cos_t, const float *sin_t, void *k_cache,
                                         void *v_cache, int q_offset, int nq, int nkv, hipStream_t s);
hipError_t iso_launch_gemm_swiglu_bf16(const void *a, const void *w, void *act, int M, int F, int K, int variant,
                                       iso_sk_ws *sk_or_null, hipStream_t s);
void iso_gemm_bf16_dtl_plan(int M, int N, int K, int num_wg, int *kind, int *team, int *grid);
size_t iso_gemm_sk_ws_bytes(int num_wg);   // device bytes a stream-K workspace for num_wg workgroups needs
int iso_gemm_sk_max_wg(void);
bool iso_gemm_swiglu_bf16_supported(int M, int F, int K);
bool iso_gemm_fp8_supported(int M, int N, int K);
bool iso_rmsnorm_fp8_supported(int H);
hipError_t iso_launch_rmsnorm_fp8(const void *x, const void *delta_or_null, const void *delta2_or_null, void *x_out_or_null,
                                  const void *g, void *q8, float *q_scale, int T, int H, float eps, hipStream_t s);
hipError_t iso_launch_quant_rows_fp8(const void *x, void *q, float *scale, int rows, int cols, hipStream_t s);
hipError_t iso_launch_gemm_fp8(const void *a8, const float *sa, const void *w8, const float *sw, void *c, int M, int N,
                               int K, int variant, iso_sk_ws *sk_or_null, hipStream_t s);
hipError_t iso_launch_gemm_swiglu_fp8(const void *a8, const float *sa, const void *w8, const float *sw, void *act, int M,
                                      int F, int K, int variant, iso_sk_ws *sk_or_null, hipStream_t s);
// stream-K with the workspace in a static device array (no allocation at call time)
hipError_t iso_gemm_static_setup(void);     // once per device, with that device current
size_t iso_gemm_static_scratch_bytes(void);
hipError_t iso_launch_gemm_bf16_sk_static(const void *a, const void *w, void *c, int M, int N, int K, unsigned *err_word,
                                          hipStream_t s);
// stream-K launch shape for nk k-slices (team size, grid, grouped mapping); returns the k-slices per team
long long iso_gemm_sk_plan(int M, int N, int nk, int num_wg, int *team, int *grid, int *grouped);
hipError_t iso_launch_attn_simple(int dtype, const void *q, const void *k, const void *v, void *out, int Tc,
                                  int q_offset, int kv_len, int nq, int nkv, int d, int q_stride, hipStream_t s);
hipError_t iso_launch_attn_bf16_mfma(const void *q, const void *k, const void *v, void *out, int Tc,
                                     int q_offset, int kv_len, int nq, int nkv, int d, int q_stride, hipStream_t s);
bool iso_attn_bf16_mfma_supported(int d);
hipError_t iso_launch_attn_bf16_dtl(const void *q, const void *k, const void *v, void *out, int Tc, int q_offset,
                                    int kv_len, int nq, int nkv, int d, int q_stride, int shape, int ksplit_req,
                                    const iso_attn_ws *ws_or_null, hipStream_t s);
size_t iso_attn_part_bytes(void);      // bytes of one partial state in an iso_attn_ws
bool iso_attn_bf16_dtl_supported(int d, int kv_len, int nkv);

// ---- small device helpers ----------------------------------------------------------------------
__device__ __forceinline__ float iso_to_f32(float v) { return v; }
__device__ __forceinline__ float iso_to_f32(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T iso_from_f32(float v);
template <> __device__ __forceinline__ float iso_from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t iso_from_f32<bf16_t>(float v) { return (bf16_t)v; }  // RNE

__device__ __forceinline__ float iso_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
// Raises a kernel's dynamic-LDS limit once per device (the attribute belongs to the function on the device that is
// current when it is set).  `done` is the caller's static mask of devices already served; ids beyond 63 are set every
// time.  Called from launchers only; host threads may race here (setting the attribute twice is harmless, the mask is
// atomic).
typedef std::atomic<unsigned long long> iso_dev_mask;
inline hipError_t iso_allow_lds(const void *kernel, int bytes, iso_dev_mask *done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && ((done->load(std::memory_order_acquire) >> dev) & 1ull)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev >= 0 && dev < 64) done->fetch_or(1ull << dev, std::memory_order_release);
    return e;
}
// Compute units of the current device (looked up once per device; 256 if the query fails).
inline int iso_num_cu(void) {
    static std::atomic<int> ncu_of[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    int n = ncu_of[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        ncu_of[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

__device__ __forceinline__ float iso_wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
