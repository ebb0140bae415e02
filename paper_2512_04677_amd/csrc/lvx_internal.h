// Internal declarations shared by the lvx translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "lvx.h"

typedef uint16_t bf16_t;  // raw bf16 bits in memory

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;

#define LVX_KEY_TILE 64  // keys per V^T tile in the cache and per LDS stage of the attention kernel

lvx_status_t lvx_fail(lvx_status_t code, const char *fmt, ...);

#define LVX_CHECK_HIP(expr)                                                                      \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess) return lvx_fail(LVX_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

#define LVX_REQUIRE(cond, code, ...)                         \
    do {                                                     \
        if (!(cond)) return lvx_fail((code), __VA_ARGS__);   \
    } while (0)

#define LVX_TRY(expr)                    \
    do {                                 \
        lvx_status_t st_ = (expr);       \
        if (st_ != LVX_OK) return st_;   \
    } while (0)

static inline bool lvx_aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

// ---- device helpers -------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
// round-to-nearest-even pack of two floats into two bf16 (lo = a, hi = b); maps to v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    bf16x2_t r;
    r[0] = (__bf16)a;
    r[1] = (__bf16)b;
    return *reinterpret_cast<uint32_t *>(&r);
}

// 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3)
__device__ __forceinline__ float gelu_tanh_f32(float x) {
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    const float e = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * u);
    return x * __builtin_amdgcn_rcpf(1.0f + e);
}
// direct-to-LDS load of 16 bytes per lane: LDS byte address = lds_addr (wave-uniform, goes to M0) + 16 * lane.
// The statement writes M0 and says so in its clobber list, so the compiler never assumes a value of its own survives in M0
// across it (clang notes that M0 is a reserved register it cannot save and restore around the statement: nothing here asks it to).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lvx_dma16(const void *gbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(gbase), "s"(lds_addr) : "memory", "m0");
}
#pragma clang diagnostic pop

#define LVX_LOG2E 1.4426950408889634f

// ---- cache handle (host) ----------------------------------------------------------------------
struct lvx_kvcache {
    lvx_cache_desc_t desc;
    int32_t sink_keys, chunk_keys, n_slots, cap_keys;  // cap_keys: capacity per head, multiple of LVX_KEY_TILE
    size_t layer_k_elems;                              // elements of K (= of V^T) per layer
    bf16_t *k_base;                                    // [layer][head][cap_keys][D]
    bf16_t *vt_base;                                   // [layer][head][cap_keys/64][D][64]
    lvx_ring_state_t *state;                           // [n_layers]
    float *sink_src;                                   // [layer][sink_keys][d] un-rotated sink keys in fp32, NULL until attached
    int32_t *sink_t;                                   // [n_layers] temporal index the sink keys are rotated to; < 0: see LVX_SINK_*
};
#define LVX_SINK_STATIC (-2)  /* keys were given already rotated (lvx_kvcache_set_sink) or there is no sink yet */
#define LVX_SINK_STALE (-1)   /* a source is installed, the cache's sink keys are not yet rotated */

static inline const bf16_t *lvx_cache_k(const lvx_kvcache *c, int layer) { return c->k_base + (size_t)layer * c->layer_k_elems; }
static inline const bf16_t *lvx_cache_vt(const lvx_kvcache *c, int layer) { return c->vt_base + (size_t)layer * c->layer_k_elems; }

// ---- internal launchers (all enqueue on `stream`, arguments already validated) ----------------
// Token-major K/V rows [n][ld] -> packed K [H][cap][D] rows key0.. and V^T tiles [H][cap/64][D][64] (k NULL: values only).
// n_batch > 1: that many independent row sets / packed arrays, batch_stride_src / batch_stride_dst elements apart.
lvx_status_t lvx_launch_pack_kv(const bf16_t *k, const bf16_t *v, int64_t ld, int n, int H, int D, int cap, int key0,
                                bf16_t *k_packed, bf16_t *vt_packed, hipStream_t stream, int n_batch = 1, int64_t batch_stride_src = 0,
                                int64_t batch_stride_dst = 0);
// Attention of q [n_q][ld_q] against packed K / V^T holding n_keys visible keys per head.
// Optional transform of the queries as the attention kernel loads them: RMSNorm over all d_model channels with the row's sum of
// squares given as n_parts partial sums (lvx_gemm_seg_t::sumsq) and a per-channel gain; the kernel also multiplies by
// scale * log2(e) and rounds to bf16 once (its pre-scaled mode).  Replaces a separate norm-only pass over q.
struct lvx_attn_qnorm_t {
    const float *sumsq;  // [n_q][ld] partial sums of squares
    const float *gain;   // [d_model]
    int32_t n_parts, ld, d_model;
    float eps;
};
lvx_status_t lvx_launch_attention(const bf16_t *q, int64_t ld_q, int n_q, int H, int D, const bf16_t *k_packed,
                                  const bf16_t *vt_packed, int cap, int n_keys, float scale, bf16_t *out, int64_t ld_out,
                                  hipStream_t stream, uint32_t *amax_slots = nullptr, bool q_prescaled = false,
                                  const lvx_attn_qnorm_t *qnorm = nullptr);
// out = bf16((x ? x : 0) + dt * h) with h in fp32: the Euler step of the stage (x given) or the narrowing of a block's
// fp32 residual stream (x NULL, dt 1).
lvx_status_t lvx_launch_euler(const bf16_t *x, const float *h, float dt, bf16_t *out, size_t n_elems, hipStream_t stream);
lvx_status_t lvx_launch_widen(const bf16_t *src, float *dst, size_t n_elems, hipStream_t stream);
lvx_status_t lvx_launch_layernorm(const void *x, int x_is_f32, int64_t ldx, const float *shift, const float *scale, float eps,
                                  int n_tokens, int d, bf16_t *u, int64_t ldu, hipStream_t stream, uint32_t *amax_slots = nullptr);
// Strided row copy [n_rows][row_elems] (row_elems % 8 == 0), bit-exact.
lvx_status_t lvx_launch_copy_rows(const bf16_t *src, int64_t ld_src, bf16_t *dst, int64_t ld_dst, int n_rows, int row_elems,
                                  hipStream_t stream);
// RoPE of token-major fp32 rows written straight into packed K rows [H][cap][D] starting at key 0 (no norm), for n_layers
// consecutive layers in one launch (strides in elements between the layers' sources and between their packed K arrays).
lvx_status_t lvx_launch_rope_to_packed_k(const lvx_rope_desc_t *desc, const float *src, int64_t ld_src, int n_tokens, int t0,
                                         bf16_t *k_packed, int cap, int n_layers, int64_t layer_stride_src, int64_t layer_stride_dst,
                                         hipStream_t stream);
// RMSNorm + RoPE with q rows in bf16 and k rows in fp32 (outputs bf16).
lvx_status_t lvx_launch_rope_qk(const lvx_rope_desc_t *desc, const bf16_t *q_in, int64_t ld_q, const void *k_in, int k_is_f32, int64_t ld_k,
                                const float *g_q, const float *g_k, int n_tokens, int t0, bf16_t *q_out, int64_t ld_out, bf16_t *k_out,
                                int64_t ld_out_k, int64_t ld_out_head_k, float q_scale, hipStream_t stream);
// Append in two steps for a producer that writes the chunk's keys into the cache itself: begin validates and names the slot
// (nothing changes), commit records the chunk in the layer's ring state.
lvx_status_t lvx_cache_append_begin(const lvx_kvcache *c, int layer, int64_t chunk_index, lvx_slot_info_t *info);
void lvx_cache_append_commit(lvx_kvcache *c, int layer, int64_t chunk_index, const lvx_slot_info_t *info);
// RMSNorm (no rotation) of n_batch sets of token-major rows (bf16, or fp32 with strides in fp32 elements), written straight into n_batch packed K arrays [H][cap][D]
// from key 0 on; gains[b] is batch b's gain vector (NULL: that batch is copied un-normalised).  n_batch <= LVX_GEMM_MAX_SEGS.
lvx_status_t lvx_launch_norm_to_packed_k(const lvx_rope_desc_t *desc, const void *src, int src_is_f32, int64_t ld_src, int n_tokens,
                                         const float *const *gains, bf16_t *k_packed, int cap, int n_batch, int64_t batch_stride_src,
                                         int64_t batch_stride_dst, hipStream_t stream);
// y = x / sqrt(mean(x^2) + eps) * g on fp32 rows, fp32 out, no rounding (g NULL: plain copy): the sink warm-up's un-rotated keys.
lvx_status_t lvx_launch_rmsnorm_f32(const lvx_rope_desc_t *desc, const float *x, int64_t ld_in, const float *g, int n_tokens, float *y,
                                    int64_t ld_out, hipStream_t stream);
lvx_status_t lvx_launch_widen_rows(const bf16_t *src, int64_t ld_src, float *dst, int64_t ld_dst, int n_rows, int row_elems,
                                   hipStream_t stream);
// the layer's fp32 sink source is in place: install its values, mark its keys stale (they await the next rotation)
lvx_status_t lvx_sink_install_values(lvx_kvcache *c, int layer, const bf16_t *v, int64_t ld, hipStream_t stream);
// Row addressing of the GEMM's A operand for an implicit-GEMM 3x3x3 convolution over a zero-padded channels-last volume
// P[frame][H+2][W+2][C]: output pixel m = (t, y, x) reads, for tap (dt, dy, dx), the C channels at P[t+dt][y+dy][x+dx].
// K runs tap-major (27 taps x C channels); C % 64 == 0 so that a 64-wide K slab lies inside one tap.
struct lvx_conv_map_t {
    int32_t enabled;
    int32_t H, W, C;           // output frame size and input channels
    int32_t slabs_per_tap;     // C / 64
    int32_t row_pitch;         // elements between padded rows: (W + 2) * C
    int32_t frame_pitch;       // elements between padded frames: (H + 2) * (W + 2) * C
};
lvx_status_t lvx_launch_conv_gemm(const bf16_t *P, const lvx_conv_map_t &cm, const bf16_t *Wt, int64_t ldw, const float *bias, int act,
                                  bf16_t *Y, int64_t ldy, int M, int N, hipStream_t stream);
// C1[M][N1] = A W1^T (bf16, or fp32 if c1_is_f32), C2[M][N2] = A W2^T (bf16) in one launch, plain store.
lvx_status_t lvx_launch_linear_dual(const bf16_t *A, int64_t lda, const bf16_t *W1, const bf16_t *W2, int64_t ldw, void *C1, int64_t ldc1,
                                    int c1_is_f32, bf16_t *C2, int64_t ldc2, int M, int N1, int N2, int K, hipStream_t stream);
// Several projections of the same activations in one GEMM launch: segment i owns the column tiles from tn_begin on (filled in
// by the launcher) and has its own weight matrix [N][ldw], output (bf16, or fp32 if f32), output row stride and width.
#define LVX_GEMM_MAX_SEGS 16
struct lvx_gemm_seg_t {
    const bf16_t *W;
    void *C;
    int64_t ldc;
    int32_t N, tn_begin, f32, ld_sumsq;
    // NULL, or [M][ld_sumsq] floats: besides the bf16 store, every wave leaves the sum of squares of its 64 columns (taken on the
    // fp32 accumulators) of each of its rows at column index (column tile within the segment) * 4 + (wave column): the partial
    // sums of a row's RMS, added up in a fixed order by the consumer (no atomics: results stay bit-reproducible).  N % 256 == 0.
    float *sumsq;
};
#define LVX_GEMM_SUMSQ_PARTS(N_) ((N_) / 64)
struct lvx_gemm_segs_t {
    int32_t n, pad;
    lvx_gemm_seg_t s[LVX_GEMM_MAX_SEGS];
};
lvx_status_t lvx_launch_linear_segments(const bf16_t *A, int64_t lda, int64_t ldw, const lvx_gemm_segs_t &segs, int M, int K, hipStream_t stream);
// internal epilogue id of the GEMM kernel: plain store per segment (bf16 or fp32)
#define LVX_EPI_SEGMENTS 100
// Per-tensor dynamic FP8 quantisation of a bf16 matrix.  The amax is collected in an array of LVX_AMAX_SLOTS fp32 bit patterns
// (256 bytes, zero before the producers write): either by lvx_launch_fp8_amax, or by the kernel that produced x (attention,
// the GELU epilogue of an FP8 linear, the LayerNorm kernel with one atomic per workgroup), which saves the extra pass.
// lvx_launch_fp8_quant reduces the slots, writes codes and scale and clears `zero_slots` (another slot array, may be NULL)
// for the next producer.
#define LVX_AMAX_SLOTS 64
lvx_status_t lvx_launch_fp8_amax(const bf16_t *x, int64_t ld, int rows, int cols, uint32_t *amax_slots, hipStream_t stream);
lvx_status_t lvx_launch_fp8_quant(const bf16_t *x, int64_t ld, int rows, int cols, uint8_t *q, int64_t ldq, const uint32_t *amax_slots,
                                  uint32_t *zero_slots, float *scale, hipStream_t stream);
// fill + amax + quant on one slot array
lvx_status_t lvx_launch_fp8_quantize(const bf16_t *x, int64_t ld, int rows, int cols, uint8_t *q, int64_t ldq, uint32_t *amax_slots,
                                     float *scale, hipStream_t stream);
lvx_status_t lvx_launch_linear_fp8(const void *dev_aq, int64_t lda, const float *dev_scale_a, const void *dev_wq, int64_t ldw,
                                   const float *dev_scale_w, void *dev_c, int64_t ldc, int32_t M, int32_t N, int32_t K, lvx_epilogue_t epi,
                                   const void *dev_resid, int64_t ldr, const float *dev_gate, uint32_t *amax_slots, hipStream_t stream);
// Optional HIP-event timing of a kernel class on the caller's stream (lvx_profile_set / lvx_profile_read): the events are
// recorded around the launches made while the object lives.
struct lvx_prof_scope_t {
    hipStream_t st;
    void *pair;
    lvx_prof_scope_t(int kind, hipStream_t stream);
    ~lvx_prof_scope_t();
};
// Packed K [H][cap][D] / V^T tiles -> token-major rows [n_keys][ld] from key first_key on (bit-exact).
lvx_status_t lvx_launch_gather_kv(const bf16_t *k_packed, const bf16_t *vt_packed, int cap, int H, int D, int first_key, int n_keys,
                                  bf16_t *k_out, bf16_t *v_out, int64_t ld, hipStream_t stream);
// Zero fill by kernel (not a memset node, so callers may capture it in a HIP graph); bytes % 16 == 0.
lvx_status_t lvx_launch_fill_zero(void *dst, size_t bytes, hipStream_t stream);
