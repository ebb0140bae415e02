/*
 * lvx — C ABI of the MI355X (gfx950) hot path of one denoising stage of a streaming causal video DiT
 * (Live Avatar, arXiv 2512.04677).
 *
 * Conventions (all entry points):
 *   - Plain C, no exceptions.  Every call returns lvx_status_t; on failure lvx_last_error() gives a
 *     thread-local message.  Argument checks happen on the host before anything is enqueued.
 *   - "dev" pointers are device (HBM) addresses owned by the caller; "host" pointers are ordinary host
 *     memory.  The library never allocates or frees device memory and never synchronises: all work is
 *     enqueued on the given HIP stream (lvx_stream_t is a hipStream_t; NULL = the default stream).
 *   - Activations are bf16, row-major, token-major: element (token n, channel c) at base[n*ld + c],
 *     channel c = head*head_dim + dim.  `ld` is a row stride in ELEMENTS.  Device pointers must be
 *     16-byte aligned and ld a multiple of 8.
 *   - Linear weights are bf16, row-major [out_features][in_features], no bias.
 *   - Gains and modulation vectors are fp32.
 *   - The KV cache's internal layout is private to the library (K head-major, V stored transposed in
 *     64-key tiles so that both are direct MFMA operands); lvx_kvcache_gather reads it back in the
 *     token-major layout for checks and for off-loading.
 */
#ifndef LVX_H
#define LVX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LVX_OK = 0,
    LVX_ERR_INVALID_ARG = 1, /* null / misaligned pointer, negative size, bad enum */
    LVX_ERR_SHAPE = 2,       /* a size the kernels do not support or that does not match the descriptor */
    LVX_ERR_STATE = 3,       /* call order violated (chunk index out of sequence, sink not set, ...) */
    LVX_ERR_UNSUPPORTED = 4, /* valid request outside what is built (e.g. head_dim not 64/128) */
    LVX_ERR_HIP = 5          /* a HIP runtime call failed; message holds hipGetErrorString */
} lvx_status_t;

typedef void *lvx_stream_t; /* hipStream_t */

const char *lvx_last_error(void);
/* Library version string, e.g. "lvx 0.1 gfx950". */
const char *lvx_version(void);

/* ------------------------------------------------------------------------------------------------
 * Rolling KV cache (paper Eq. 1; Alg. 3 / Alg. 4 cache lines; Sec. 3.3 "History Corrupt" and sink frame).
 *
 * One cache = one denoising timestep's state for all layers: per layer a sink segment of
 * sink_frames*frame_h*frame_w keys that is never evicted, followed by window_chunks+1 chunk slots of
 * chunk_frames*frame_h*frame_w keys each.  The forward of chunk i must see its own K/V (blocks attend
 * to themselves in full, Sec. 3.2) and the `window_chunks` chunks before it, so the chunk's K/V are
 * written first, into slot i mod (window_chunks+1), overwriting chunk i-(window_chunks+1): that is the
 * cache update of Alg. 3 (drop the oldest entry of a full cache, then append) with the append moved before the attention.  Attention is invariant to
 * key order (no mask, K carries its rotary phase), so the visible keys are always the contiguous prefix
 *   [0, sink_keys + min(i+1, window_chunks+1)*chunk_keys).
 * ------------------------------------------------------------------------------------------------ */
typedef struct {
    int32_t n_layers;      /* 40 */
    int32_t n_heads;       /* 40 */
    int32_t head_dim;      /* 128 (64 also supported) */
    int32_t frame_h;       /* 30  tokens per latent-frame column */
    int32_t frame_w;       /* 52 */
    int32_t chunk_frames;  /* 3  latent frames per block (Sec. 4.1) */
    int32_t window_chunks; /* 4  past blocks kept, w in Eq. 1 */
    int32_t sink_frames;   /* 1 */
} lvx_cache_desc_t;

typedef struct lvx_kvcache lvx_kvcache_t; /* opaque host-side handle */

/* Result of the ring arithmetic for one append. */
typedef struct {
    int32_t slot;           /* chunk slot written: chunk_index mod (window_chunks+1) */
    int64_t evicted_chunk;  /* chunk index overwritten, -1 while the ring is filling */
    int32_t n_valid_chunks; /* chunks held after the append, including the new one */
    int32_t key_offset;     /* first key row of the slot, counted from the sink's first key */
    int32_t key_count;      /* visible keys after the append (sink + valid chunks) */
} lvx_slot_info_t;

#define LVX_MAX_SLOTS 16
typedef struct {
    int64_t last_chunk;                 /* last chunk index appended to this layer, -1 if none */
    int32_t sink_set;                   /* 1 once lvx_kvcache_set_sink ran for this layer */
    int32_t n_valid_chunks;
    int32_t key_count;
    int32_t n_slots;                    /* window_chunks+1 */
    int64_t slot_chunk[LVX_MAX_SLOTS];  /* chunk index living in each slot, -1 if empty */
} lvx_ring_state_t;

/* Bytes of device storage the caller must provide for K and V of all layers. 0 on a bad descriptor. */
size_t lvx_kvcache_bytes(const lvx_cache_desc_t *desc /* host */);

/* Pure host arithmetic of the ring (no device, no handle): where chunk `chunk_index` goes and what it
 * evicts.  Errors: null pointers, bad descriptor, negative chunk_index. */
lvx_status_t lvx_ring_slot(const lvx_cache_desc_t *desc /* host */, int64_t chunk_index, lvx_slot_info_t *out /* host */);

/* Creates the host handle over caller-owned device storage (>= lvx_kvcache_bytes, 256-byte aligned) and
 * enqueues a zero fill of it (stale keys past the visible prefix must be finite).  The storage must stay
 * alive until lvx_kvcache_destroy.  Errors: INVALID_ARG (null/misaligned), SHAPE (bad descriptor, storage too
 * small), UNSUPPORTED (head_dim not in {64,128}, window_chunks+1 > LVX_MAX_SLOTS). */
lvx_status_t lvx_kvcache_init(const lvx_cache_desc_t *desc /* host */, void *dev_storage, size_t bytes,
                              lvx_stream_t stream, lvx_kvcache_t **out /* host */);
/* Frees host state only. */
lvx_status_t lvx_kvcache_destroy(lvx_kvcache_t *cache);

/* Writes the sink frame's K (already normalised and rotated) and V, token-major [sink_keys][ld], into the
 * never-evicted segment of `layer` (Sec. 3.3: the sink stays in KV memory permanently). */
lvx_status_t lvx_kvcache_set_sink(lvx_kvcache_t *cache, int32_t layer, const void *dev_k, const void *dev_v,
                                  int64_t ld, lvx_stream_t stream);

/* Cache update of Alg. 3 (a full cache drops its oldest entry, then the new one is appended): writes chunk `chunk_index`'s K-hat and V, token-major
 * [chunk_keys][ld], into its ring slot of `layer`; the oldest chunk is overwritten once the ring is full; the
 * sink segment is untouched.  chunk_index must be last_chunk+1 for that layer (0 first) else LVX_ERR_STATE.
 * `out` (host, may be NULL) receives the slot arithmetic.  The copy is bit-exact. */
lvx_status_t lvx_chunk_append_evict(lvx_kvcache_t *cache, int32_t layer, const void *dev_k, const void *dev_v,
                                    int64_t ld, int64_t chunk_index, lvx_slot_info_t *out /* host */,
                                    lvx_stream_t stream);

lvx_status_t lvx_kvcache_get_state(const lvx_kvcache_t *cache, int32_t layer, lvx_ring_state_t *out /* host */);
/* Restores ring bookkeeping after the caller restored the device storage (resume after off-loading). */
lvx_status_t lvx_kvcache_set_state(lvx_kvcache_t *cache, int32_t layer, const lvx_ring_state_t *in /* host */);

/* Reads keys [first_key, first_key+n_keys) of `layer` back as token-major [n_keys][ld] K and V (bit-exact). */
lvx_status_t lvx_kvcache_gather(const lvx_kvcache_t *cache, int32_t layer, int32_t first_key, int32_t n_keys,
                                void *dev_k_out, void *dev_v_out, int64_t ld, lvx_stream_t stream);

/* ------------------------------------------------------------------------------------------------
 * Fused Q/K RMSNorm + 3-D rotary embedding (rotary indices per latent frame: Appendix D "Rolling RoPE";
 * the axis split, theta and the norm are the workload's, not the paper's).
 *   y = x / sqrt(mean_c(x^2) + eps) * g          over all n_heads*head_dim channels of a token (g NULL: skip)
 *   pair k of axis a (dims base_a+2k, base_a+2k+1):  (u,v) -> (u cos - v sin, u sin + v cos),
 *   angle = pos_a * theta^(-2k/axes[a]),  pos = (t0 + n / (frame_h*frame_w), (n / frame_w) % frame_h, n % frame_w).
 * Angles are formed in fp64 on the device, the rest in fp32.  In-place (out == in) is allowed.
 * Either of q / k may be NULL (then its output is ignored).
 * ------------------------------------------------------------------------------------------------ */
typedef struct {
    int32_t n_heads, head_dim;
    int32_t axes[3];     /* dims given to t, y, x; even, sum = head_dim (44, 42, 42) */
    float theta;         /* 10000 */
    int32_t frame_h, frame_w;
    float eps;           /* 1e-6 */
    int32_t apply_rope;  /* 0 = norm only (cross-attention) */
} lvx_rope_desc_t;

lvx_status_t lvx_rope3d(const lvx_rope_desc_t *desc /* host */, const void *dev_q_in, const void *dev_k_in, int64_t ld_in,
                        const float *dev_g_q, const float *dev_g_k, int32_t n_tokens, int32_t t0,
                        void *dev_q_out, void *dev_k_out, int64_t ld_out, lvx_stream_t stream);
/* The same with q_in / k_in in fp32 (ld_in in fp32 elements; outputs bf16): what the block runs on the un-rounded q | k
 * columns of its QKV projection. */
lvx_status_t lvx_rope3d_f32in(const lvx_rope_desc_t *desc /* host */, const float *dev_q_in, const float *dev_k_in, int64_t ld_in,
                              const float *dev_g_q, const float *dev_g_k, int32_t n_tokens, int32_t t0,
                              void *dev_q_out, void *dev_k_out, int64_t ld_out, lvx_stream_t stream);

/* ------------------------------------------------------------------------------------------------
 * Rolling RoPE and the adaptive attention sink (Sec. 3.3; Appendix D; Phi(sink) and the sink assignment of Alg. 3 /
 * Alg. 4).  The sink's rotary temporal index is re-assigned at every block step so that its distance to the current
 * block stays bounded; the paper rewrites the cached sink keys in place.  Here the un-rotated (normalised) sink keys are
 * kept beside the cache, in fp32, and every re-assignment rotates them afresh into the cache's sink rows, so rotations never
 * compound their bf16 roundings over a long rollout and a sink key is rounded to bf16 once, after its rotation.  The index
 * itself (App. D leaves it at a small offset ahead of the current block) is the caller's: the paper gives no value.
 *
 *   lvx_sink_source_bytes           device bytes for the un-rotated sink keys of all layers ([layer][sink_keys][d] fp32)
 *   lvx_kvcache_attach_sink_source  hands that storage (caller-owned, 256-byte aligned, alive as long as the handle) over
 *   lvx_kvcache_reset_sink          installs a sink for `layer`: dev_k_src = normalised, NOT rotated keys, dev_v = values,
 *                                   both token-major [sink_keys][ld] bf16 (the keys widened exactly to fp32, the values copied
 *                                   bit for bit).  The ring is untouched.  Until
 *                                   the next lvx_sink_rope_update the layer's sink keys are stale and lvx_chunk_attention /
 *                                   lvx_dit_block / lvx_denoise_stage return LVX_ERR_STATE for it.
 *   lvx_sink_rope_update            Phi: sink keys of `layer` (-1: every layer) := RoPE(source) with the sink's first frame
 *                                   at temporal index t_sink, spatial indices from the frame grid; values untouched.
 *   lvx_kvcache_get_sink_index      last t_sink applied to `layer`; -1 = reset but not rotated; -2 = static sink / none
 *   lvx_kvcache_set_sink_index      restores that bookkeeping after the caller restored the device storage (resume, as
 *                                   lvx_kvcache_set_state does for the ring)
 *   lvx_kvcache_gather_sink_source  reads the stored source back, token-major fp32 [sink_keys][ld] (ld in fp32 elements; bit-exact)
 * Errors: STATE without attached storage, on a layer whose sink came from lvx_kvcache_set_sink (already rotated, no
 * source) or on a cache without sink segment; SHAPE if the rope descriptor disagrees with the cache; INVALID_ARG else.
 * ------------------------------------------------------------------------------------------------ */
size_t lvx_sink_source_bytes(const lvx_cache_desc_t *desc /* host */);
lvx_status_t lvx_kvcache_attach_sink_source(lvx_kvcache_t *cache, void *dev_storage, size_t bytes);
lvx_status_t lvx_kvcache_reset_sink(lvx_kvcache_t *cache, int32_t layer, const void *dev_k_src, const void *dev_v, int64_t ld,
                                    lvx_stream_t stream);
lvx_status_t lvx_sink_rope_update(lvx_kvcache_t *cache, const lvx_rope_desc_t *rope /* host */, int32_t layer, int32_t t_sink,
                                  lvx_stream_t stream);
lvx_status_t lvx_kvcache_get_sink_index(const lvx_kvcache_t *cache, int32_t layer, int32_t *out /* host */);
lvx_status_t lvx_kvcache_set_sink_index(lvx_kvcache_t *cache, int32_t layer, int32_t t_sink);
lvx_status_t lvx_kvcache_gather_sink_source(const lvx_kvcache_t *cache, int32_t layer, void *dev_k_src_out, int64_t ld,
                                            lvx_stream_t stream);

/* ------------------------------------------------------------------------------------------------
 * Chunk-to-cache attention (Eq. 1; Appendix C attention paragraph: current tokens against the concatenation
 * of cached K/V and themselves):  O[n,h,:] = softmax_m(scale * <q[n,h,:], K[m,h,:]>) V[m,h,:] over the visible
 * prefix of `layer` (every key visible, no mask).  q, out: [n_q][ld] bf16.  bf16 MFMA, fp32 online softmax.
 * Errors: STATE if the layer has no visible keys yet.
 * ------------------------------------------------------------------------------------------------ */
lvx_status_t lvx_chunk_attention(const lvx_kvcache_t *cache, int32_t layer, const void *dev_q, int64_t ld_q,
                                 int32_t n_q, float scale, void *dev_out, int64_t ld_out, lvx_stream_t stream);
/* The same for queries that already carry the softmax scale: dev_q holds q * (scale * log2(e)), folded in before q was rounded
 * to bf16 (what the DiT block's RMSNorm + RoPE kernel emits), so that softmax_m(scale <q,K>) = 2^(<q',K>) / sum.  The kernel
 * then starts its score accumulators at minus the softmax reference and the score leaves the matrix core as the exponent.
 * Folding the factor into an ALREADY rounded q would round it a second time; for that case use lvx_chunk_attention. */
lvx_status_t lvx_chunk_attention_prescaled(const lvx_kvcache_t *cache, int32_t layer, const void *dev_q_scaled, int64_t ld_q,
                                           int32_t n_q, void *dev_out, int64_t ld_out, lvx_stream_t stream);

/* ------------------------------------------------------------------------------------------------
 * Building blocks of the DiT block, exported for unit parity tests.
 * ------------------------------------------------------------------------------------------------ */
typedef enum {
    LVX_EPI_STORE = 0,      /* C = A W^T */
    LVX_EPI_GELU_TANH = 1,  /* C = gelu_tanh(A W^T) */
    LVX_EPI_RESID_GATE = 2, /* C = R + gate[n] * (A W^T); gate NULL = 1; C may alias R */
    LVX_EPI_RESID_GATE_F32 = 3, /* same, with C and R in fp32 (ldc, ldr in fp32 elements): the in-block residual stream */
    LVX_EPI_BIAS = 4,       /* C = A W^T + bias[n]; the bias (fp32 [N], NULL = 0) is passed in the gate argument */
    LVX_EPI_BIAS_SILU = 5,  /* C = silu(A W^T + bias[n]) */
    LVX_EPI_STORE_F32 = 6   /* C = A W^T with C in fp32 (ldc in fp32 elements): no rounding of the accumulator */
} lvx_epilogue_t;

/* C[M][N] = epilogue(A[M][K] * W[N][K]^T), bf16 in/out, fp32 accumulate on MFMA.  K % 64 == 0, N % 8 == 0. */
lvx_status_t lvx_linear(const void *dev_a, int64_t lda, const void *dev_w, int64_t ldw, void *dev_c, int64_t ldc,
                        int32_t M, int32_t N, int32_t K, lvx_epilogue_t epi, const void *dev_resid, int64_t ldr,
                        const float *dev_gate, lvx_stream_t stream);

/* Two projections of the same activations in one launch (App. C linears):  C1[M][N1] = A W1^T,  C2[M][N2] = A W2^T, plain
 * store, W1 / W2 share the row stride ldw.  c1_is_f32 != 0: C1 is fp32 (ldc1 in fp32 elements), its accumulators are stored
 * un-rounded -- what a key projection wants, whose result is normalised and rotated before the one rounding to bf16 that the
 * cache holds.  C2 is always bf16.  The block's own launches are built on the same segment mechanism: q | k (fp32) | v of the
 * self-attention in one launch, the context's K (fp32) and V of a group of layers in one launch.  K % 64 == 0, N1, N2 % 8 == 0. */
lvx_status_t lvx_linear_dual(const void *dev_a, int64_t lda, const void *dev_w1, const void *dev_w2, int64_t ldw, void *dev_c1,
                             int64_t ldc1, int32_t c1_is_f32, void *dev_c2, int64_t ldc2, int32_t M, int32_t N1, int32_t N2, int32_t K,
                             lvx_stream_t stream);

/* FP8 linears (Appendix C, FP8 quantisation paragraph: every linear of the DiT runs in E4M3 with one dynamic scale per tensor).
 *   lvx_fp8_quantize: x bf16 [rows][ld] -> q [rows][ldq] E4M3 codes (OCP form: bias 7, largest finite value 448) and one fp32
 *     dequantisation scale = amax/448 (1 for an all-zero tensor), amax = max|x| over the whole matrix:
 *     code = E4M3(x * (448/amax)), nearest-even, saturating; scale factors and that product are formed in fp32.
 *     dev_scratch256: 256 bytes of device scratch (16-byte aligned).  cols % 16 == 0, ldq % 16 == 0.  Used for weights
 *     (once) and activations (every call) alike.
 *   lvx_linear_fp8: C[M][N] = epilogue(scale_a * scale_w * (Aq[M][K] . Wq[N][K]^T)), fp32 accumulate on the FP8 matrix
 *     cores, C / R / gate and the epilogues as in lvx_linear.  K % 128 == 0, N % 8 == 0, lda and ldw in bytes, % 16 == 0. */
lvx_status_t lvx_fp8_quantize(const void *dev_x, int64_t ld, int32_t rows, int32_t cols, void *dev_q, int64_t ldq,
                              void *dev_scratch256, float *dev_scale, lvx_stream_t stream);
lvx_status_t lvx_linear_fp8(const void *dev_aq, int64_t lda, const float *dev_scale_a, const void *dev_wq, int64_t ldw,
                            const float *dev_scale_w, void *dev_c, int64_t ldc, int32_t M, int32_t N, int32_t K,
                            lvx_epilogue_t epi, const void *dev_resid, int64_t ldr, const float *dev_gate, lvx_stream_t stream);

/* lvx_fp8_quantize for callers that cannot allocate device memory -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc -- and so have no scratch buffer to hand over: same inputs, outputs, arithmetic and result
 * (bit for bit), but the amax slots live in a 256-byte array inside the library (one per GPU, held until the process ends)
 * instead of dev_scratch256.  The call allocates and frees nothing and, like every other entry point, does not synchronise;
 * the array is cleared by a kernel at the start of every call.  Tensors of more than LVX_FP8_QUANTIZE_STATIC_MAX_ELEMS elements
 * are refused (LVX_ERR_SHAPE).  All calls on one GPU share that GPU's array: two calls whose work overlaps in time on one GPU
 * (different streams, or two threads) race on it and give wrong scales -- serialise them, or use lvx_fp8_quantize with one
 * scratch buffer per stream.  The first call on a device looks the array's address up (hipGetSymbolAddress); make that call
 * outside any stream capture. */
#define LVX_FP8_QUANTIZE_STATIC_MAX_ELEMS (1ll << 31)
lvx_status_t lvx_fp8_quantize_static(const void *dev_x, int64_t ld, int32_t rows, int32_t cols, void *dev_q, int64_t ldq,
                                     float *dev_scale, lvx_stream_t stream);

/* u = LayerNorm(x) * (1 + scale) + shift, no affine, biased variance, eps inside the root.  shift/scale fp32 [d]
 * or NULL (0).  x, u: [n][ld] bf16. */
lvx_status_t lvx_layernorm_modulate(const void *dev_x, int64_t ldx, const float *dev_shift, const float *dev_scale,
                                    float eps, int32_t n_tokens, int32_t d, void *dev_u, int64_t ldu, lvx_stream_t stream);

/* ------------------------------------------------------------------------------------------------
 * DiT block and denoise stage (Alg. 4, DiT-device branch: forward with the local rolling cache, cache update,
 * Euler step x <- x + v dt).  Block wiring (the paper defers to its base architecture; this is the workload's):
 *   u  = LN(x)(1+scale1)+shift1;  [q|k|v] = u W_qkv^T;  q^,k^ = RoPE(RMSNorm(q,k));  append(k^, v);
 *   x += gate1 * (Attn(q^, cache) W_o^T);
 *   x += Attn(RMSNorm(LN(x) Wc_q^T), RMSNorm(ctx Wc_k^T), ctx Wc_v^T) Wc_o^T;
 *   x += gate2 * (gelu_tanh((LN(x)(1+scale2)+shift2) W_1^T) W_2^T).
 * mod6: fp32 [6][d] = shift1, scale1, gate1, shift2, scale2, gate2; NULL = 0,0,1,0,0,1.
 * Weight rows may be padded (ldw_d / ldw_ffn): a row stride of in_features + 64 elements keeps consecutive rows off the
 * same memory channel when in_features * 2 bytes is a multiple of 2 KiB (5120 and 13824 both are) and is measurably
 * faster; the library pads its own workspace rows the same way.
 * ------------------------------------------------------------------------------------------------ */
typedef struct {
    const void *W_qkv;  /* [3d][d] rows: q, k, v */
    const void *W_o;    /* [d][d] */
    const void *Wc_q, *Wc_k, *Wc_v, *Wc_o; /* [d][d] */
    const void *W_1;    /* [ffn][d] */
    const void *W_2;    /* [d][ffn] */
    const float *g_q, *g_k;   /* [d] self-attention RMSNorm gains, NULL = no norm */
    const float *gc_q, *gc_k; /* [d] cross-attention RMSNorm gains, NULL = no norm */
} lvx_block_weights_t;

/* FP8 form of a block's linear weights (Appendix C): E4M3 codes from lvx_fp8_quantize, one per-tensor scale each (the fused
 * QKV matrix is one tensor).  Shapes as in lvx_block_weights_t, row strides ldw8_d / ldw8_ffn bytes. */
typedef struct {
    const void *W_qkv, *W_o, *Wc_q, *Wc_k, *Wc_v, *Wc_o, *W_1, *W_2;
    const float *scales; /* device, 8 floats: dequantisation scales in the order of the pointers above */
} lvx_block_weights_fp8_t;

typedef struct {
    int32_t n_layers;
    int32_t d_ffn;
    int32_t ldw_d;                     /* row stride (elements) of the weights with in_features = d_model; 0 = dense */
    int32_t ldw_ffn;                   /* row stride (elements) of W_2 (in_features = d_ffn); 0 = dense */
    lvx_rope_desc_t rope;              /* n_heads*head_dim = d_model; must agree with the cache descriptor */
    const lvx_block_weights_t *blocks; /* host array [n_layers] of device pointers */
    /* NULL: bf16 linears.  Else host array [n_layers]: every linear of the block quantises its input activation per tensor
     * (dynamically, each call) and multiplies on the FP8 matrix cores; the bf16 weight pointers in `blocks` are then unused
     * (may be NULL), its RMSNorm gains are still read.  d_model and d_ffn must then be multiples of 128. */
    const lvx_block_weights_fp8_t *blocks_fp8;
    int32_t ldw8_d, ldw8_ffn;          /* row strides (bytes) of the FP8 weights; 0 = dense */
} lvx_stage_t;

size_t lvx_workspace_bytes(const lvx_stage_t *stage /* host */, int32_t n_tokens, int32_t n_ctx);

/* The cross-attention keys and values of layers [layer0, layer0 + n_layers) for one context, exactly as the blocks compute and
 * read them (the conditions C_i of Alg. 3 / Alg. 4 are one set per forward, so a stage prepares them for a group of layers in
 * one GEMM launch): K = RMSNorm(ctx Wc_k^T) * gc_k, V = ctx Wc_v^T, read back token-major as [n_layers][n_ctx][ld] bf16 each.
 * Exported for parity checks of that path; the blocks keep these tensors in the attention kernel's packed layout inside the
 * workspace.  n_layers is at most the stage's own group size (at most 8; the group is sized so that its tiles fill whole rounds
 * of the chip: 5 layers for 544 context rows at d_model 5120) -- LVX_ERR_SHAPE otherwise; bf16 stages only;
 * workspace >= lvx_workspace_bytes(stage, 1, n_ctx). */
lvx_status_t lvx_context_kv(const lvx_stage_t *stage /* host */, int32_t layer0, int32_t n_layers, const void *dev_ctx, int32_t n_ctx,
                            void *dev_k_out, void *dev_v_out, int64_t ld, void *dev_workspace, size_t ws_bytes, lvx_stream_t stream);

/* One block on the current chunk.  x_inout [n_tokens][d] bf16 (ld = d); ctx [n_ctx][d] bf16; t0 = temporal rotary
 * index of the chunk's first frame; n_tokens must equal the cache's chunk size.  workspace: device scratch of
 * lvx_workspace_bytes, 256-byte aligned. */
lvx_status_t lvx_dit_block(const lvx_stage_t *stage /* host */, int32_t layer, lvx_kvcache_t *cache, void *dev_x_inout,
                           int32_t n_tokens, const void *dev_ctx, int32_t n_ctx, const float *dev_mod6,
                           int64_t chunk_index, int32_t t0, void *dev_workspace, size_t ws_bytes, lvx_stream_t stream);

/* The same block on an fp32 residual stream x_inout [n_tokens][d] (what lvx_denoise_stage iterates between its widening
 * of the bf16 input and its Euler step; exported so that a stage can be checked layer by layer). */
lvx_status_t lvx_dit_block_f32(const lvx_stage_t *stage /* host */, int32_t layer, lvx_kvcache_t *cache, float *dev_x_inout,
                               int32_t n_tokens, const void *dev_ctx, int32_t n_ctx, const float *dev_mod6, int64_t chunk_index,
                               int32_t t0, void *dev_workspace, size_t ws_bytes, lvx_stream_t stream);

/* All blocks, then x <- x + dt * stack(x).  The residual stream is widened to fp32 once, carried in fp32 through all
 * blocks, and narrowed to bf16 only by the Euler step.  mod6_per_layer: fp32 [n_layers][6][d] or NULL. */
lvx_status_t lvx_denoise_stage(const lvx_stage_t *stage /* host */, lvx_kvcache_t *cache, void *dev_x_inout, int32_t n_tokens,
                               const void *dev_ctx, int32_t n_ctx, const float *dev_mod6_per_layer, float dt,
                               int64_t chunk_index, int32_t t0, void *dev_workspace, size_t ws_bytes, lvx_stream_t stream);

/* Alg. 3, the loop over the T denoising steps of ONE block on one device: for s = 0 .. n_steps-1 (in execution order, i.e. the
 * paper's j = T .. 1) the whole stage runs with caches[s], the rolling cache of that timestep (a block attends only to history
 * of its own noise level, Sec. 3.3 "timestep-forcing"), and with that step's modulation; then x <- x + dt * stack(x) and the
 * cache's pop/append.  caches: host array of n_steps distinct handles; mod6_per_step_layer: fp32 [n_steps][n_layers][6][d] or
 * NULL.  t_sink >= 0: every step first re-assigns the sink index of its cache (lvx_sink_rope_update on all layers); t_sink < 0:
 * sinks are left as they are.  All steps are validated before anything is enqueued (STATE if any layer of any cache does not
 * expect chunk_index, or lacks a sink source when t_sink >= 0). */
lvx_status_t lvx_sample_chunk(const lvx_stage_t *stage /* host */, lvx_kvcache_t *const *caches /* host */, int32_t n_steps,
                              void *dev_x_inout, int32_t n_tokens, const void *dev_ctx, int32_t n_ctx,
                              const float *dev_mod6_per_step_layer, float dt, int64_t chunk_index, int32_t t0, int32_t t_sink,
                              void *dev_workspace, size_t ws_bytes, lvx_stream_t stream);

/* Warm-up of a sink frame (Appendix D: after the sink swap of the adaptive attention sink the stack is run once more to produce the
 * new sink's K/V): the sink frame's tokens x_sink [sink_keys][d] bf16 run through all blocks; per layer the un-rotated,
 * normalised keys and the values of these tokens are installed as the sink (as lvx_kvcache_reset_sink does) and rotated to
 * temporal index t_sink.  Reading (the paper does not say): the sink frame attends to itself only; every other step is the
 * block's.  The ring of past blocks is untouched.  dev_x_out (may be NULL) receives the stack's output for the sink tokens,
 * [sink_keys][d] bf16.  workspace: lvx_workspace_bytes(stage, sink_keys, n_ctx).  Needs attached sink source storage. */
lvx_status_t lvx_sink_prefill(const lvx_stage_t *stage /* host */, lvx_kvcache_t *cache, const void *dev_x_sink, const void *dev_ctx,
                              int32_t n_ctx, const float *dev_mod6_per_layer, int32_t t_sink, void *dev_x_out,
                              void *dev_workspace, size_t ws_bytes, lvx_stream_t stream);

/* ------------------------------------------------------------------------------------------------
 * Streaming causal convolution with a two-frame feature cache (Appendix C, "Streaming VAE Feature Caching": each causal
 * convolution of the decoder keeps its two most recent input frames and prepends them as causal context for the next frames).
 *   y[t, y, x, o] = act(bias[o] + sum_{dt,dy,dx,c} w[o][(dt*3+dy)*3+dx][c] * x[t+dt-2, y+dy-1, x+dx-1, c])
 * zeros outside the frame and before the first frame of the sequence; frames arrive in order over any number of steps and the
 * result equals the convolution of the whole sequence.  Channels last, bf16: x [n_frames][H][W][c_in], y [n_frames][H][W][c_out],
 * w [c_out][27*c_in] with row stride ldw (taps time-major, then row, then column; channels innermost), bias fp32 [c_out] or
 * NULL, act 0 = none, 1 = SiLU.  fp32 accumulation on the matrix cores.  c_in % 64 == 0, c_out % 8 == 0.
 * The state (a zero-padded volume of max_frames + 2 frames, lvx_causal_conv_state_bytes) is caller-owned device memory,
 * 256-byte aligned, alive as long as the handle; init zero-fills it (the sequence starts from a zero history), reset starts a
 * new sequence.  Steps on one handle must be stream-ordered.
 * ------------------------------------------------------------------------------------------------ */
typedef struct {
    int32_t c_in, c_out;
    int32_t height, width; /* frame size at this layer */
    int32_t max_frames;    /* most frames one step may carry */
} lvx_conv_desc_t;
typedef struct lvx_causal_conv lvx_causal_conv_t; /* opaque host-side handle */

size_t lvx_causal_conv_state_bytes(const lvx_conv_desc_t *desc /* host */);
lvx_status_t lvx_causal_conv_init(const lvx_conv_desc_t *desc /* host */, void *dev_state, size_t bytes, lvx_stream_t stream,
                                  lvx_causal_conv_t **out /* host */);
lvx_status_t lvx_causal_conv_destroy(lvx_causal_conv_t *conv);
lvx_status_t lvx_causal_conv_reset(lvx_causal_conv_t *conv, lvx_stream_t stream);
lvx_status_t lvx_causal_conv_step(lvx_causal_conv_t *conv, const void *dev_x, int32_t n_frames, const void *dev_w, int64_t ldw,
                                  const float *dev_bias, int32_t act, void *dev_y, lvx_stream_t stream);

/* ------------------------------------------------------------------------------------------------
 * Optional timing of the kernel classes inside lvx_dit_block / lvx_denoise_stage with HIP events recorded on the
 * caller's stream (the benchmark's roofline figures come from here).  Not thread-safe; level 0 = off (default),
 * 1 = the chunk-to-cache attention launches only, 2 = every class below (together they cover every launch of a stage call).  lvx_profile_read waits for the recorded
 * events (it synchronises on them), writes per-class totals into host arrays of LVX_PROF_KINDS entries and resets.
 * ------------------------------------------------------------------------------------------------ */
enum {
    LVX_PROF_ATTN_SELF = 0, LVX_PROF_GEMM_QKV = 1, LVX_PROF_GEMM_O = 2, LVX_PROF_GEMM_CROSS = 3, LVX_PROF_GEMM_FFN1 = 4,
    LVX_PROF_GEMM_FFN2 = 5, LVX_PROF_ATTN_CROSS = 6, LVX_PROF_ROPE_NORM = 7, LVX_PROF_APPEND = 8, LVX_PROF_LAYERNORM = 9,
    LVX_PROF_FP8_QUANT = 10, /* per-tensor quantisation of the linears' input activations (FP8 stages only); this time is also
                                contained in the class of the linear it precedes */
    LVX_PROF_CTX_KV = 11,      /* the context's K / V projections (a group of layers per launch), their RMSNorm and pack */
    LVX_PROF_CROSS_QNORM = 12, /* RMSNorm of the cross-attention queries */
    LVX_PROF_MISC = 13,        /* widening of the input, Euler step / narrowing, zero fills at the start of a call */
    LVX_PROF_SINK_ROPE = 14,   /* lvx_sink_rope_update */
    LVX_PROF_KINDS = 15
};
lvx_status_t lvx_profile_set(int32_t level);
lvx_status_t lvx_profile_read(double *ms_total /* host [LVX_PROF_KINDS] */, int64_t *launches /* host [LVX_PROF_KINDS] */);

#ifdef __cplusplus
}
#endif
#endif /* LVX_H */
