// DiT block and denoise stage: host-side sequencing of the kernels on one HIP stream, no synchronisation inside.
// (Paper Alg. 4, DiT-device branch: forward with the device's local rolling KV cache, cache update, Euler step;
// Sec. 3.4: throughput of the pipeline is set by this single denoise forward.)
#include "lvx_internal.h"

#include <math.h>

#include <vector>

namespace {

// ---- optional per-kernel-class timing with HIP events on the caller's stream (for the benchmark's roofline figures)
struct prof_pair_t {
    hipEvent_t a, b;
    int kind;
};
int g_prof_level = 0;
std::vector<prof_pair_t> g_prof_pool;
size_t g_prof_used = 0;

}  // namespace

lvx_prof_scope_t::lvx_prof_scope_t(int kind, hipStream_t stream) : st(stream), pair(nullptr) {
    if (g_prof_level == 0 || (g_prof_level == 1 && kind != LVX_PROF_ATTN_SELF)) return;
    if (g_prof_used == g_prof_pool.size()) {
        prof_pair_t n;
        if (hipEventCreate(&n.a) != hipSuccess) return;
        if (hipEventCreate(&n.b) != hipSuccess) {
            (void)hipEventDestroy(n.a);
            return;
        }
        g_prof_pool.push_back(n);
    }
    const size_t idx = g_prof_used++;  // the pool may grow while this scope lives: keep the index, not a pointer
    g_prof_pool[idx].kind = kind;
    (void)hipEventRecord(g_prof_pool[idx].a, st);
    pair = (void *)(idx + 1);
}

lvx_prof_scope_t::~lvx_prof_scope_t() {
    if (pair != nullptr) (void)hipEventRecord(g_prof_pool[(size_t)pair - 1].b, st);
}

namespace {
typedef lvx_prof_scope_t prof_scope_t;

// Layers whose context K / V projections, norm and pack are done together (one GEMM launch of 2 x group segments).
constexpr int CTX_GROUP = LVX_GEMM_MAX_SEGS / 2;

struct ws_layout_t {
    size_t u, big, qk32, q_sumsq, ctx_k32, ctx_kv, pack_k, pack_v, h, q8, q8_ctx, q8_misc, total;  // byte offsets
    int64_t ld_q8, ld_q8c;                            // row strides (bytes) of the FP8 activation buffers
    int cap_ctx, ctx_group;
    int64_t ld_u, ld_qkv, ld_cq, ld_ffn, ld_ckv;      // padded row strides (elements) of the bf16 workspace matrices
    int64_t ld_qk32;                                  // row stride (fp32 elements) of the un-rounded q | k columns
};

// Rows of the workspace matrices are padded by 64 elements (128 bytes): with d_model = 5120 or d_ffn = 13824 a dense row is
// a multiple of 2 KiB, which makes the GEMM's 8-rows-per-instruction loads pile up on few memory channels.
constexpr int WS_PAD = 64;

size_t round256(size_t b) { return (b + 255) / 256 * 256; }

// Layers per context-projection launch: the group size (at most CTX_GROUP) whose 128 x 256 tiles fill whole rounds of the
// chip's 256 compute units best, i.e. the fewest rounds per layer (544 context rows, d_model 5120: 5 layers = 1000 tiles = 3.9
// rounds, where 8 layers = 1600 tiles would need 7 rounds for 6.25 rounds of work).
int ctx_group_size(int n_layers, int n_ctx, size_t d) {
    const int max_g = n_layers < CTX_GROUP ? n_layers : CTX_GROUP;
    const long tiles_per_layer = (long)((n_ctx + 127) / 128) * 2 * (long)((d + 255) / 256);
    int best = 1;
    double best_cost = 1e30;
    for (int g = 1; g <= max_g; ++g) {
        const double cost = (double)((tiles_per_layer * g + 255) / 256) / g;
        if (cost < best_cost - 1e-9 || (cost < best_cost + 1e-9 && g > best)) best = g, best_cost = cost;
    }
    return best;
}

ws_layout_t ws_layout(const lvx_stage_t *s, int n_tokens, int n_ctx) {
    ws_layout_t w;
    const size_t d = (size_t)s->rope.n_heads * s->rope.head_dim;
    const size_t wide = 3 * d > (size_t)s->d_ffn ? 3 * d : (size_t)s->d_ffn;
    w.cap_ctx = (n_ctx + LVX_KEY_TILE - 1) / LVX_KEY_TILE * LVX_KEY_TILE;
    w.ld_u = (int64_t)d + WS_PAD;
    w.ld_qkv = (int64_t)3 * d + WS_PAD;
    w.ld_cq = (int64_t)d + WS_PAD;
    w.ld_ffn = (int64_t)s->d_ffn + WS_PAD;
    w.ld_ckv = (int64_t)2 * d + WS_PAD;
    w.ld_qk32 = (int64_t)d + WS_PAD / 2;
    size_t off = 0;
    w.u = off;       off += round256((size_t)n_tokens * w.ld_u * 2);
    w.big = off;     off += round256((size_t)n_tokens * (wide + WS_PAD) * 2);
    w.qk32 = off;    // fp32 k columns of the QKV projection (bf16 stages only; an FP8 stage stores them in bf16)
    if (s->blocks_fp8 == nullptr) off += round256((size_t)n_tokens * w.ld_qk32 * 4);
    w.q_sumsq = off;  // partial sums of squares of the cross-attention's query rows (bf16 stages), d / 64 per row
    if (s->blocks_fp8 == nullptr) off += round256((size_t)n_tokens * LVX_GEMM_SUMSQ_PARTS(d) * 4);
    // context K | V rows and their packed forms for a group of layers at once (bf16 stages; an FP8 stage uses one slot)
    w.ctx_group = s->blocks_fp8 != nullptr ? 1 : ctx_group_size(s->n_layers, n_ctx, d);
    w.ctx_kv = off;  off += round256((size_t)w.ctx_group * n_ctx * w.ld_ckv * 2);
    w.ctx_k32 = off;  // un-rounded context keys before their RMSNorm (bf16 stages), row stride ld_u fp32 elements
    if (s->blocks_fp8 == nullptr) off += round256((size_t)w.ctx_group * n_ctx * w.ld_u * 4);
    w.pack_k = off;  off += round256((size_t)w.ctx_group * w.cap_ctx * d * 2);
    w.pack_v = off;  off += round256((size_t)w.ctx_group * w.cap_ctx * d * 2);
    w.h = off;       off += round256((size_t)n_tokens * d * 4);  // fp32 residual stream
    w.q8 = w.q8_ctx = w.q8_misc = off;
    const size_t wide_in = d > (size_t)s->d_ffn ? d : (size_t)s->d_ffn;
    w.ld_q8 = (int64_t)wide_in + 128;
    w.ld_q8c = (int64_t)d + 128;
    if (s->blocks_fp8 != nullptr) {  // quantised input activation of the running linear, quantised context, amax scratch + scales
        w.q8 = off;       off += round256((size_t)n_tokens * w.ld_q8);
        w.q8_ctx = off;   off += round256((size_t)n_ctx * w.ld_q8c);
        w.q8_misc = off;  off += 1024;  // two amax slot arrays (2 x 256 bytes), activation and context scales
    }
    w.total = off;
    return w;
}

lvx_status_t check_stage(const lvx_stage_t *s, const lvx_kvcache *c, int n_tokens, int n_ctx, bool allow_sink_rows = false) {
    LVX_REQUIRE(s != nullptr, LVX_ERR_INVALID_ARG, "stage descriptor is NULL");
    LVX_REQUIRE(s->blocks != nullptr && s->n_layers > 0, LVX_ERR_INVALID_ARG, "stage has no blocks");
    LVX_REQUIRE(s->rope.n_heads > 0 && (s->rope.head_dim == 64 || s->rope.head_dim == 128), LVX_ERR_UNSUPPORTED,
                "head_dim %d not supported (64 or 128)", s->rope.head_dim);
    const int d = s->rope.n_heads * s->rope.head_dim;
    LVX_REQUIRE(d % 64 == 0 && s->d_ffn > 0 && s->d_ffn % 64 == 0, LVX_ERR_SHAPE, "d_model %d and d_ffn %d must be multiples of 64", d,
                s->d_ffn);
    LVX_REQUIRE(n_tokens > 0 && n_ctx > 0, LVX_ERR_SHAPE, "n_tokens %d and n_ctx %d must be positive", n_tokens, n_ctx);
    LVX_REQUIRE((s->ldw_d == 0 || (s->ldw_d >= d && s->ldw_d % 8 == 0)) && (s->ldw_ffn == 0 || (s->ldw_ffn >= s->d_ffn && s->ldw_ffn % 8 == 0)),
                LVX_ERR_SHAPE, "weight row strides must be 0 (dense) or multiples of 8 not below in_features");
    if (s->blocks_fp8 != nullptr) {
        LVX_REQUIRE(d % 128 == 0 && s->d_ffn % 128 == 0, LVX_ERR_SHAPE, "FP8 linears need d_model %d and d_ffn %d to be multiples of 128", d,
                    s->d_ffn);
        LVX_REQUIRE((s->ldw8_d == 0 || (s->ldw8_d >= d && s->ldw8_d % 16 == 0)) &&
                        (s->ldw8_ffn == 0 || (s->ldw8_ffn >= s->d_ffn && s->ldw8_ffn % 16 == 0)),
                    LVX_ERR_SHAPE, "FP8 weight row strides must be 0 (dense) or multiples of 16 not below in_features");
    }
    if (c != nullptr) {
        LVX_REQUIRE(c->desc.n_heads == s->rope.n_heads && c->desc.head_dim == s->rope.head_dim && c->desc.frame_h == s->rope.frame_h &&
                        c->desc.frame_w == s->rope.frame_w,
                    LVX_ERR_SHAPE, "stage and cache descriptors disagree on heads / head_dim / frame size");
        LVX_REQUIRE(c->desc.n_layers >= s->n_layers, LVX_ERR_SHAPE, "cache has %d layers, stage has %d", c->desc.n_layers, s->n_layers);
        LVX_REQUIRE(n_tokens == c->chunk_keys || (allow_sink_rows && n_tokens == c->sink_keys), LVX_ERR_SHAPE,
                    "n_tokens %d must equal the cache's chunk size %d", n_tokens, c->chunk_keys);
    }
    return LVX_OK;
}

// x: the fp32 residual stream [n][d].
// sink_prefill = false: the chunk's forward (its K-hat / V go to the ring slot of chunk_index, attention over the visible prefix).
// sink_prefill = true : the sink frame's forward (Appendix D, warm-up of the adaptive attention sink): the n = sink_keys rows
//   install the layer's un-rotated sink keys and its values, the sink keys are rotated to temporal index t0, and the rows
//   attend to the sink segment only; the ring is not touched.
// amax_cur (FP8 stages): which of the two amax slot arrays the next producer writes and the next quantisation reads; both arrays
//   are zero when the entry point starts (call_begin), every quantisation clears the other one.
// Context K / V of layers [l0, l1) (at most CTX_GROUP; bf16 stages): the context is the same for every layer of a forward
// (Alg. 4 hands one condition set C_i to the whole stack), so their 2 (l1 - l0) projections run as ONE GEMM launch (a single
// layer's pair is 200 tiles on 256 compute units), followed by one launch that normalises the K rows straight into the
// packed layout the attention kernel reads and one that transposes the V rows into it.  Slot j of the group holds layer l0 + j.
lvx_status_t precompute_ctx(const lvx_stage_t *s, int l0, int l1, const bf16_t *ctx, int n_ctx, char *ws, const ws_layout_t &L, hipStream_t st) {
    const int H = s->rope.n_heads, D = s->rope.head_dim, d = H * D;
    const int64_t ldw = s->ldw_d > 0 ? s->ldw_d : d, ldk = L.ld_ckv;
    bf16_t *ctx_kv = (bf16_t *)(ws + L.ctx_kv), *pack_k = (bf16_t *)(ws + L.pack_k), *pack_v = (bf16_t *)(ws + L.pack_v);
    float *ctx_k32 = (float *)(ws + L.ctx_k32);
    const int g = l1 - l0;
    const int64_t slot_rows = (int64_t)n_ctx * ldk, slot_packed = (int64_t)L.cap_ctx * d, ld32 = L.ld_u, slot_rows32 = (int64_t)n_ctx * ld32;
    lvx_gemm_segs_t segs;
    segs.n = 2 * g;
    const float *gains[CTX_GROUP];
    for (int j = 0; j < g; ++j) {
        const lvx_block_weights_t &w = s->blocks[l0 + j];
        segs.s[2 * j] = {(const bf16_t *)w.Wc_k, ctx_k32 + j * slot_rows32, ld32, d, 0, 1, 0};  // keys in fp32: rounded once, after the norm
        segs.s[2 * j + 1] = {(const bf16_t *)w.Wc_v, ctx_kv + j * slot_rows + d, ldk, d, 0, 0, 0};
        gains[j] = w.gc_k;
    }
    prof_scope_t ps(LVX_PROF_CTX_KV, st);
    LVX_TRY(lvx_launch_linear_segments(ctx, d, ldw, segs, n_ctx, d, st));
    LVX_TRY(lvx_launch_norm_to_packed_k(&s->rope, ctx_k32, 1, ld32, n_ctx, gains, pack_k, L.cap_ctx, g, slot_rows32, slot_packed, st));
    return lvx_launch_pack_kv(nullptr, ctx_kv + d, ldk, n_ctx, H, D, L.cap_ctx, 0, pack_k, pack_v, st, g, slot_rows, slot_packed);
}

// ctx_slot: slot of the context group that holds this layer's packed context K / V (bf16 stages, see precompute_ctx).
lvx_status_t run_block(const lvx_stage_t *s, int layer, lvx_kvcache *c, float *x, int n, const bf16_t *ctx, int n_ctx,
                       const float *mod6, int64_t chunk_index, int t0, char *ws, const ws_layout_t &L, hipStream_t st, int *amax_cur,
                       int ctx_slot, bool sink_prefill = false, bool ctx_codes_ready = false) {
    const lvx_block_weights_t &w = s->blocks[layer];
    const int H = s->rope.n_heads, D = s->rope.head_dim, d = H * D, f = s->d_ffn;
    const float eps = s->rope.eps;
    const float scale = 1.0f / sqrtf((float)D);
    bf16_t *u = (bf16_t *)(ws + L.u);
    bf16_t *big = (bf16_t *)(ws + L.big);
    bf16_t *ctx_kv = (bf16_t *)(ws + L.ctx_kv);
    bf16_t *pack_k = (bf16_t *)(ws + L.pack_k) + (size_t)ctx_slot * L.cap_ctx * (s->rope.n_heads * s->rope.head_dim);
    bf16_t *pack_v = (bf16_t *)(ws + L.pack_v) + (size_t)ctx_slot * L.cap_ctx * (s->rope.n_heads * s->rope.head_dim);
    const float *shift1 = mod6 ? mod6 : nullptr, *scale1 = mod6 ? mod6 + d : nullptr, *gate1 = mod6 ? mod6 + 2 * d : nullptr;
    const float *shift2 = mod6 ? mod6 + 3 * d : nullptr, *scale2 = mod6 ? mod6 + 4 * d : nullptr, *gate2 = mod6 ? mod6 + 5 * d : nullptr;

    const int64_t ldw = s->ldw_d > 0 ? s->ldw_d : d, ldw2 = s->ldw_ffn > 0 ? s->ldw_ffn : f;
    const int64_t ldu = L.ld_u, ldq = L.ld_qkv, ldc = L.ld_cq, ldf = L.ld_ffn, ldk = L.ld_ckv;

    // One linear of the block: bf16, or (Appendix C) FP8 with the input activation quantised per tensor right before it.
    // which: index into the FP8 weight pointers / scales (0 W_qkv .. 7 W_2); reuse_ctx: the context was already quantised.
    const lvx_block_weights_fp8_t *w8 = s->blocks_fp8 ? &s->blocks_fp8[layer] : nullptr;
    const int64_t ldw8 = s->ldw8_d > 0 ? s->ldw8_d : d, ldw8_2 = s->ldw8_ffn > 0 ? s->ldw8_ffn : f;
    uint32_t *slots = (uint32_t *)(ws + L.q8_misc);
    float *scale_act = (float *)(ws + L.q8_misc + 512), *scale_ctx = (float *)(ws + L.q8_misc + 528);
    // where the kernel that produces the next linear's input leaves that tensor's amax (NULL in a bf16 stage)
    auto amax_out = [&]() -> uint32_t * { return w8 ? slots + LVX_AMAX_SLOTS * (*amax_cur) : nullptr; };
    // amax_ready: the producer of A already left A's amax in the current slot array (else a separate pass collects it);
    // feeds_fp8: this linear's own output is the next linear's input, its epilogue collects that amax
    auto linear = [&](const bf16_t *A, int64_t lda, const void *Wbf, int which, void *C, int64_t ldc_, int M, int N, int K, lvx_epilogue_t epi,
                      const void *R, int64_t ldr, const float *gate, bool is_ctx, bool reuse_ctx, bool amax_ready,
                      bool feeds_fp8) -> lvx_status_t {
        if (w8 == nullptr) return lvx_linear(A, lda, Wbf, K == f ? ldw2 : ldw, C, ldc_, M, N, K, epi, R, ldr, gate, st);
        const void *const w8p[8] = {w8->W_qkv, w8->W_o, w8->Wc_q, w8->Wc_k, w8->Wc_v, w8->Wc_o, w8->W_1, w8->W_2};
        uint8_t *aq = (uint8_t *)(ws + (is_ctx ? L.q8_ctx : L.q8));
        const int64_t ldaq = is_ctx ? L.ld_q8c : L.ld_q8;
        float *sa = is_ctx ? scale_ctx : scale_act;
        if (!reuse_ctx) {
            prof_scope_t ps(LVX_PROF_FP8_QUANT, st);
            uint32_t *cur = slots + LVX_AMAX_SLOTS * (*amax_cur), *other = slots + LVX_AMAX_SLOTS * (1 - *amax_cur);
            if (!amax_ready) LVX_TRY(lvx_launch_fp8_amax(A, lda, M, K, cur, st));
            LVX_TRY(lvx_launch_fp8_quant(A, lda, M, K, aq, ldaq, cur, other, sa, st));
            *amax_cur ^= 1;
        }
        return lvx_launch_linear_fp8(aq, ldaq, sa, w8p[which], K == f ? ldw8_2 : ldw8, w8->scales + which, C, ldc_, M, N, K, epi, R, ldr, gate,
                                     feeds_fp8 ? amax_out() : nullptr, st);
    };

    // self-attention branch.  bf16 stage: the k columns of the QKV projection leave the GEMM in fp32 and are rounded to bf16
    // once, by the RMSNorm + RoPE kernel, after the rotation (the cached K-hat then carries two bf16 roundings, u and itself,
    // instead of three); the q and v columns are stored in bf16 (the queries' extra rounding changes the block's output by
    // 2e-5 of its RMS, and fp32 columns cost the GEMM's epilogue and the RoPE kernel their bytes).  FP8 stage: all three in bf16.
    float *k32 = (float *)(ws + L.qk32);
    const int64_t ld32 = L.ld_qk32;
    { prof_scope_t ps(LVX_PROF_LAYERNORM, st); LVX_TRY(lvx_launch_layernorm(x, 1, d, shift1, scale1, eps, n, d, u, ldu, st, amax_out())); }
    {
        prof_scope_t ps(LVX_PROF_GEMM_QKV, st);
        if (w8 == nullptr) {
            const bf16_t *Wq = (const bf16_t *)w.W_qkv;
            lvx_gemm_segs_t segs;
            segs.n = 3;
            segs.s[0] = {Wq, big, ldq, d, 0, 0, 0};
            segs.s[1] = {Wq + (size_t)d * ldw, k32, ld32, d, 0, 1, 0};
            segs.s[2] = {Wq + (size_t)2 * d * ldw, big + 2 * d, ldq, d, 0, 0, 0};
            LVX_TRY(lvx_launch_linear_segments(u, ldu, ldw, segs, n, d, st));
        } else
            LVX_TRY(linear(u, ldu, w.W_qkv, 0, big, ldq, n, 3 * d, d, LVX_EPI_STORE, nullptr, 0, nullptr, false, false, true, false));
    }
    if (!sink_prefill) {
        {
            // the RoPE kernel writes the chunk's keys straight into their ring slot of the cache (one write instead of a write, a
            // read and a write); the append then only has the values left to transpose.  bf16 stage: k comes un-rounded (fp32).
            lvx_slot_info_t slot;
            LVX_TRY(lvx_cache_append_begin(c, layer, chunk_index, &slot));
            bf16_t *k_slot = const_cast<bf16_t *>(lvx_cache_k(c, layer)) + (size_t)slot.key_offset * D;
            {
                prof_scope_t ps(LVX_PROF_ROPE_NORM, st);
                if (w8 == nullptr)
                    LVX_TRY(lvx_launch_rope_qk(&s->rope, big, ldq, k32, 1, ld32, w.g_q, w.g_k, n, t0, big, ldq, k_slot, D, (int64_t)c->cap_keys * D,
                                               scale * LVX_LOG2E, st));
                else
                    LVX_TRY(lvx_launch_rope_qk(&s->rope, big, ldq, big + d, 0, ldq, w.g_q, w.g_k, n, t0, big, ldq, k_slot, D,
                                               (int64_t)c->cap_keys * D, scale * LVX_LOG2E, st));
            }
            {
                prof_scope_t ps(LVX_PROF_APPEND, st);
                LVX_TRY(lvx_launch_pack_kv(nullptr, big + 2 * d, ldq, n, H, D, c->cap_keys, slot.key_offset, const_cast<bf16_t *>(lvx_cache_k(c, layer)),
                                           const_cast<bf16_t *>(lvx_cache_vt(c, layer)), st));
            }
            lvx_cache_append_commit(c, layer, chunk_index, &slot);
        }
        {
            prof_scope_t ps(LVX_PROF_ATTN_SELF, st);
            // the queries were written pre-scaled by the RoPE kernel above
            LVX_TRY(lvx_launch_attention(big, ldq, n, H, D, lvx_cache_k(c, layer), lvx_cache_vt(c, layer), c->cap_keys, c->state[layer].key_count,
                                         scale, u, ldu, st, amax_out(), true));
        }
    } else {
        // the sink's un-rotated keys go into the cache's fp32 source storage: un-rounded from the projection in a bf16 stage,
        // widened from the bf16 projection in an FP8 stage
        float *src32 = c->sink_src + (size_t)layer * c->sink_keys * d;
        if (w8 == nullptr) {
            LVX_TRY(lvx_rope3d(&s->rope, big, nullptr, ldq, w.g_q, nullptr, n, t0, big, nullptr, ldq, st));  // q: norm + RoPE
            LVX_TRY(lvx_launch_rmsnorm_f32(&s->rope, k32, ld32, w.g_k, n, src32, d, st));                    // k: norm only
        } else {
            lvx_rope_desc_t k_norm_only = s->rope;
            k_norm_only.apply_rope = 0;
            LVX_TRY(lvx_rope3d(&s->rope, big, nullptr, ldq, w.g_q, nullptr, n, t0, big, nullptr, ldq, st));
            if (w.g_k) LVX_TRY(lvx_rope3d(&k_norm_only, nullptr, big + d, ldq, nullptr, w.g_k, n, 0, nullptr, big + d, ldq, st));
            LVX_TRY(lvx_launch_widen_rows(big + d, ldq, src32, d, n, d, st));
        }
        LVX_TRY(lvx_sink_install_values(c, layer, big + 2 * d, ldq, st));
        LVX_TRY(lvx_sink_rope_update(c, &s->rope, layer, t0, st));
        LVX_TRY(lvx_launch_attention(big, ldq, n, H, D, lvx_cache_k(c, layer), lvx_cache_vt(c, layer), c->cap_keys, c->sink_keys, scale, u,
                                     ldu, st, amax_out()));
    }
    { prof_scope_t ps(LVX_PROF_GEMM_O, st); LVX_TRY(linear(u, ldu, w.W_o, 1, x, d, n, d, d, LVX_EPI_RESID_GATE_F32, x, d, gate1, false, false, true, false)); }

    // cross-attention to the audio + text context
    { prof_scope_t ps(LVX_PROF_LAYERNORM, st); LVX_TRY(lvx_launch_layernorm(x, 1, d, nullptr, nullptr, eps, n, d, u, ldu, st, amax_out())); }
    // bf16 stage with a query gain: the projection leaves each row's partial sums of squares beside its bf16 output and the
    // attention kernel normalises, scales and rounds the queries as it loads them (no norm-only pass over q)
    const bool fuse_qnorm = w8 == nullptr && w.gc_q != nullptr && D == 128 && d % 512 == 0 && d <= 8192;
    float *q_sumsq = (float *)(ws + L.q_sumsq);
    const int q_parts = LVX_GEMM_SUMSQ_PARTS(d);
    {
        prof_scope_t ps(LVX_PROF_GEMM_CROSS, st);
        if (fuse_qnorm) {
            lvx_gemm_segs_t segs;
            segs.n = 1;
            segs.s[0] = {(const bf16_t *)w.Wc_q, big, ldc, d, 0, 0, q_parts, q_sumsq};
            LVX_TRY(lvx_launch_linear_segments(u, ldu, ldw, segs, n, d, st));
        } else
            LVX_TRY(linear(u, ldu, w.Wc_q, 2, big, ldc, n, d, d, LVX_EPI_STORE, nullptr, 0, nullptr, false, false, true, false));
    }
    lvx_rope_desc_t norm_only = s->rope;
    norm_only.apply_rope = 0;
    if (w.gc_q && !fuse_qnorm) { prof_scope_t ps(LVX_PROF_CROSS_QNORM, st); LVX_TRY(lvx_rope3d(&norm_only, big, nullptr, ldc, w.gc_q, nullptr, n, 0, big, nullptr, ldc, st)); }
    if (w8 != nullptr) {  // FP8 stage: this layer's context projections, norm and pack, into slot 0 (the context is quantised once)
        prof_scope_t ps(LVX_PROF_CTX_KV, st);
        // (the context is the same for every layer of a call: its codes and scale are formed by the first layer and reused)
        LVX_TRY(linear(ctx, d, w.Wc_k, 3, ctx_kv, ldk, n_ctx, d, d, LVX_EPI_STORE, nullptr, 0, nullptr, true, ctx_codes_ready, false, false));
        LVX_TRY(linear(ctx, d, w.Wc_v, 4, ctx_kv + d, ldk, n_ctx, d, d, LVX_EPI_STORE, nullptr, 0, nullptr, true, true, false, false));
        const float *gains[1] = {w.gc_k};
        LVX_TRY(lvx_launch_norm_to_packed_k(&s->rope, ctx_kv, 0, ldk, n_ctx, gains, pack_k, L.cap_ctx, 1, 0, 0, st));
        LVX_TRY(lvx_launch_pack_kv(nullptr, ctx_kv + d, ldk, n_ctx, H, D, L.cap_ctx, 0, pack_k, pack_v, st));
    }
    {
        prof_scope_t ps(LVX_PROF_ATTN_CROSS, st);
        const lvx_attn_qnorm_t qn = {q_sumsq, w.gc_q, q_parts, q_parts, d, s->rope.eps};
        LVX_TRY(lvx_launch_attention(big, ldc, n, H, D, pack_k, pack_v, L.cap_ctx, n_ctx, scale, u, ldu, st, amax_out(), false, fuse_qnorm ? &qn : nullptr));
    }
    { prof_scope_t ps(LVX_PROF_GEMM_CROSS, st); LVX_TRY(linear(u, ldu, w.Wc_o, 5, x, d, n, d, d, LVX_EPI_RESID_GATE_F32, x, d, nullptr, false, false, true, false)); }

    // feed-forward
    { prof_scope_t ps(LVX_PROF_LAYERNORM, st); LVX_TRY(lvx_launch_layernorm(x, 1, d, shift2, scale2, eps, n, d, u, ldu, st, amax_out())); }
    { prof_scope_t ps(LVX_PROF_GEMM_FFN1, st); LVX_TRY(linear(u, ldu, w.W_1, 6, big, ldf, n, f, d, LVX_EPI_GELU_TANH, nullptr, 0, nullptr, false, false, true, true)); }
    { prof_scope_t ps(LVX_PROF_GEMM_FFN2, st); LVX_TRY(linear(big, ldf, w.W_2, 7, x, d, n, d, f, LVX_EPI_RESID_GATE_F32, x, d, gate2, false, false, true, false)); }
    return LVX_OK;
}

// Once per entry-point call: the packed context K / V^T buffers are cleared when the context does not fill its last 64-key
// tile (the keys past n_ctx are masked in the attention but must be finite; the per-layer pack only writes keys below n_ctx),
// and an FP8 stage clears both amax slot arrays.
lvx_status_t call_begin(const lvx_stage_t *s, char *ws, const ws_layout_t &L, hipStream_t st, int n_ctx) {
    prof_scope_t ps(LVX_PROF_MISC, st);
    if (L.cap_ctx != n_ctx) LVX_TRY(lvx_launch_fill_zero(ws + L.pack_k, L.h - L.pack_k, st));
    if (s->blocks_fp8 == nullptr) return LVX_OK;
    return lvx_launch_fill_zero(ws + L.q8_misc, 2 * LVX_AMAX_SLOTS * sizeof(uint32_t), st);
}

// Blocks l0 .. l1-1 on the fp32 stream h.  mod6: modulation of layer l0 (NULL = none), the following layers' mod6_stride
// floats apart.  In a bf16 stage the context K / V of up to CTX_GROUP layers are prepared together, ahead of the first of them.
lvx_status_t run_layers(const lvx_stage_t *s, int l0, int l1, lvx_kvcache *c, float *h, int n, const bf16_t *ctx, int n_ctx, const float *mod6,
                        size_t mod6_stride, int64_t chunk_index, int t0, char *ws, const ws_layout_t &L, hipStream_t st, int *amax_cur,
                        bool sink_prefill) {
    for (int l = l0; l < l1; ++l) {
        int slot = 0;
        if (s->blocks_fp8 == nullptr) {
            slot = (l - l0) % L.ctx_group;
            if (slot == 0) LVX_TRY(precompute_ctx(s, l, l + L.ctx_group < l1 ? l + L.ctx_group : l1, ctx, n_ctx, ws, L, st));
        }
        const float *m6 = mod6 ? mod6 + (size_t)(l - l0) * mod6_stride : nullptr;
        LVX_TRY(run_block(s, l, c, h, n, ctx, n_ctx, m6, chunk_index, t0, ws, L, st, amax_cur, slot, sink_prefill, l > l0));
    }
    return LVX_OK;
}

lvx_status_t widen_in(const bf16_t *x, float *h, size_t n_elems, hipStream_t st) {
    prof_scope_t ps(LVX_PROF_MISC, st);
    return lvx_launch_widen(x, h, n_elems, st);
}

lvx_status_t euler_out(const bf16_t *x, const float *h, float dt, bf16_t *out, size_t n_elems, hipStream_t st) {
    prof_scope_t ps(LVX_PROF_MISC, st);
    return lvx_launch_euler(x, h, dt, out, n_elems, st);
}

lvx_status_t check_common(const lvx_stage_t *s, lvx_kvcache *c, void *x, int n, const void *ctx, int n_ctx, void *ws, size_t ws_bytes,
                          int64_t chunk_index, int t0) {
    LVX_REQUIRE(c != nullptr, LVX_ERR_INVALID_ARG, "cache handle is NULL");
    LVX_TRY(check_stage(s, c, n, n_ctx));
    LVX_REQUIRE(x != nullptr && ctx != nullptr && ws != nullptr, LVX_ERR_INVALID_ARG, "x, ctx or workspace is NULL");
    LVX_REQUIRE(lvx_aligned16(x) && lvx_aligned16(ctx) && (((uintptr_t)ws) & 255u) == 0, LVX_ERR_INVALID_ARG,
                "x / ctx must be 16-byte and workspace 256-byte aligned");
    const size_t need = lvx_workspace_bytes(s, n, n_ctx);
    LVX_REQUIRE(ws_bytes >= need, LVX_ERR_SHAPE, "workspace too small: %zu bytes given, %zu needed", ws_bytes, need);
    LVX_REQUIRE(chunk_index >= 0 && t0 >= 0, LVX_ERR_INVALID_ARG, "chunk_index and t0 must be non-negative");
    return LVX_OK;
}

// Everything the forward of chunk `chunk_index` will ask of layers [l0, l1) of the cache, checked before the first launch so
// that a refused call leaves the ring bookkeeping of every layer as it was: the layer expects this chunk, has its sink, and
// the sink keys are rotated (not left stale by lvx_kvcache_reset_sink).
lvx_status_t check_layers_ready(const lvx_kvcache *c, int l0, int l1, int64_t chunk_index) {
    for (int l = l0; l < l1; ++l) {
        LVX_REQUIRE(c->state[l].last_chunk + 1 == chunk_index, LVX_ERR_STATE, "layer %d expects chunk %lld, got %lld", l,
                    (long long)(c->state[l].last_chunk + 1), (long long)chunk_index);
        LVX_REQUIRE(c->sink_keys == 0 || c->state[l].sink_set, LVX_ERR_STATE, "layer %d: sink not set before the first append", l);
        LVX_REQUIRE(c->sink_t[l] != LVX_SINK_STALE, LVX_ERR_STATE,
                    "layer %d: the sink was reset and its keys are not rotated yet (lvx_sink_rope_update)", l);
    }
    return LVX_OK;
}

}  // namespace

extern "C" lvx_status_t lvx_profile_set(int32_t level) {
    LVX_REQUIRE(level >= 0 && level <= 2, LVX_ERR_INVALID_ARG, "profile level %d not in 0..2", level);
    g_prof_level = level;
    return LVX_OK;
}

extern "C" lvx_status_t lvx_profile_read(double *ms_total, int64_t *launches) {
    LVX_REQUIRE(ms_total != nullptr && launches != nullptr, LVX_ERR_INVALID_ARG, "output arrays are NULL");
    for (int k = 0; k < LVX_PROF_KINDS; ++k) {
        ms_total[k] = 0.0;
        launches[k] = 0;
    }
    for (size_t i = 0; i < g_prof_used; ++i) {
        prof_pair_t &p = g_prof_pool[i];
        LVX_CHECK_HIP(hipEventSynchronize(p.b));
        float ms = 0.f;
        LVX_CHECK_HIP(hipEventElapsedTime(&ms, p.a, p.b));
        ms_total[p.kind] += ms;
        launches[p.kind] += 1;
    }
    g_prof_used = 0;
    return LVX_OK;
}

extern "C" size_t lvx_workspace_bytes(const lvx_stage_t *stage, int32_t n_tokens, int32_t n_ctx) {
    if (check_stage(stage, nullptr, n_tokens, n_ctx) != LVX_OK) return 0;
    return ws_layout(stage, n_tokens, n_ctx).total;
}

extern "C" lvx_status_t lvx_context_kv(const lvx_stage_t *stage, int32_t layer0, int32_t n_layers, const void *dev_ctx, int32_t n_ctx,
                                       void *dev_k_out, void *dev_v_out, int64_t ld, void *dev_workspace, size_t ws_bytes, lvx_stream_t stream) {
    LVX_TRY(check_stage(stage, nullptr, 1, n_ctx));
    LVX_REQUIRE(stage->blocks_fp8 == nullptr, LVX_ERR_UNSUPPORTED, "lvx_context_kv serves bf16 stages (an FP8 stage projects the context layer by layer)");
    LVX_REQUIRE(layer0 >= 0 && n_layers >= 1 && layer0 + n_layers <= stage->n_layers, LVX_ERR_INVALID_ARG, "layers [%d,%d) outside the stage's %d",
                layer0, layer0 + n_layers, stage->n_layers);
    LVX_REQUIRE(dev_ctx != nullptr && dev_k_out != nullptr && dev_v_out != nullptr && dev_workspace != nullptr, LVX_ERR_INVALID_ARG,
                "ctx, an output or the workspace is NULL");
    LVX_REQUIRE(lvx_aligned16(dev_ctx) && lvx_aligned16(dev_k_out) && lvx_aligned16(dev_v_out) && (((uintptr_t)dev_workspace) & 255u) == 0,
                LVX_ERR_INVALID_ARG, "ctx / outputs must be 16-byte and workspace 256-byte aligned");
    const int H = stage->rope.n_heads, D = stage->rope.head_dim, d = H * D;
    LVX_REQUIRE(ld >= d && ld % 8 == 0, LVX_ERR_SHAPE, "row stride %lld must be a multiple of 8 and >= d_model", (long long)ld);
    const ws_layout_t L = ws_layout(stage, 1, n_ctx);
    LVX_REQUIRE(n_layers <= L.ctx_group, LVX_ERR_SHAPE, "at most %d layers per call", L.ctx_group);
    LVX_REQUIRE(ws_bytes >= L.total, LVX_ERR_SHAPE, "workspace too small: %zu bytes given, %zu needed (lvx_workspace_bytes(stage, 1, n_ctx))", ws_bytes,
                L.total);
    char *ws = (char *)dev_workspace;
    hipStream_t st = (hipStream_t)stream;
    LVX_TRY(call_begin(stage, ws, L, st, n_ctx));
    LVX_TRY(precompute_ctx(stage, layer0, layer0 + n_layers, (const bf16_t *)dev_ctx, n_ctx, ws, L, st));
    for (int j = 0; j < n_layers; ++j)
        LVX_TRY(lvx_launch_gather_kv((const bf16_t *)(ws + L.pack_k) + (size_t)j * L.cap_ctx * d, (const bf16_t *)(ws + L.pack_v) + (size_t)j * L.cap_ctx * d,
                                     L.cap_ctx, H, D, 0, n_ctx, (bf16_t *)dev_k_out + (size_t)j * n_ctx * ld, (bf16_t *)dev_v_out + (size_t)j * n_ctx * ld, ld,
                                     st));
    return LVX_OK;
}

extern "C" lvx_status_t lvx_dit_block(const lvx_stage_t *stage, int32_t layer, lvx_kvcache_t *cache, void *dev_x_inout, int32_t n_tokens,
                                      const void *dev_ctx, int32_t n_ctx, const float *dev_mod6, int64_t chunk_index, int32_t t0,
                                      void *dev_workspace, size_t ws_bytes, lvx_stream_t stream) {
    LVX_TRY(check_common(stage, cache, dev_x_inout, n_tokens, dev_ctx, n_ctx, dev_workspace, ws_bytes, chunk_index, t0));
    LVX_REQUIRE(layer >= 0 && layer < stage->n_layers, LVX_ERR_INVALID_ARG, "layer %d out of range [0,%d)", layer, stage->n_layers);
    LVX_TRY(check_layers_ready(cache, layer, layer + 1, chunk_index));
    const ws_layout_t L = ws_layout(stage, n_tokens, n_ctx);
    const size_t n_elems = (size_t)n_tokens * stage->rope.n_heads * stage->rope.head_dim;
    float *h = (float *)((char *)dev_workspace + L.h);
    LVX_TRY(widen_in((const bf16_t *)dev_x_inout, h, n_elems, (hipStream_t)stream));
    int amax_cur = 0;
    LVX_TRY(call_begin(stage, (char *)dev_workspace, L, (hipStream_t)stream, n_ctx));
    LVX_TRY(run_layers(stage, layer, layer + 1, cache, h, n_tokens, (const bf16_t *)dev_ctx, n_ctx, dev_mod6, 0, chunk_index, t0,
                       (char *)dev_workspace, L, (hipStream_t)stream, &amax_cur, false));
    return euler_out(nullptr, h, 1.0f, (bf16_t *)dev_x_inout, n_elems, (hipStream_t)stream);
}

extern "C" lvx_status_t lvx_dit_block_f32(const lvx_stage_t *stage, int32_t layer, lvx_kvcache_t *cache, float *dev_x_inout, int32_t n_tokens,
                                          const void *dev_ctx, int32_t n_ctx, const float *dev_mod6, int64_t chunk_index, int32_t t0,
                                          void *dev_workspace, size_t ws_bytes, lvx_stream_t stream) {
    LVX_TRY(check_common(stage, cache, dev_x_inout, n_tokens, dev_ctx, n_ctx, dev_workspace, ws_bytes, chunk_index, t0));
    LVX_REQUIRE(layer >= 0 && layer < stage->n_layers, LVX_ERR_INVALID_ARG, "layer %d out of range [0,%d)", layer, stage->n_layers);
    LVX_TRY(check_layers_ready(cache, layer, layer + 1, chunk_index));
    const ws_layout_t L = ws_layout(stage, n_tokens, n_ctx);
    int amax_cur = 0;
    LVX_TRY(call_begin(stage, (char *)dev_workspace, L, (hipStream_t)stream, n_ctx));
    return run_layers(stage, layer, layer + 1, cache, dev_x_inout, n_tokens, (const bf16_t *)dev_ctx, n_ctx, dev_mod6, 0, chunk_index, t0,
                      (char *)dev_workspace, L, (hipStream_t)stream, &amax_cur, false);
}

extern "C" lvx_status_t lvx_denoise_stage(const lvx_stage_t *stage, lvx_kvcache_t *cache, void *dev_x_inout, int32_t n_tokens,
                                          const void *dev_ctx, int32_t n_ctx, const float *dev_mod6_per_layer, float dt,
                                          int64_t chunk_index, int32_t t0, void *dev_workspace, size_t ws_bytes, lvx_stream_t stream) {
    LVX_TRY(check_common(stage, cache, dev_x_inout, n_tokens, dev_ctx, n_ctx, dev_workspace, ws_bytes, chunk_index, t0));
    LVX_TRY(check_layers_ready(cache, 0, stage->n_layers, chunk_index));
    const ws_layout_t L = ws_layout(stage, n_tokens, n_ctx);
    const int d = stage->rope.n_heads * stage->rope.head_dim;
    bf16_t *x = (bf16_t *)dev_x_inout;
    float *h = (float *)((char *)dev_workspace + L.h);
    const size_t n_elems = (size_t)n_tokens * d;
    LVX_TRY(widen_in(x, h, n_elems, (hipStream_t)stream));
    int amax_cur = 0;
    LVX_TRY(call_begin(stage, (char *)dev_workspace, L, (hipStream_t)stream, n_ctx));
    LVX_TRY(run_layers(stage, 0, stage->n_layers, cache, h, n_tokens, (const bf16_t *)dev_ctx, n_ctx, dev_mod6_per_layer, (size_t)6 * d, chunk_index,
                       t0, (char *)dev_workspace, L, (hipStream_t)stream, &amax_cur, false));
    // Euler step of Alg. 3 / Alg. 4:  x <- x + v dt, the stack output standing in for the velocity
    return euler_out(x, h, dt, x, n_elems, (hipStream_t)stream);
}

// Warm-up of a (new) sink frame, Appendix D: after the first block the model's own output replaces the reference image as
// the sink and the stack is run once more to produce its K/V.  The sink's tokens go through every block attending to themselves.
extern "C" lvx_status_t lvx_sink_prefill(const lvx_stage_t *stage, lvx_kvcache_t *cache, const void *dev_x_sink, const void *dev_ctx,
                                         int32_t n_ctx, const float *dev_mod6_per_layer, int32_t t_sink, void *dev_x_out,
                                         void *dev_workspace, size_t ws_bytes, lvx_stream_t stream) {
    LVX_REQUIRE(cache != nullptr, LVX_ERR_INVALID_ARG, "cache handle is NULL");
    const int n = cache->sink_keys;
    LVX_REQUIRE(n > 0, LVX_ERR_STATE, "this cache has no sink segment (sink_frames = 0)");
    LVX_TRY(check_stage(stage, cache, n, n_ctx, true));
    LVX_REQUIRE(cache->sink_src != nullptr, LVX_ERR_STATE, "no sink source storage attached (lvx_kvcache_attach_sink_source)");
    LVX_REQUIRE(dev_x_sink != nullptr && dev_ctx != nullptr && dev_workspace != nullptr, LVX_ERR_INVALID_ARG, "x_sink, ctx or workspace is NULL");
    LVX_REQUIRE(lvx_aligned16(dev_x_sink) && lvx_aligned16(dev_ctx) && (((uintptr_t)dev_workspace) & 255u) == 0, LVX_ERR_INVALID_ARG,
                "x_sink / ctx must be 16-byte and workspace 256-byte aligned");
    LVX_REQUIRE(t_sink >= 0, LVX_ERR_INVALID_ARG, "t_sink must be non-negative");
    LVX_REQUIRE(lvx_aligned16(dev_x_out), LVX_ERR_INVALID_ARG, "x_out must be 16-byte aligned");
    const size_t need = lvx_workspace_bytes(stage, n, n_ctx);
    LVX_REQUIRE(ws_bytes >= need, LVX_ERR_SHAPE, "workspace too small: %zu bytes given, %zu needed", ws_bytes, need);
    const ws_layout_t L = ws_layout(stage, n, n_ctx);
    const int d = stage->rope.n_heads * stage->rope.head_dim;
    float *h = (float *)((char *)dev_workspace + L.h);
    LVX_TRY(widen_in((const bf16_t *)dev_x_sink, h, (size_t)n * d, (hipStream_t)stream));
    int amax_cur = 0;
    LVX_TRY(call_begin(stage, (char *)dev_workspace, L, (hipStream_t)stream, n_ctx));
    LVX_TRY(run_layers(stage, 0, stage->n_layers, cache, h, n, (const bf16_t *)dev_ctx, n_ctx, dev_mod6_per_layer, (size_t)6 * d, 0, t_sink,
                       (char *)dev_workspace, L, (hipStream_t)stream, &amax_cur, true));
    if (dev_x_out != nullptr) return euler_out(nullptr, h, 1.0f, (bf16_t *)dev_x_out, (size_t)n * d, (hipStream_t)stream);
    return LVX_OK;
}

// Alg. 3, inner loop over the denoising steps of one block on one device: step s runs the whole stage with the s-th
// timestep's own rolling cache (timestep forcing, Sec. 3.3: a block and the cache it attends to share the noise level) and the
// s-th modulation, then the Euler update; the weights are shared.
extern "C" lvx_status_t lvx_sample_chunk(const lvx_stage_t *stage, lvx_kvcache_t *const *caches, int32_t n_steps, void *dev_x_inout,
                                         int32_t n_tokens, const void *dev_ctx, int32_t n_ctx, const float *dev_mod6_per_step_layer,
                                         float dt, int64_t chunk_index, int32_t t0, int32_t t_sink, void *dev_workspace,
                                         size_t ws_bytes, lvx_stream_t stream) {
    LVX_REQUIRE(caches != nullptr && n_steps > 0, LVX_ERR_INVALID_ARG, "caches is NULL or n_steps %d is not positive", n_steps);
    LVX_REQUIRE(stage != nullptr, LVX_ERR_INVALID_ARG, "stage descriptor is NULL");
    // validate every step before enqueueing anything, so a refused call leaves all caches as they were
    for (int s = 0; s < n_steps; ++s) {
        LVX_TRY(check_common(stage, caches[s], dev_x_inout, n_tokens, dev_ctx, n_ctx, dev_workspace, ws_bytes, chunk_index, t0));
        for (int q = 0; q < s; ++q) LVX_REQUIRE(caches[q] != caches[s], LVX_ERR_INVALID_ARG, "steps %d and %d share a cache", q, s);
        for (int l = 0; l < stage->n_layers; ++l) {
            LVX_REQUIRE(caches[s]->state[l].last_chunk + 1 == chunk_index, LVX_ERR_STATE, "step %d layer %d expects chunk %lld, got %lld", s, l,
                        (long long)(caches[s]->state[l].last_chunk + 1), (long long)chunk_index);
            if (t_sink >= 0)
                LVX_REQUIRE(caches[s]->sink_src != nullptr && caches[s]->sink_t[l] != LVX_SINK_STATIC, LVX_ERR_STATE,
                            "step %d layer %d has no sink source to re-index", s, l);
            else
                LVX_REQUIRE(caches[s]->sink_t[l] != LVX_SINK_STALE, LVX_ERR_STATE, "step %d layer %d: sink keys not rotated", s, l);
        }
    }
    const size_t per_step = (size_t)stage->n_layers * 6 * stage->rope.n_heads * stage->rope.head_dim;
    for (int s = 0; s < n_steps; ++s) {
        if (t_sink >= 0) LVX_TRY(lvx_sink_rope_update(caches[s], &stage->rope, -1, t_sink, stream));
        const float *m6 = dev_mod6_per_step_layer ? dev_mod6_per_step_layer + (size_t)s * per_step : nullptr;
        LVX_TRY(lvx_denoise_stage(stage, caches[s], dev_x_inout, n_tokens, dev_ctx, n_ctx, m6, dt, chunk_index, t0, dev_workspace, ws_bytes,
                                  stream));
    }
    return LVX_OK;
}
