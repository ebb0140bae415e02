// Host logic of the C-ABI boundary under AddressSanitizer + UndefinedBehaviorSanitizer: descriptor checks, the ring arithmetic
// against a brute-force ring, size functions, and the argument checks of every entry point that can be refused before anything
// touches a device.  Built from the library's sources with host-only sanitizers (no device code) and run on the CPU by
// tests/test_host_sanitizers.py; no kernel is launched.  Exit status 0 = every expectation held.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "lvx.h"

static int failures = 0;
#define EXPECT(cond)                                                       \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond);  \
            ++failures;                                                    \
        }                                                                  \
    } while (0)

int main() {
    lvx_cache_desc_t d = {40, 40, 128, 30, 52, 3, 4, 1};
    EXPECT(lvx_kvcache_bytes(&d) == (size_t)2 * 2 * 40 * 40 * 24960 * 128);
    EXPECT(lvx_kvcache_bytes(nullptr) == 0);
    lvx_cache_desc_t bad = d;
    bad.head_dim = 96;
    EXPECT(lvx_kvcache_bytes(&bad) == 0);
    bad = d;
    bad.window_chunks = LVX_MAX_SLOTS;  // window + 1 slots would not fit the state
    EXPECT(lvx_kvcache_bytes(&bad) == 0);

    // ring arithmetic against a brute-force ring of slots, 300 steps, windows 1..6
    for (int w = 1; w <= 6; ++w) {
        lvx_cache_desc_t r = d;
        r.window_chunks = w;
        std::vector<int64_t> slots(w + 1, -1);
        for (int64_t i = 0; i < 300; ++i) {
            lvx_slot_info_t info;
            std::memset(&info, 0xff, sizeof info);
            EXPECT(lvx_ring_slot(&r, i, &info) == LVX_OK);
            const int s = (int)(i % (w + 1));
            EXPECT(info.slot == s);
            EXPECT(info.evicted_chunk == slots[s]);
            slots[s] = i;
            int valid = 0;
            for (int64_t c : slots) valid += c >= 0;
            EXPECT(info.n_valid_chunks == valid);
            EXPECT(info.key_offset == 1560 + s * 4680);
            EXPECT(info.key_count == 1560 + valid * 4680);
        }
    }
    lvx_slot_info_t info;
    EXPECT(lvx_ring_slot(nullptr, 0, &info) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_ring_slot(&d, 0, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_ring_slot(&d, -1, &info) == LVX_ERR_INVALID_ARG);
    EXPECT(std::strstr(lvx_last_error(), "negative") != nullptr);

    void *p = (void *)(uintptr_t)4096, *odd = (void *)(uintptr_t)4100;
    lvx_kvcache_t *h = nullptr;
    const size_t need = lvx_kvcache_bytes(&d);
    EXPECT(lvx_kvcache_init(&d, nullptr, need, nullptr, &h) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_kvcache_init(&d, (void *)(uintptr_t)(4096 + 16), need, nullptr, &h) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_kvcache_init(&d, p, need - 1, nullptr, &h) == LVX_ERR_SHAPE);
    EXPECT(lvx_kvcache_init(&d, p, need, nullptr, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(h == nullptr);
    EXPECT(lvx_kvcache_destroy(nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_chunk_append_evict(nullptr, 0, p, p, 5120, 0, nullptr, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_chunk_attention(nullptr, 0, p, 5120, 10, 1.0f, p, 5120, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_chunk_attention_prescaled(nullptr, 0, p, 5120, 10, p, 5120, nullptr) == LVX_ERR_INVALID_ARG);

    EXPECT(lvx_linear(p, 100, p, 100, p, 64, 4, 64, 100, LVX_EPI_STORE, nullptr, 0, nullptr, nullptr) == LVX_ERR_SHAPE);
    EXPECT(lvx_linear(p, 128, p, 128, p, 64, 4, 60, 128, LVX_EPI_STORE, nullptr, 0, nullptr, nullptr) == LVX_ERR_SHAPE);
    EXPECT(lvx_linear(p, 64, p, 128, p, 64, 4, 64, 128, LVX_EPI_STORE, nullptr, 0, nullptr, nullptr) == LVX_ERR_SHAPE);
    EXPECT(lvx_linear(p, 128, p, 128, p, 64, 4, 64, 128, (lvx_epilogue_t)7, nullptr, 0, nullptr, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_linear(p, 128, p, 128, p, 64, 4, 64, 128, LVX_EPI_RESID_GATE, nullptr, 0, nullptr, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_linear(odd, 128, p, 128, p, 64, 4, 64, 128, LVX_EPI_STORE, nullptr, 0, nullptr, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_linear_dual(p, 128, p, p, 128, p, 64, 1, p, 64, 4, 64, 64, 100, nullptr) == LVX_ERR_SHAPE);
    EXPECT(lvx_linear_dual(p, 128, p, nullptr, 128, p, 64, 0, p, 64, 4, 64, 64, 128, nullptr) == LVX_ERR_INVALID_ARG);

    lvx_rope_desc_t r = {40, 128, {44, 42, 42}, 10000.0f, 30, 52, 1e-6f, 1};
    lvx_rope_desc_t rbad = r;
    rbad.axes[0] = 46;  // sum of the axis dims != head_dim
    EXPECT(lvx_rope3d(&rbad, p, p, 5120, nullptr, nullptr, 4, 0, p, p, 5120, nullptr) != LVX_OK);
    EXPECT(lvx_rope3d(&r, p, p, 5000, nullptr, nullptr, 4, 0, p, p, 5120, nullptr) == LVX_ERR_SHAPE);
    EXPECT(lvx_rope3d(&r, nullptr, nullptr, 5120, nullptr, nullptr, 4, 0, nullptr, nullptr, 5120, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_rope3d_f32in(&r, (const float *)p, (const float *)p, 5000, nullptr, nullptr, 4, 0, p, p, 5120, nullptr) == LVX_ERR_SHAPE);
    EXPECT(lvx_layernorm_modulate(p, 5120, nullptr, nullptr, 1e-6f, 4, 5124, p, 5120, nullptr) == LVX_ERR_SHAPE);

    // stage descriptors and workspace sizes
    lvx_block_weights_t blocks[2];
    std::memset(blocks, 0, sizeof blocks);
    lvx_stage_t st;
    std::memset(&st, 0, sizeof st);
    st.n_layers = 2;
    st.d_ffn = 13824;
    st.rope = r;
    st.blocks = blocks;
    const size_t ws = lvx_workspace_bytes(&st, 4680, 544);
    EXPECT(ws >= (size_t)4680 * (5120 * 2 + 15360 * 2 + 5120 * 4 + 5120 * 4));
    EXPECT(lvx_workspace_bytes(&st, 4680, 544) == ws);
    EXPECT(lvx_workspace_bytes(nullptr, 4680, 544) == 0);
    lvx_stage_t sbad = st;
    sbad.d_ffn = 13820;
    EXPECT(lvx_workspace_bytes(&sbad, 4680, 544) == 0);
    EXPECT(lvx_dit_block(&st, 0, nullptr, p, 4680, p, 544, nullptr, 0, 1, p, ws, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_denoise_stage(nullptr, nullptr, p, 4680, p, 544, nullptr, -0.25f, 0, 1, p, ws, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_sink_prefill(&st, nullptr, p, p, 544, nullptr, 1, nullptr, p, (size_t)1 << 30, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(std::strstr(lvx_last_error(), "NULL") != nullptr);

    // sink management and FP8 entry points
    EXPECT(lvx_sink_source_bytes(&d) == (size_t)40 * 1560 * 5120 * 4);
    EXPECT(lvx_kvcache_attach_sink_source(nullptr, p, (size_t)1 << 30) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_sink_rope_update(nullptr, &r, 0, 1, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_fp8_quantize(nullptr, 64, 4, 64, p, 64, p, (float *)p, nullptr) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_fp8_quantize(p, 64, 4, 60, p, 64, p, (float *)p, nullptr) == LVX_ERR_SHAPE);
    EXPECT(lvx_fp8_quantize_static(p, 1 << 20, 1 << 12, 1 << 20, p, 1 << 20, (float *)p, nullptr) == LVX_ERR_SHAPE);
    EXPECT(std::strstr(lvx_last_error(), "exceeds") != nullptr);

    // streaming convolution state
    lvx_conv_desc_t cd = {384, 384, 100, 180, 4};
    EXPECT(lvx_causal_conv_state_bytes(&cd) == (size_t)6 * 102 * 182 * 384 * 2);
    lvx_conv_desc_t cbad = {96, 96, 100, 180, 4};
    EXPECT(lvx_causal_conv_state_bytes(&cbad) == 0);
    lvx_causal_conv_t *ch = nullptr;
    EXPECT(lvx_causal_conv_init(&cd, nullptr, lvx_causal_conv_state_bytes(&cd), nullptr, &ch) == LVX_ERR_INVALID_ARG);
    EXPECT(lvx_causal_conv_reset(nullptr, nullptr) == LVX_ERR_INVALID_ARG);

    std::printf("%s (%d failures)\n", failures ? "host checks FAILED" : "host checks passed", failures);
    return failures ? 1 : 0;
}
