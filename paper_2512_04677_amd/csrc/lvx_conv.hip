// Streaming causal 3x3x3 convolution with a two-frame feature cache (paper Appendix C, "Streaming VAE Feature Caching": every
// causal convolution of the decoder keeps the activations of its two most recent input frames and prepends them as causal
// context when the next frames arrive, so decoding is incremental and nothing is recomputed).
//
// State of one layer = a zero-padded channels-last volume P[max_frames + 2][H + 2][W + 2][C_in] in caller-owned device memory:
// frames 0 and 1 are the feature cache (zeros before the first frame), frames 2.. receive the new input frames, the one-pixel
// border stays zero (spatial padding).  A step copies the cache forward, scatters the new frames into the interior and runs
// one implicit GEMM on the matrix cores: rows = output pixels, K = 27 taps x C_in channels read straight from P by the GEMM's
// direct-to-LDS loads (a tap is a constant shift in P), columns = C_out.  No im2col buffer is ever written.
#include "lvx_internal.h"

#include <new>

struct lvx_causal_conv {
    lvx_conv_desc_t desc;
    bf16_t *vol;          // the padded volume
    int64_t frame_elems;  // (H+2)*(W+2)*C_in
    int32_t last_frames;  // frames scattered by the previous step (0 = none yet)
};

namespace {

// interior copy: x [n_frames][H][W][C] -> P[2 + f][1 + y][1 + x][:]
__global__ void __launch_bounds__(256) lvx_conv_scatter_kernel(const bf16_t *__restrict__ x, bf16_t *__restrict__ vol, int n_frames, int H,
                                                               int W, int chunks_per_pixel, int64_t frame_elems, int row_pitch) {
    const size_t total = (size_t)n_frames * H * W * chunks_per_pixel;
    const int C = chunks_per_pixel * 8;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t pix = i / chunks_per_pixel;
        const int c = (int)(i % chunks_per_pixel);
        const int xw = (int)(pix % W);
        const int y = (int)((pix / W) % H);
        const int f = (int)(pix / ((size_t)W * H));
        const uint4 v = reinterpret_cast<const uint4 *>(x + pix * C)[c];
        reinterpret_cast<uint4 *>(vol + (size_t)(f + 2) * frame_elems + (size_t)(y + 1) * row_pitch + (size_t)(xw + 1) * C)[c] = v;
    }
}

int grid_for(size_t n_items) {
    size_t g = (n_items + 255) / 256;
    if (g > 256 * 16) g = 256 * 16;
    return (int)(g ? g : 1);
}

lvx_status_t check_conv_desc(const lvx_conv_desc_t *d) {
    LVX_REQUIRE(d != nullptr, LVX_ERR_INVALID_ARG, "conv descriptor is NULL");
    LVX_REQUIRE(d->c_in > 0 && d->c_out > 0 && d->height > 0 && d->width > 0 && d->max_frames > 0, LVX_ERR_SHAPE,
                "conv descriptor has a non-positive size");
    LVX_REQUIRE(d->c_in % 64 == 0, LVX_ERR_UNSUPPORTED, "c_in %d must be a multiple of 64 (one K slab per tap and channel group)", d->c_in);
    LVX_REQUIRE(d->c_out % 8 == 0, LVX_ERR_SHAPE, "c_out %d must be a multiple of 8", d->c_out);
    const uint64_t vol_bytes = (uint64_t)(d->max_frames + 2) * (d->height + 2) * (d->width + 2) * d->c_in * 2;
    LVX_REQUIRE(vol_bytes < (1ull << 32), LVX_ERR_SHAPE, "padded volume of %llu bytes exceeds 4 GiB (32-bit offsets inside the kernel)",
                (unsigned long long)vol_bytes);
    LVX_REQUIRE((uint64_t)d->max_frames * d->height * d->width < (1ull << 31), LVX_ERR_SHAPE, "too many output pixels per step");
    return LVX_OK;
}

}  // namespace

extern "C" size_t lvx_causal_conv_state_bytes(const lvx_conv_desc_t *desc) {
    if (check_conv_desc(desc) != LVX_OK) return 0;
    return (size_t)(desc->max_frames + 2) * (desc->height + 2) * (desc->width + 2) * desc->c_in * sizeof(bf16_t);
}

extern "C" lvx_status_t lvx_causal_conv_init(const lvx_conv_desc_t *desc, void *dev_state, size_t bytes, lvx_stream_t stream,
                                             lvx_causal_conv_t **out) {
    LVX_TRY(check_conv_desc(desc));
    LVX_REQUIRE(out != nullptr, LVX_ERR_INVALID_ARG, "out handle pointer is NULL");
    LVX_REQUIRE(dev_state != nullptr && (((uintptr_t)dev_state) & 255u) == 0, LVX_ERR_INVALID_ARG,
                "state storage must be non-NULL and 256-byte aligned");
    const size_t need = lvx_causal_conv_state_bytes(desc);
    LVX_REQUIRE(bytes >= need, LVX_ERR_SHAPE, "state storage too small: %zu bytes given, %zu needed", bytes, need);
    lvx_causal_conv *c = new (std::nothrow) lvx_causal_conv;
    LVX_REQUIRE(c != nullptr, LVX_ERR_INVALID_ARG, "out of host memory");
    c->desc = *desc;
    c->vol = (bf16_t *)dev_state;
    c->frame_elems = (int64_t)(desc->height + 2) * (desc->width + 2) * desc->c_in;
    c->last_frames = 0;
    // zero history (the sequence starts from zeros on the past side) and zero borders
    lvx_status_t st = lvx_launch_fill_zero(dev_state, need / 16 * 16, (hipStream_t)stream);
    if (st != LVX_OK) {
        delete c;
        return st;
    }
    *out = c;
    return LVX_OK;
}

extern "C" lvx_status_t lvx_causal_conv_destroy(lvx_causal_conv_t *conv) {
    LVX_REQUIRE(conv != nullptr, LVX_ERR_INVALID_ARG, "conv handle is NULL");
    delete conv;
    return LVX_OK;
}

extern "C" lvx_status_t lvx_causal_conv_reset(lvx_causal_conv_t *c, lvx_stream_t stream) {
    LVX_REQUIRE(c != nullptr, LVX_ERR_INVALID_ARG, "conv handle is NULL");
    c->last_frames = 0;
    return lvx_launch_fill_zero(c->vol, (size_t)2 * c->frame_elems * sizeof(bf16_t) / 16 * 16, (hipStream_t)stream);
}

extern "C" lvx_status_t lvx_causal_conv_step(lvx_causal_conv_t *c, const void *dev_x, int32_t n_frames, const void *dev_w, int64_t ldw,
                                             const float *dev_bias, int32_t act, void *dev_y, lvx_stream_t stream) {
    LVX_REQUIRE(c != nullptr, LVX_ERR_INVALID_ARG, "conv handle is NULL");
    LVX_REQUIRE(dev_x != nullptr && dev_w != nullptr && dev_y != nullptr, LVX_ERR_INVALID_ARG, "x, w or y is NULL");
    LVX_REQUIRE(lvx_aligned16(dev_x) && lvx_aligned16(dev_w) && lvx_aligned16(dev_y) && lvx_aligned16(dev_bias), LVX_ERR_INVALID_ARG,
                "pointers must be 16-byte aligned");
    const lvx_conv_desc_t &d = c->desc;
    LVX_REQUIRE(n_frames > 0 && n_frames <= d.max_frames, LVX_ERR_SHAPE, "n_frames %d not in 1..%d", n_frames, d.max_frames);
    const int K = 27 * d.c_in;
    LVX_REQUIRE(ldw >= K && ldw % 8 == 0, LVX_ERR_SHAPE, "weight row stride %lld must be a multiple of 8 and >= 27*c_in = %d", (long long)ldw, K);
    LVX_REQUIRE((uint64_t)d.c_out * (uint64_t)ldw * 2 < (1ull << 32), LVX_ERR_SHAPE, "weight matrix larger than 4 GiB");
    LVX_REQUIRE(act == 0 || act == 1, LVX_ERR_INVALID_ARG, "act %d must be 0 (none) or 1 (SiLU)", act);
    hipStream_t st = (hipStream_t)stream;
    const int row_pitch = (d.width + 2) * d.c_in;
    // the two most recent input frames of the previous step become frames 0 and 1 (frame by frame, oldest first: the ranges
    // overlap when the previous step had a single frame)
    if (c->last_frames > 0) {
        const int lf = c->last_frames;
        for (int j = 0; j < 2; ++j)
            LVX_TRY(lvx_launch_copy_rows(c->vol + (size_t)(lf + j) * c->frame_elems, c->frame_elems, c->vol + (size_t)j * c->frame_elems,
                                         c->frame_elems, 1, (int)c->frame_elems, st));
    }
    const size_t chunks = (size_t)n_frames * d.height * d.width * (d.c_in / 8);
    hipLaunchKernelGGL(lvx_conv_scatter_kernel, dim3(grid_for(chunks)), dim3(256), 0, st, (const bf16_t *)dev_x, c->vol, n_frames, d.height,
                       d.width, d.c_in / 8, c->frame_elems, row_pitch);
    LVX_CHECK_HIP(hipGetLastError());
    lvx_conv_map_t cm;
    cm.enabled = 1;
    cm.H = d.height;
    cm.W = d.width;
    cm.C = d.c_in;
    cm.slabs_per_tap = d.c_in / 64;
    cm.row_pitch = row_pitch;
    cm.frame_pitch = (int32_t)c->frame_elems;
    LVX_TRY(lvx_launch_conv_gemm(c->vol, cm, (const bf16_t *)dev_w, ldw, dev_bias, act, (bf16_t *)dev_y, d.c_out, n_frames * d.height * d.width,
                                 d.c_out, st));
    c->last_frames = n_frames;
    return LVX_OK;
}
