// HBM-bound row kernels: fused Q/K RMSNorm + 3-D rotary embedding, and LayerNorm + modulation.
//
// One 64-lane wave owns one token row (all heads), four rows per workgroup, no LDS and no barriers: the row is
// read once with 16-byte loads, kept in registers, reduced with wave shuffles, transformed and written once.
// Rotary indices count latent frames and reach ~4e4 in long rollouts (paper Appendix D, "Rolling RoPE"; Sec. 4.3
// 10 000 s experiment), where an fp32 product pos*freq already loses ~1e-3 rad, so each token's head_dim/2 angles
// are formed and reduced in fp64 (one per lane, shared by all heads and by q and k) and only the resulting
// sin/cos are kept in fp32.
#include "lvx_internal.h"

#include <math.h>

namespace {

struct gain_table_t {  // per-batch gain vectors of the k input (n = 0: g_k serves every batch)
    int32_t n, pad;
    const float *g[LVX_GEMM_MAX_SEGS];
};

struct rope_table_t {
    double inv_freq[64];  // theta^(-2k/d_a) of pair p (p = global pair index inside the head)
    int32_t axis[64];     // 0 = t, 1 = y, 2 = x
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
    return v;
}

constexpr int ROWS_PER_WG = 4;

// CPL = 8-element chunks per lane (row length <= 64*8*CPL).  IN_MODE: 0 = q and k rows are bf16, 1 = both fp32, 2 = q bf16 and
// k fp32 (row strides and batch strides of an fp32 input count fp32 elements; ld_in is q's row stride, ld_in_k is k's).
// F32OUT (norm-only form, needs fp32 input): the result is stored in fp32, token-major, un-rounded
template <int CPL, int IN_MODE, bool F32OUT = false>
__global__ void __launch_bounds__(64 * ROWS_PER_WG)
    lvx_rope_norm_kernel(const void *q_in, const void *k_in, int64_t ld_in, int64_t ld_in_k,
                         const float *__restrict__ g_q, const float *__restrict__ g_k, int n_tokens, int t0, bf16_t *q_out,
                         bf16_t *k_out, int64_t ld_out, int64_t ld_out_head, int d_model, int head_dim, int frame_h, int frame_w,
                         float eps, int apply_rope, rope_table_t tab, int n_batch, int64_t batch_stride_in, int64_t batch_stride_out,
                         gain_table_t gtab, float q_scale, int64_t ld_out_k, int64_t ld_out_head_k) {
    // n_batch independent row sets of n_tokens rows each (the sink keys of several layers in one launch); positions and t0
    // are those of the row inside its set
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 6);
    if (row >= (int64_t)n_tokens * n_batch) return;
    const int batch = (int)(row / n_tokens);
    const int token = (int)(row % n_tokens);
    const int n_chunks = d_model / 8;
    const int cph = head_dim / 8;  // chunks per head: 8 or 16, divides 64, so (lane + 64 j) % cph == lane % cph

    float cs = 1.f, sn = 0.f;
    if (apply_rope && lane < head_dim / 2) {
        const int ax = tab.axis[lane];
        const int pos = ax == 0 ? t0 + token / (frame_h * frame_w) : (ax == 1 ? (token / frame_w) % frame_h : token % frame_w);
        double s, c;
        sincos((double)pos * tab.inv_freq[lane], &s, &c);
        cs = (float)c;
        sn = (float)s;
    }
    float c4[4], s4[4];
    const int p0 = (lane % cph) * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        c4[j] = __shfl(cs, p0 + j);
        s4[j] = __shfl(sn, p0 + j);
    }

#pragma unroll
    for (int which = 0; which < 2; ++which) {
        if (gridDim.y == 2 && which != (int)blockIdx.y) continue;  // q and k rows of a token go to different waves
        const void *in = which == 0 ? q_in : k_in;
        bf16_t *outp = which == 0 ? q_out : k_out;
        const float *g = which == 0 ? g_q : (gtab.n > 0 ? gtab.g[batch] : g_k);
        if (in == nullptr) continue;
        const bool F32IN = IN_MODE == 1 || (IN_MODE == 2 && which == 1);
        const size_t row_off = (size_t)batch * batch_stride_in + (size_t)token * (which == 0 ? ld_in : ld_in_k);
        float x[CPL][8];
        float ss = 0.f;
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int c = lane + 64 * j;
            if (c < n_chunks) {
                if (F32IN) {
                    const float4 *src = reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(in) + row_off) + 2 * c;
                    const float4 a = src[0], b = src[1];
                    x[j][0] = a.x, x[j][1] = a.y, x[j][2] = a.z, x[j][3] = a.w, x[j][4] = b.x, x[j][5] = b.y, x[j][6] = b.z, x[j][7] = b.w;
                } else {
                    const u32x4_t v = reinterpret_cast<const u32x4_t *>(reinterpret_cast<const bf16_t *>(in) + row_off)[c];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        x[j][2 * e] = bf16_lo(v[e]);
                        x[j][2 * e + 1] = bf16_hi(v[e]);
                    }
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) ss += x[j][e] * x[j][e];
            }
        }
        float rinv = 1.f;
        if (g != nullptr) {
            ss = wave_sum(ss);
            rinv = 1.0f / sqrtf(ss / (float)d_model + eps);
        }
        if (which == 0) rinv *= q_scale;  // 1, or the attention's logit scale folded into the queries before their rounding
        // element (token, head, e) of the output lives at token*ld_out + head*ld_out_head + e: token-major rows have
        // ld_out_head = head_dim, packed cache K rows [head][key][head_dim] have ld_out = head_dim, ld_out_head = cap*head_dim
        // (the k rows may have strides of their own: q token-major for the attention, k straight into the cache's packed rows)
        const int64_t ldo = which == 0 ? ld_out : ld_out_k, ldoh = which == 0 ? ld_out_head : ld_out_head_k;
        bf16_t *dst = outp + (size_t)batch * batch_stride_out + (size_t)token * ldo;
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int c = lane + 64 * j;
            if (c < n_chunks) {
                float4 g0 = make_float4(1.f, 1.f, 1.f, 1.f), g1 = g0;
                if (g != nullptr) {
                    g0 = *reinterpret_cast<const float4 *>(g + c * 8);
                    g1 = *reinterpret_cast<const float4 *>(g + c * 8 + 4);
                }
                const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
                if (F32OUT) {  // normalised, un-rotated, un-rounded
                    float4 *o = reinterpret_cast<float4 *>(reinterpret_cast<float *>(outp) + (size_t)token * ld_out) + 2 * c;
                    o[0] = make_float4(x[j][0] * rinv * gg[0], x[j][1] * rinv * gg[1], x[j][2] * rinv * gg[2], x[j][3] * rinv * gg[3]);
                    o[1] = make_float4(x[j][4] * rinv * gg[4], x[j][5] * rinv * gg[5], x[j][6] * rinv * gg[6], x[j][7] * rinv * gg[7]);
                    continue;
                }
                u32x4_t y;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a = x[j][2 * e] * rinv * gg[2 * e];
                    const float b = x[j][2 * e + 1] * rinv * gg[2 * e + 1];
                    y[e] = pack_bf16x2(a * c4[e] - b * s4[e], a * s4[e] + b * c4[e]);
                }
                *reinterpret_cast<u32x4_t *>(dst + (size_t)(c / cph) * ldoh + (c % cph) * 8) = y;
            }
        }
    }
}

// Input row is bf16 or fp32 (the residual stream is carried in fp32 inside a block / stage); output is bf16.
template <int CPL, bool F32IN, bool AMAX>
__global__ void __launch_bounds__(64 * ROWS_PER_WG)
    lvx_layernorm_modulate_kernel(const void *__restrict__ x_in, int64_t ldx, const float *__restrict__ shift,
                                  const float *__restrict__ scale, float eps, int n_tokens, int d, bf16_t *__restrict__ u_out,
                                  int64_t ldu, uint32_t *__restrict__ amax_slots) {
    const int lane = threadIdx.x & 63;
    const int token = blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 6);
    // AMAX: the output feeds an FP8 linear, whose per-tensor scale needs max |u| over the whole tensor: every
    // workgroup adds the largest magnitude among the bf16 values it stores (one atomic per workgroup, spread over the slots)
    __shared__ uint32_t wg_amax[ROWS_PER_WG];
    uint32_t amax_b = 0;
    if (token < n_tokens) {
        const int n_chunks = d / 8;
        float x[CPL][8];
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int c = lane + 64 * j;
            if (c < n_chunks) {
                if (F32IN) {
                    const float4 *src = reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(x_in) + (size_t)token * ldx) + 2 * c;
                    const float4 a = src[0], b = src[1];
                    x[j][0] = a.x, x[j][1] = a.y, x[j][2] = a.z, x[j][3] = a.w, x[j][4] = b.x, x[j][5] = b.y, x[j][6] = b.z, x[j][7] = b.w;
                } else {
                    const u32x4_t v = reinterpret_cast<const u32x4_t *>(reinterpret_cast<const bf16_t *>(x_in) + (size_t)token * ldx)[c];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        x[j][2 * e] = bf16_lo(v[e]);
                        x[j][2 * e + 1] = bf16_hi(v[e]);
                    }
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) sum += x[j][e];
            }
        }
        const float mean = wave_sum(sum) / (float)d;
        float sq = 0.f;
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int c = lane + 64 * j;
            if (c < n_chunks) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float a = x[j][e] - mean;
                    sq += a * a;
                }
            }
        }
        const float rinv = 1.0f / sqrtf(wave_sum(sq) / (float)d + eps);
        u32x4_t *dst = reinterpret_cast<u32x4_t *>(u_out + (size_t)token * ldu);
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int c = lane + 64 * j;
            if (c < n_chunks) {
                float sc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, sh[8] = {0, 0, 0, 0, 0, 0, 0, 0};
                if (scale != nullptr) {
                    const float4 a = *reinterpret_cast<const float4 *>(scale + c * 8), b = *reinterpret_cast<const float4 *>(scale + c * 8 + 4);
                    sc[0] = a.x, sc[1] = a.y, sc[2] = a.z, sc[3] = a.w, sc[4] = b.x, sc[5] = b.y, sc[6] = b.z, sc[7] = b.w;
                }
                if (shift != nullptr) {
                    const float4 a = *reinterpret_cast<const float4 *>(shift + c * 8), b = *reinterpret_cast<const float4 *>(shift + c * 8 + 4);
                    sh[0] = a.x, sh[1] = a.y, sh[2] = a.z, sh[3] = a.w, sh[4] = b.x, sh[5] = b.y, sh[6] = b.z, sh[7] = b.w;
                }
                u32x4_t y;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a = (x[j][2 * e] - mean) * rinv * (1.f + sc[2 * e]) + sh[2 * e];
                    const float b = (x[j][2 * e + 1] - mean) * rinv * (1.f + sc[2 * e + 1]) + sh[2 * e + 1];
                    y[e] = pack_bf16x2(a, b);
                    if (AMAX) {
                        const uint32_t lo = y[e] & 0x7fffu, hi = (y[e] >> 16) & 0x7fffu;
                        amax_b = amax_b > lo ? amax_b : lo;
                        amax_b = amax_b > hi ? amax_b : hi;
                    }
                }
                dst[c] = y;
            }
        }
    }
    if (AMAX) {  // every wave of the workgroup gets here
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)amax_b, s);
            amax_b = amax_b > o ? amax_b : o;
        }
        if (lane == 0) wg_amax[threadIdx.x >> 6] = amax_b;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t m = wg_amax[0];
#pragma unroll
            for (int w = 1; w < ROWS_PER_WG; ++w) m = m > wg_amax[w] ? m : wg_amax[w];
            if (m != 0) atomicMax(amax_slots + (blockIdx.x & (LVX_AMAX_SLOTS - 1)), m << 16);
        }
    }
}

}  // namespace

static lvx_status_t check_rope_desc(const lvx_rope_desc_t *r) {
    LVX_REQUIRE(r != nullptr, LVX_ERR_INVALID_ARG, "rope descriptor is NULL");
    LVX_REQUIRE(r->n_heads > 0 && r->frame_h > 0 && r->frame_w > 0, LVX_ERR_SHAPE, "rope descriptor has a non-positive size");
    LVX_REQUIRE(r->head_dim == 64 || r->head_dim == 128, LVX_ERR_UNSUPPORTED, "head_dim %d not supported (64 or 128)", r->head_dim);
    if (r->apply_rope) {
        LVX_REQUIRE(r->axes[0] >= 0 && r->axes[1] >= 0 && r->axes[2] >= 0 && r->axes[0] % 2 == 0 && r->axes[1] % 2 == 0 &&
                        r->axes[2] % 2 == 0 && r->axes[0] + r->axes[1] + r->axes[2] == r->head_dim,
                    LVX_ERR_SHAPE, "rope axes (%d,%d,%d) must be even and sum to head_dim %d", r->axes[0], r->axes[1], r->axes[2],
                    r->head_dim);
        LVX_REQUIRE(r->theta > 1.f, LVX_ERR_INVALID_ARG, "rope theta must be > 1");
    }
    LVX_REQUIRE((int64_t)r->n_heads * r->head_dim <= 64 * 8 * 16, LVX_ERR_UNSUPPORTED, "n_heads*head_dim %lld exceeds 8192",
                (long long)r->n_heads * r->head_dim);
    return LVX_OK;
}

static lvx_status_t launch_rope(const lvx_rope_desc_t *desc, const void *q_in, const void *k_in, int64_t ld_in, const float *g_q,
                                const float *g_k, int n_tokens, int t0, bf16_t *q_out, bf16_t *k_out, int64_t ld_out, int64_t ld_out_head,
                                hipStream_t stream, int n_batch = 1, int64_t batch_stride_in = 0, int64_t batch_stride_out = 0,
                                int in_mode = 0, const gain_table_t *gains = nullptr, int64_t ld_in_k = -1, float q_scale = 1.0f,
                                int64_t ld_out_k = -1, int64_t ld_out_head_k = -1) {
    if (ld_in_k < 0) ld_in_k = ld_in;
    if (ld_out_k < 0) ld_out_k = ld_out, ld_out_head_k = ld_out_head;
    gain_table_t gtab = {};
    if (gains != nullptr) gtab = *gains;
    const int d = desc->n_heads * desc->head_dim;
    rope_table_t tab;
    for (int p = 0; p < 64; ++p) {
        tab.inv_freq[p] = 0.0;
        tab.axis[p] = 0;
    }
    if (desc->apply_rope) {
        int p = 0;
        for (int ax = 0; ax < 3; ++ax)
            for (int k = 0; k < desc->axes[ax] / 2; ++k, ++p) {
                tab.inv_freq[p] = pow((double)desc->theta, -2.0 * k / (double)desc->axes[ax]);
                tab.axis[p] = ax;
            }
    }
    // with both inputs present the q rows and the k rows are handled by different workgroups (twice the waves in flight,
    // half the dependent load -> reduce -> store chain per wave)
    const dim3 grid((unsigned)(((int64_t)n_tokens * n_batch + ROWS_PER_WG - 1) / ROWS_PER_WG), (q_in != nullptr && k_in != nullptr) ? 2 : 1),
        block(64 * ROWS_PER_WG);
    const int cpl = (d / 8 + 63) / 64;
#define LVX_ROPE_LAUNCH(CPL, MODE)                                                                                               \
    hipLaunchKernelGGL((lvx_rope_norm_kernel<CPL, MODE>), grid, block, 0, stream, q_in, k_in, ld_in, ld_in_k, g_q, g_k, n_tokens, t0, q_out, \
                       k_out, ld_out, ld_out_head, d, desc->head_dim, desc->frame_h, desc->frame_w, desc->eps, desc->apply_rope, tab,    \
                       n_batch, batch_stride_in, batch_stride_out, gtab, q_scale, ld_out_k, ld_out_head_k)
#define LVX_ROPE_LAUNCH_MODE(MODE)          \
    if (cpl <= 2)                           \
        LVX_ROPE_LAUNCH(2, MODE);           \
    else if (cpl <= 10)                     \
        LVX_ROPE_LAUNCH(10, MODE);          \
    else                                    \
        LVX_ROPE_LAUNCH(16, MODE)
    if (in_mode == 1) {
        LVX_ROPE_LAUNCH_MODE(1);
    } else if (in_mode == 2) {
        LVX_ROPE_LAUNCH_MODE(2);
    } else {
        LVX_ROPE_LAUNCH_MODE(0);
    }
#undef LVX_ROPE_LAUNCH_MODE
#undef LVX_ROPE_LAUNCH
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

static lvx_status_t rope3d_entry(const lvx_rope_desc_t *desc, const void *dev_q_in, const void *dev_k_in, int64_t ld_in, bool f32_in,
                                 const float *dev_g_q, const float *dev_g_k, int32_t n_tokens, int32_t t0, void *dev_q_out,
                                 void *dev_k_out, int64_t ld_out, lvx_stream_t stream, float q_scale = 1.0f) {
    lvx_status_t st = check_rope_desc(desc);
    if (st != LVX_OK) return st;
    LVX_REQUIRE(dev_q_in != nullptr || dev_k_in != nullptr, LVX_ERR_INVALID_ARG, "both q and k are NULL");
    LVX_REQUIRE((dev_q_in == nullptr) == (dev_q_out == nullptr) && (dev_k_in == nullptr) == (dev_k_out == nullptr), LVX_ERR_INVALID_ARG,
                "each input needs its output pointer");
    LVX_REQUIRE(lvx_aligned16(dev_q_in) && lvx_aligned16(dev_k_in) && lvx_aligned16(dev_q_out) && lvx_aligned16(dev_k_out) &&
                    lvx_aligned16(dev_g_q) && lvx_aligned16(dev_g_k),
                LVX_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    const int d = desc->n_heads * desc->head_dim;
    LVX_REQUIRE(ld_in >= d && ld_in % 8 == 0 && ld_out >= d && ld_out % 8 == 0, LVX_ERR_SHAPE,
                "row strides must be multiples of 8 and >= n_heads*head_dim");
    LVX_REQUIRE(n_tokens >= 0 && t0 >= 0, LVX_ERR_INVALID_ARG, "n_tokens and t0 must be non-negative");
    if (n_tokens == 0) return LVX_OK;

    return launch_rope(desc, dev_q_in, dev_k_in, ld_in, dev_g_q, dev_g_k, n_tokens, t0, (bf16_t *)dev_q_out, (bf16_t *)dev_k_out, ld_out,
                       desc->head_dim, (hipStream_t)stream, 1, 0, 0, f32_in ? 1 : 0, nullptr, -1, q_scale);
}

extern "C" lvx_status_t lvx_rope3d(const lvx_rope_desc_t *desc, const void *dev_q_in, const void *dev_k_in, int64_t ld_in,
                                   const float *dev_g_q, const float *dev_g_k, int32_t n_tokens, int32_t t0, void *dev_q_out,
                                   void *dev_k_out, int64_t ld_out, lvx_stream_t stream) {
    return rope3d_entry(desc, dev_q_in, dev_k_in, ld_in, false, dev_g_q, dev_g_k, n_tokens, t0, dev_q_out, dev_k_out, ld_out, stream);
}

extern "C" lvx_status_t lvx_rope3d_f32in(const lvx_rope_desc_t *desc, const float *dev_q_in, const float *dev_k_in, int64_t ld_in,
                                         const float *dev_g_q, const float *dev_g_k, int32_t n_tokens, int32_t t0, void *dev_q_out,
                                         void *dev_k_out, int64_t ld_out, lvx_stream_t stream) {
    return rope3d_entry(desc, dev_q_in, dev_k_in, ld_in, true, dev_g_q, dev_g_k, n_tokens, t0, dev_q_out, dev_k_out, ld_out, stream);
}

// The block's RMSNorm + RoPE: q rows bf16 (ld_q elements); k rows fp32 (ld_k fp32 elements: a bf16 stage's QKV projection keeps its
// k columns un-rounded, they become the cached keys) or bf16 (ld_k bf16 elements).  Outputs bf16: q token-major with row stride
// ld_out, multiplied by q_scale before the rounding (the attention kernel's pre-scaled mode); k with element (token, head, e) at
// token * ld_out_k + head * ld_out_head_k + e (token-major rows, or straight into the cache's packed rows).
lvx_status_t lvx_launch_rope_qk(const lvx_rope_desc_t *desc, const bf16_t *q_in, int64_t ld_q, const void *k_in, int k_is_f32, int64_t ld_k,
                                const float *g_q, const float *g_k, int n_tokens, int t0, bf16_t *q_out, int64_t ld_out, bf16_t *k_out,
                                int64_t ld_out_k, int64_t ld_out_head_k, float q_scale, hipStream_t stream) {
    lvx_status_t st = check_rope_desc(desc);
    if (st != LVX_OK) return st;
    if (n_tokens == 0) return LVX_OK;
    return launch_rope(desc, q_in, k_in, ld_q, g_q, g_k, n_tokens, t0, q_out, k_out, ld_out, desc->head_dim, stream, 1, 0, 0, k_is_f32 ? 2 : 0,
                       nullptr, ld_k, q_scale, ld_out_k, ld_out_head_k);
}

lvx_status_t lvx_launch_rope_to_packed_k(const lvx_rope_desc_t *desc, const float *src, int64_t ld_src, int n_tokens, int t0,
                                         bf16_t *k_packed, int cap, int n_layers, int64_t layer_stride_src, int64_t layer_stride_dst,
                                         hipStream_t stream) {
    lvx_status_t st = check_rope_desc(desc);
    if (st != LVX_OK) return st;
    if (n_tokens == 0 || n_layers == 0) return LVX_OK;
    return launch_rope(desc, nullptr, src, ld_src, nullptr, nullptr, n_tokens, t0, nullptr, k_packed, desc->head_dim,
                       (int64_t)cap * desc->head_dim, stream, n_layers, layer_stride_src, layer_stride_dst, 1);
}

lvx_status_t lvx_launch_norm_to_packed_k(const lvx_rope_desc_t *desc, const void *src, int src_is_f32, int64_t ld_src, int n_tokens,
                                         const float *const *gains, bf16_t *k_packed, int cap, int n_batch, int64_t batch_stride_src,
                                         int64_t batch_stride_dst, hipStream_t stream) {
    lvx_status_t st = check_rope_desc(desc);
    if (st != LVX_OK) return st;
    LVX_REQUIRE(n_batch >= 0 && n_batch <= LVX_GEMM_MAX_SEGS, LVX_ERR_INVALID_ARG, "norm to packed K: %d batches (0..%d)", n_batch, LVX_GEMM_MAX_SEGS);
    if (n_tokens == 0 || n_batch == 0) return LVX_OK;
    lvx_rope_desc_t norm_only = *desc;
    norm_only.apply_rope = 0;
    gain_table_t gt = {};
    gt.n = n_batch;
    for (int b = 0; b < n_batch; ++b) gt.g[b] = gains[b];
    return launch_rope(&norm_only, nullptr, src, ld_src, nullptr, nullptr, n_tokens, 0, nullptr, k_packed, desc->head_dim,
                       (int64_t)cap * desc->head_dim, stream, n_batch, batch_stride_src, batch_stride_dst, src_is_f32 ? 1 : 0, &gt);
}

lvx_status_t lvx_launch_rmsnorm_f32(const lvx_rope_desc_t *desc, const float *x, int64_t ld_in, const float *g, int n_tokens, float *y,
                                    int64_t ld_out, hipStream_t stream) {
    lvx_status_t st = check_rope_desc(desc);
    if (st != LVX_OK) return st;
    if (n_tokens == 0) return LVX_OK;
    const int d = desc->n_heads * desc->head_dim;
    rope_table_t tab = {};
    const dim3 grid((unsigned)((n_tokens + ROWS_PER_WG - 1) / ROWS_PER_WG)), block(64 * ROWS_PER_WG);
    const int cpl = (d / 8 + 63) / 64;
#define LVX_NORM32_LAUNCH(CPL)                                                                                                     \
    hipLaunchKernelGGL((lvx_rope_norm_kernel<CPL, 1, true>), grid, block, 0, stream, (const void *)nullptr, (const void *)x, ld_in, ld_in, \
                       (const float *)nullptr, g, n_tokens, 0, (bf16_t *)nullptr, (bf16_t *)y, ld_out, (int64_t)desc->head_dim, d,    \
                       desc->head_dim, desc->frame_h, desc->frame_w, desc->eps, 0, tab, 1, (int64_t)0, (int64_t)0, gain_table_t{}, 1.0f, ld_out, (int64_t)desc->head_dim)
    if (cpl <= 2)
        LVX_NORM32_LAUNCH(2);
    else if (cpl <= 10)
        LVX_NORM32_LAUNCH(10);
    else
        LVX_NORM32_LAUNCH(16);
#undef LVX_NORM32_LAUNCH
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

lvx_status_t lvx_launch_layernorm(const void *x, int x_is_f32, int64_t ldx, const float *shift, const float *scale, float eps,
                                  int n_tokens, int d, bf16_t *u, int64_t ldu, hipStream_t stream, uint32_t *amax_slots) {
    LVX_REQUIRE(x != nullptr && u != nullptr, LVX_ERR_INVALID_ARG, "x or u is NULL");
    LVX_REQUIRE(lvx_aligned16(x) && lvx_aligned16(u) && lvx_aligned16(shift) && lvx_aligned16(scale), LVX_ERR_INVALID_ARG,
                "pointers must be 16-byte aligned");
    LVX_REQUIRE(d > 0 && d % 8 == 0 && d <= 64 * 8 * 16, LVX_ERR_SHAPE, "d %d must be a positive multiple of 8, at most 8192", d);
    LVX_REQUIRE(ldx >= d && ldx % 8 == 0 && ldu >= d && ldu % 8 == 0, LVX_ERR_SHAPE, "row strides must be multiples of 8 and >= d");
    LVX_REQUIRE(n_tokens >= 0, LVX_ERR_INVALID_ARG, "n_tokens must be non-negative");
    if (n_tokens == 0) return LVX_OK;
    const dim3 grid((n_tokens + ROWS_PER_WG - 1) / ROWS_PER_WG), block(64 * ROWS_PER_WG);
    const int cpl = (d / 8 + 63) / 64;
#define LVX_LN_LAUNCH(CPL, F32)                                                                                                      \
    do {                                                                                                                             \
        if (amax_slots != nullptr)                                                                                                   \
            hipLaunchKernelGGL((lvx_layernorm_modulate_kernel<CPL, F32, true>), grid, block, 0, stream, x, ldx, shift, scale, eps, n_tokens, d, \
                               u, ldu, amax_slots);                                                                                  \
        else                                                                                                                         \
            hipLaunchKernelGGL((lvx_layernorm_modulate_kernel<CPL, F32, false>), grid, block, 0, stream, x, ldx, shift, scale, eps, n_tokens, d, \
                               u, ldu, amax_slots);                                                                                  \
    } while (0)
    if (x_is_f32) {
        if (cpl <= 2)
            LVX_LN_LAUNCH(2, true);
        else if (cpl <= 10)
            LVX_LN_LAUNCH(10, true);
        else
            LVX_LN_LAUNCH(16, true);
    } else {
        if (cpl <= 2)
            LVX_LN_LAUNCH(2, false);
        else if (cpl <= 10)
            LVX_LN_LAUNCH(10, false);
        else
            LVX_LN_LAUNCH(16, false);
    }
#undef LVX_LN_LAUNCH
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

extern "C" lvx_status_t lvx_layernorm_modulate(const void *dev_x, int64_t ldx, const float *dev_shift, const float *dev_scale, float eps,
                                               int32_t n_tokens, int32_t d, void *dev_u, int64_t ldu, lvx_stream_t stream) {
    return lvx_launch_layernorm(dev_x, 0, ldx, dev_shift, dev_scale, eps, n_tokens, d, (bf16_t *)dev_u, ldu, (hipStream_t)stream, nullptr);
}
