// Rolling KV cache: host ring bookkeeping + the append / sink / gather kernels.
//
// Protocol (cache update of Alg. 3 / Alg. 4: a cache that already holds L entries drops its oldest, then appends; Sec. 3.3: one sink
// frame stays for ever; Sec. 3.2: a block attends to itself in full).  The forward of chunk i has to see chunk i's own
// K/V, so the write happens before the attention and the ring has window+1 slots: chunk i lands in slot
// i mod (window+1) and physically overwrites chunk i-(window+1), which the list protocol had already dropped after
// the forward of chunk i-1.
//
// HBM layout per layer (private): K  [head][cap_keys][D]            -> a 64-key K tile of one head is 64*D contiguous bf16
//                                 V^T[head][cap_keys/64][D][64]     -> a 64-key V tile is stored transposed, contiguous,
// so both tiles stream into LDS with 16-byte loads and are direct MFMA A-operands (contraction index contiguous).
// Key rows: [0, sink_keys) sink, then slot s at sink_keys + s*chunk_keys.
#include "lvx_internal.h"

#include <new>
#include <string.h>

// ------------------------------------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

lvx_status_t lvx_fail(lvx_status_t code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" const char *lvx_last_error(void) { return g_err; }
extern "C" const char *lvx_version(void) { return "lvx 0.1 gfx950"; }

// ------------------------------------------------------------------------------------------------ kernels
__global__ void __launch_bounds__(256) lvx_fill_zero_kernel(uint4 *p, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (; i < n16; i += stride) p[i] = z;
}

// One workgroup = one head x one 64-key tile of the destination.  Copies the rows of K that fall into the tile and
// writes the matching part of the transposed V tile (through LDS).  Only keys in [key0, key0+n) are touched: a tile
// shared with a neighbouring slot keeps the neighbour's keys.
template <int D>
__global__ void __launch_bounds__(256) lvx_pack_kv_kernel(const bf16_t *__restrict__ k, const bf16_t *__restrict__ v, int64_t ld,
                                                          int n, int cap, int key0, int tile0, bf16_t *__restrict__ kp,
                                                          bf16_t *__restrict__ vtp, int64_t batch_stride_src, int64_t batch_stride_dst) {
    // blockIdx.z: independent row set / packed array (the context values of several layers in one launch)
    if (k != nullptr) k += (size_t)blockIdx.z * batch_stride_src;
    v += (size_t)blockIdx.z * batch_stride_src;
    kp += (size_t)blockIdx.z * batch_stride_dst;
    vtp += (size_t)blockIdx.z * batch_stride_dst;
    constexpr int KT = LVX_KEY_TILE;
    constexpr int CPR = D / 8;        // 16-byte chunks per row
    constexpr int LDS_LD = D + 8;     // padded row, keeps 16-byte alignment
    __shared__ __attribute__((aligned(16))) bf16_t vs[KT * LDS_LD];

    const int tile = tile0 + blockIdx.x;
    const int h = blockIdx.y;
    const int tid = threadIdx.x;
    const int key_lo = tile * KT;
    const int n_tiles = cap / KT;

    for (int g = tid; g < KT * CPR; g += 256) {
        const int r = g / CPR, c = g % CPR;
        const int key = key_lo + r;
        const int src = key - key0;
        uint4 val = make_uint4(0, 0, 0, 0);
        if (src >= 0 && src < n) {
            const size_t so = (size_t)src * ld + (size_t)h * D + c * 8;
            if (k != nullptr) *reinterpret_cast<uint4 *>(kp + ((size_t)h * cap + key) * D + c * 8) = *reinterpret_cast<const uint4 *>(k + so);
            val = *reinterpret_cast<const uint4 *>(v + so);
        }
        *reinterpret_cast<uint4 *>(&vs[r * LDS_LD + c * 8]) = val;
    }
    __syncthreads();
    bf16_t *vt_tile = vtp + ((size_t)h * n_tiles + tile) * (size_t)D * KT;
    for (int g = tid; g < D * (KT / 8); g += 256) {
        const int d = g / (KT / 8), kc = g % (KT / 8);
        const int lo = key_lo + kc * 8 - key0;  // source index of the first of 8 keys
        if (lo + 7 < 0 || lo >= n) continue;
        bf16_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = vs[(kc * 8 + j) * LDS_LD + d];
        bf16_t *dst = vt_tile + (size_t)d * KT + kc * 8;
        if (lo >= 0 && lo + 7 < n) {
            uint4 o;
            o.x = e[0] | ((uint32_t)e[1] << 16);
            o.y = e[2] | ((uint32_t)e[3] << 16);
            o.z = e[4] | ((uint32_t)e[5] << 16);
            o.w = e[6] | ((uint32_t)e[7] << 16);
            *reinterpret_cast<uint4 *>(dst) = o;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (lo + j >= 0 && lo + j < n) dst[j] = e[j];
        }
    }
}

// Inverse of the pack: thread = (key, head, 16-byte chunk).  Check / off-load path, not tuned.
template <int D>
__global__ void __launch_bounds__(256) lvx_gather_kv_kernel(const bf16_t *__restrict__ kp, const bf16_t *__restrict__ vtp, int cap,
                                                            int H, int first_key, int n_keys, bf16_t *__restrict__ k_out,
                                                            bf16_t *__restrict__ v_out, int64_t ld) {
    constexpr int KT = LVX_KEY_TILE;
    constexpr int CPR = D / 8;
    const size_t total = (size_t)n_keys * H * CPR;
    const int n_tiles = cap / KT;
    for (size_t g = (size_t)blockIdx.x * 256 + threadIdx.x; g < total; g += (size_t)gridDim.x * 256) {
        const int c = (int)(g % CPR);
        const int h = (int)((g / CPR) % H);
        const int r = (int)(g / ((size_t)CPR * H));
        const int key = first_key + r;
        const size_t oo = (size_t)r * ld + (size_t)h * D + c * 8;
        *reinterpret_cast<uint4 *>(k_out + oo) = *reinterpret_cast<const uint4 *>(kp + ((size_t)h * cap + key) * D + c * 8);
        const bf16_t *vt_tile = vtp + ((size_t)h * n_tiles + key / KT) * (size_t)D * KT;
#pragma unroll
        for (int j = 0; j < 8; ++j) v_out[oo + j] = vt_tile[(size_t)(c * 8 + j) * KT + key % KT];
    }
}

// 8 elements per thread: out = bf16(x + dt * h), h fp32, x bf16 or absent
__global__ void __launch_bounds__(256) lvx_euler_kernel(const uint4 *x, const float4 *__restrict__ h, float dt, uint4 *out, size_t n8) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        uint4 a = make_uint4(0, 0, 0, 0);
        if (x != nullptr) a = x[i];
        const float4 h0 = h[2 * i], h1 = h[2 * i + 1];
        uint4 o;
        o.x = pack_bf16x2(bf16_lo(a.x) + dt * h0.x, bf16_hi(a.x) + dt * h0.y);
        o.y = pack_bf16x2(bf16_lo(a.y) + dt * h0.z, bf16_hi(a.y) + dt * h0.w);
        o.z = pack_bf16x2(bf16_lo(a.z) + dt * h1.x, bf16_hi(a.z) + dt * h1.y);
        o.w = pack_bf16x2(bf16_lo(a.w) + dt * h1.z, bf16_hi(a.w) + dt * h1.w);
        out[i] = o;
    }
}

__global__ void __launch_bounds__(256) lvx_widen_kernel(const uint4 *__restrict__ src, float4 *__restrict__ dst, size_t n8) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        const uint4 a = src[i];
        dst[2 * i] = make_float4(bf16_lo(a.x), bf16_hi(a.x), bf16_lo(a.y), bf16_hi(a.y));
        dst[2 * i + 1] = make_float4(bf16_lo(a.z), bf16_hi(a.z), bf16_lo(a.w), bf16_hi(a.w));
    }
}

// bf16 rows [n_rows][ld_src] -> fp32 rows [n_rows][ld_dst], 8 elements per thread (exact widening)
__global__ void __launch_bounds__(256) lvx_widen_rows_kernel(const bf16_t *__restrict__ src, int64_t ld_src, float *__restrict__ dst,
                                                             int64_t ld_dst, int n_rows, int chunks_per_row) {
    const size_t total = (size_t)n_rows * chunks_per_row;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t r = i / chunks_per_row, c = i % chunks_per_row;
        const uint4 a = reinterpret_cast<const uint4 *>(src + r * ld_src)[c];
        float4 *o = reinterpret_cast<float4 *>(dst + r * ld_dst) + 2 * c;
        o[0] = make_float4(bf16_lo(a.x), bf16_hi(a.x), bf16_lo(a.y), bf16_hi(a.y));
        o[1] = make_float4(bf16_lo(a.z), bf16_hi(a.z), bf16_lo(a.w), bf16_hi(a.w));
    }
}

__global__ void __launch_bounds__(256) lvx_copy_rows_kernel(const bf16_t *__restrict__ src, int64_t ld_src, bf16_t *__restrict__ dst,
                                                            int64_t ld_dst, int n_rows, int chunks_per_row) {
    const size_t total = (size_t)n_rows * chunks_per_row;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t r = i / chunks_per_row, c = i % chunks_per_row;
        reinterpret_cast<uint4 *>(dst + r * ld_dst)[c] = reinterpret_cast<const uint4 *>(src + r * ld_src)[c];
    }
}

static int grid_for(size_t n_items) {
    size_t g = (n_items + 255) / 256;
    if (g > 256 * 32) g = 256 * 32;
    if (g == 0) g = 1;
    return (int)g;
}

lvx_status_t lvx_launch_euler(const bf16_t *x, const float *h, float dt, bf16_t *out, size_t n_elems, hipStream_t stream) {
    const size_t n8 = n_elems / 8;
    hipLaunchKernelGGL(lvx_euler_kernel, dim3(grid_for(n8)), dim3(256), 0, stream, (const uint4 *)x, (const float4 *)h, dt, (uint4 *)out, n8);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

lvx_status_t lvx_launch_widen(const bf16_t *src, float *dst, size_t n_elems, hipStream_t stream) {
    const size_t n8 = n_elems / 8;
    hipLaunchKernelGGL(lvx_widen_kernel, dim3(grid_for(n8)), dim3(256), 0, stream, (const uint4 *)src, (float4 *)dst, n8);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

lvx_status_t lvx_launch_copy_rows(const bf16_t *src, int64_t ld_src, bf16_t *dst, int64_t ld_dst, int n_rows, int row_elems,
                                  hipStream_t stream) {
    if (n_rows == 0) return LVX_OK;
    const size_t total = (size_t)n_rows * (row_elems / 8);
    hipLaunchKernelGGL(lvx_copy_rows_kernel, dim3(grid_for(total)), dim3(256), 0, stream, src, ld_src, dst, ld_dst, n_rows, row_elems / 8);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

lvx_status_t lvx_launch_widen_rows(const bf16_t *src, int64_t ld_src, float *dst, int64_t ld_dst, int n_rows, int row_elems,
                                   hipStream_t stream) {
    if (n_rows == 0) return LVX_OK;
    const size_t total = (size_t)n_rows * (row_elems / 8);
    hipLaunchKernelGGL(lvx_widen_rows_kernel, dim3(grid_for(total)), dim3(256), 0, stream, src, ld_src, dst, ld_dst, n_rows, row_elems / 8);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

lvx_status_t lvx_launch_fill_zero(void *dst, size_t bytes, hipStream_t stream) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return LVX_OK;
    hipLaunchKernelGGL(lvx_fill_zero_kernel, dim3(grid_for(n16)), dim3(256), 0, stream, (uint4 *)dst, n16);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

lvx_status_t lvx_launch_pack_kv(const bf16_t *k, const bf16_t *v, int64_t ld, int n, int H, int D, int cap, int key0,
                                bf16_t *k_packed, bf16_t *vt_packed, hipStream_t stream, int n_batch, int64_t batch_stride_src,
                                int64_t batch_stride_dst) {
    if (n <= 0 || n_batch <= 0) return LVX_OK;
    const int tile0 = key0 / LVX_KEY_TILE;
    const int tile1 = (key0 + n - 1) / LVX_KEY_TILE;
    dim3 grid(tile1 - tile0 + 1, H, n_batch);
    if (D == 128)
        hipLaunchKernelGGL(lvx_pack_kv_kernel<128>, grid, dim3(256), 0, stream, k, v, ld, n, cap, key0, tile0, k_packed, vt_packed,
                           batch_stride_src, batch_stride_dst);
    else if (D == 64)
        hipLaunchKernelGGL(lvx_pack_kv_kernel<64>, grid, dim3(256), 0, stream, k, v, ld, n, cap, key0, tile0, k_packed, vt_packed,
                           batch_stride_src, batch_stride_dst);
    else
        return lvx_fail(LVX_ERR_UNSUPPORTED, "head_dim %d not supported (64 or 128)", D);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

// ------------------------------------------------------------------------------------------------ host logic
static lvx_status_t check_desc(const lvx_cache_desc_t *d) {
    LVX_REQUIRE(d != nullptr, LVX_ERR_INVALID_ARG, "cache descriptor is NULL");
    LVX_REQUIRE(d->n_layers > 0 && d->n_heads > 0 && d->frame_h > 0 && d->frame_w > 0 && d->chunk_frames > 0 &&
                    d->window_chunks >= 0 && d->sink_frames >= 0,
                LVX_ERR_SHAPE, "cache descriptor has a non-positive size");
    LVX_REQUIRE(d->head_dim == 64 || d->head_dim == 128, LVX_ERR_UNSUPPORTED, "head_dim %d not supported (64 or 128)", d->head_dim);
    LVX_REQUIRE(d->window_chunks + 1 <= LVX_MAX_SLOTS, LVX_ERR_UNSUPPORTED, "window_chunks+1 exceeds %d slots", LVX_MAX_SLOTS);
    const int64_t cap = (int64_t)d->frame_h * d->frame_w * ((int64_t)d->sink_frames + (int64_t)d->chunk_frames * (d->window_chunks + 1));
    LVX_REQUIRE(cap < (1ll << 30), LVX_ERR_SHAPE, "cache too large: %lld keys per head", (long long)cap);
    return LVX_OK;
}

static int cap_keys_of(const lvx_cache_desc_t *d) {
    const int fk = d->frame_h * d->frame_w;
    const int total = fk * (d->sink_frames + d->chunk_frames * (d->window_chunks + 1));
    return (total + LVX_KEY_TILE - 1) / LVX_KEY_TILE * LVX_KEY_TILE;
}

extern "C" size_t lvx_kvcache_bytes(const lvx_cache_desc_t *desc) {
    if (check_desc(desc) != LVX_OK) return 0;
    return (size_t)2 * sizeof(bf16_t) * desc->n_layers * desc->n_heads * (size_t)cap_keys_of(desc) * desc->head_dim;
}

extern "C" lvx_status_t lvx_ring_slot(const lvx_cache_desc_t *desc, int64_t chunk_index, lvx_slot_info_t *out) {
    lvx_status_t st = check_desc(desc);
    if (st != LVX_OK) return st;
    LVX_REQUIRE(out != nullptr, LVX_ERR_INVALID_ARG, "out is NULL");
    LVX_REQUIRE(chunk_index >= 0, LVX_ERR_INVALID_ARG, "chunk_index %lld is negative", (long long)chunk_index);
    const int n_slots = desc->window_chunks + 1;
    const int fk = desc->frame_h * desc->frame_w;
    const int sink_keys = fk * desc->sink_frames, chunk_keys = fk * desc->chunk_frames;
    out->slot = (int32_t)(chunk_index % n_slots);
    out->evicted_chunk = chunk_index >= n_slots ? chunk_index - n_slots : -1;
    out->n_valid_chunks = (int32_t)(chunk_index + 1 < n_slots ? chunk_index + 1 : n_slots);
    out->key_offset = sink_keys + out->slot * chunk_keys;
    out->key_count = sink_keys + out->n_valid_chunks * chunk_keys;
    return LVX_OK;
}

extern "C" lvx_status_t lvx_kvcache_init(const lvx_cache_desc_t *desc, void *dev_storage, size_t bytes, lvx_stream_t stream,
                                         lvx_kvcache_t **out) {
    lvx_status_t st = check_desc(desc);
    if (st != LVX_OK) return st;
    LVX_REQUIRE(out != nullptr, LVX_ERR_INVALID_ARG, "out handle pointer is NULL");
    LVX_REQUIRE(dev_storage != nullptr, LVX_ERR_INVALID_ARG, "dev_storage is NULL");
    LVX_REQUIRE((((uintptr_t)dev_storage) & 255u) == 0, LVX_ERR_INVALID_ARG, "dev_storage must be 256-byte aligned");
    const size_t need = lvx_kvcache_bytes(desc);
    LVX_REQUIRE(bytes >= need, LVX_ERR_SHAPE, "cache storage too small: %zu bytes given, %zu needed", bytes, need);

    lvx_kvcache *c = new (std::nothrow) lvx_kvcache;
    LVX_REQUIRE(c != nullptr, LVX_ERR_INVALID_ARG, "out of host memory");
    c->desc = *desc;
    const int fk = desc->frame_h * desc->frame_w;
    c->sink_keys = fk * desc->sink_frames;
    c->chunk_keys = fk * desc->chunk_frames;
    c->n_slots = desc->window_chunks + 1;
    c->cap_keys = cap_keys_of(desc);
    c->layer_k_elems = (size_t)desc->n_heads * c->cap_keys * desc->head_dim;
    c->k_base = (bf16_t *)dev_storage;
    c->vt_base = c->k_base + c->layer_k_elems * desc->n_layers;
    c->state = new (std::nothrow) lvx_ring_state_t[desc->n_layers];
    if (!c->state) {
        delete c;
        return lvx_fail(LVX_ERR_INVALID_ARG, "out of host memory");
    }
    c->sink_src = nullptr;
    c->sink_t = new (std::nothrow) int32_t[desc->n_layers];
    if (!c->sink_t) {
        delete[] c->state;
        delete c;
        return lvx_fail(LVX_ERR_INVALID_ARG, "out of host memory");
    }
    for (int l = 0; l < desc->n_layers; ++l) c->sink_t[l] = LVX_SINK_STATIC;
    for (int l = 0; l < desc->n_layers; ++l) {
        lvx_ring_state_t &s = c->state[l];
        memset(&s, 0, sizeof(s));
        s.last_chunk = -1;
        s.n_slots = c->n_slots;
        s.key_count = 0;
        for (int i = 0; i < LVX_MAX_SLOTS; ++i) s.slot_chunk[i] = -1;
    }
    const size_t n16 = need / 16;
    hipLaunchKernelGGL(lvx_fill_zero_kernel, dim3(grid_for(n16)), dim3(256), 0, (hipStream_t)stream, (uint4 *)dev_storage, n16);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        delete[] c->state;
        delete[] c->sink_t;
        delete c;
        return lvx_fail(LVX_ERR_HIP, "zero fill launch: %s", hipGetErrorString(e));
    }
    *out = c;
    return LVX_OK;
}

extern "C" lvx_status_t lvx_kvcache_destroy(lvx_kvcache_t *cache) {
    LVX_REQUIRE(cache != nullptr, LVX_ERR_INVALID_ARG, "cache handle is NULL");
    delete[] cache->state;
    delete[] cache->sink_t;
    delete cache;
    return LVX_OK;
}

static lvx_status_t check_layer_and_rows(const lvx_kvcache *c, int32_t layer, const void *k, const void *v, int64_t ld) {
    LVX_REQUIRE(c != nullptr, LVX_ERR_INVALID_ARG, "cache handle is NULL");
    LVX_REQUIRE(layer >= 0 && layer < c->desc.n_layers, LVX_ERR_INVALID_ARG, "layer %d out of range [0,%d)", layer, c->desc.n_layers);
    LVX_REQUIRE(k != nullptr && v != nullptr, LVX_ERR_INVALID_ARG, "K or V pointer is NULL");
    LVX_REQUIRE(lvx_aligned16(k) && lvx_aligned16(v), LVX_ERR_INVALID_ARG, "K and V must be 16-byte aligned");
    LVX_REQUIRE(ld >= (int64_t)c->desc.n_heads * c->desc.head_dim && ld % 8 == 0, LVX_ERR_SHAPE,
                "row stride %lld must be a multiple of 8 and >= n_heads*head_dim", (long long)ld);
    return LVX_OK;
}

extern "C" lvx_status_t lvx_kvcache_set_sink(lvx_kvcache_t *c, int32_t layer, const void *dev_k, const void *dev_v, int64_t ld,
                                             lvx_stream_t stream) {
    lvx_status_t st = check_layer_and_rows(c, layer, dev_k, dev_v, ld);
    if (st != LVX_OK) return st;
    LVX_REQUIRE(c->sink_keys > 0, LVX_ERR_STATE, "this cache has no sink segment (sink_frames = 0)");
    st = lvx_launch_pack_kv((const bf16_t *)dev_k, (const bf16_t *)dev_v, ld, c->sink_keys, c->desc.n_heads, c->desc.head_dim,
                            c->cap_keys, 0, (bf16_t *)lvx_cache_k(c, layer), (bf16_t *)lvx_cache_vt(c, layer), (hipStream_t)stream);
    if (st != LVX_OK) return st;
    lvx_ring_state_t &s = c->state[layer];
    s.sink_set = 1;
    s.key_count = c->sink_keys + s.n_valid_chunks * c->chunk_keys;
    c->sink_t[layer] = LVX_SINK_STATIC;
    return LVX_OK;
}

// ---- Rolling RoPE / adaptive attention sink (paper Sec. 3.3, Appendix D) ------------------------------------------
extern "C" size_t lvx_sink_source_bytes(const lvx_cache_desc_t *desc) {
    if (check_desc(desc) != LVX_OK) return 0;
    return (size_t)desc->n_layers * desc->frame_h * desc->frame_w * desc->sink_frames * desc->n_heads * desc->head_dim * sizeof(float);
}

extern "C" lvx_status_t lvx_kvcache_attach_sink_source(lvx_kvcache_t *c, void *dev_storage, size_t bytes) {
    LVX_REQUIRE(c != nullptr, LVX_ERR_INVALID_ARG, "cache handle is NULL");
    LVX_REQUIRE(c->sink_keys > 0, LVX_ERR_STATE, "this cache has no sink segment (sink_frames = 0)");
    LVX_REQUIRE(dev_storage != nullptr && (((uintptr_t)dev_storage) & 255u) == 0, LVX_ERR_INVALID_ARG,
                "sink source storage must be non-NULL and 256-byte aligned");
    const size_t need = lvx_sink_source_bytes(&c->desc);
    LVX_REQUIRE(bytes >= need, LVX_ERR_SHAPE, "sink source storage too small: %zu bytes given, %zu needed", bytes, need);
    c->sink_src = (float *)dev_storage;
    return LVX_OK;
}

// Shared tail of lvx_kvcache_reset_sink and of the sink warm-up: the layer's fp32 source is already in place; V goes to its
// final place, the K rows of the sink segment stay as they are until the next rotation overwrites them.
lvx_status_t lvx_sink_install_values(lvx_kvcache *c, int layer, const bf16_t *v, int64_t ld, hipStream_t stream) {
    LVX_TRY(lvx_launch_pack_kv(nullptr, v, ld, c->sink_keys, c->desc.n_heads, c->desc.head_dim, c->cap_keys, 0,
                               (bf16_t *)lvx_cache_k(c, layer), (bf16_t *)lvx_cache_vt(c, layer), stream));
    lvx_ring_state_t &s = c->state[layer];
    s.sink_set = 1;
    s.key_count = c->sink_keys + s.n_valid_chunks * c->chunk_keys;
    c->sink_t[layer] = LVX_SINK_STALE;
    return LVX_OK;
}

extern "C" lvx_status_t lvx_kvcache_reset_sink(lvx_kvcache_t *c, int32_t layer, const void *dev_k_src, const void *dev_v, int64_t ld,
                                               lvx_stream_t stream) {
    lvx_status_t st = check_layer_and_rows(c, layer, dev_k_src, dev_v, ld);
    if (st != LVX_OK) return st;
    LVX_REQUIRE(c->sink_keys > 0, LVX_ERR_STATE, "this cache has no sink segment (sink_frames = 0)");
    LVX_REQUIRE(c->sink_src != nullptr, LVX_ERR_STATE, "no sink source storage attached (lvx_kvcache_attach_sink_source)");
    const int d = c->desc.n_heads * c->desc.head_dim;
    // the source is kept in fp32 (exact widening of the bf16 keys given here; the sink warm-up stores un-rounded fp32 keys)
    LVX_TRY(lvx_launch_widen_rows((const bf16_t *)dev_k_src, ld, c->sink_src + (size_t)layer * c->sink_keys * d, d, c->sink_keys, d,
                                  (hipStream_t)stream));
    return lvx_sink_install_values(c, layer, (const bf16_t *)dev_v, ld, (hipStream_t)stream);
}

extern "C" lvx_status_t lvx_sink_rope_update(lvx_kvcache_t *c, const lvx_rope_desc_t *rope, int32_t layer, int32_t t_sink,
                                             lvx_stream_t stream) {
    LVX_REQUIRE(c != nullptr && rope != nullptr, LVX_ERR_INVALID_ARG, "cache handle or rope descriptor is NULL");
    LVX_REQUIRE(layer >= -1 && layer < c->desc.n_layers, LVX_ERR_INVALID_ARG, "layer %d out of range [-1,%d)", layer, c->desc.n_layers);
    LVX_REQUIRE(t_sink >= 0, LVX_ERR_INVALID_ARG, "t_sink must be non-negative");
    LVX_REQUIRE(rope->n_heads == c->desc.n_heads && rope->head_dim == c->desc.head_dim && rope->frame_h == c->desc.frame_h &&
                    rope->frame_w == c->desc.frame_w && rope->apply_rope,
                LVX_ERR_SHAPE, "rope descriptor disagrees with the cache (heads / head_dim / frame size) or has apply_rope = 0");
    LVX_REQUIRE(c->sink_src != nullptr, LVX_ERR_STATE, "no sink source storage attached (lvx_kvcache_attach_sink_source)");
    const int l0 = layer < 0 ? 0 : layer, l1 = layer < 0 ? c->desc.n_layers : layer + 1;
    for (int l = l0; l < l1; ++l)
        LVX_REQUIRE(c->sink_t[l] != LVX_SINK_STATIC, LVX_ERR_STATE, "layer %d has no sink source (lvx_kvcache_reset_sink / lvx_sink_prefill)", l);
    const int d = c->desc.n_heads * c->desc.head_dim;
    lvx_status_t st;
    {
        lvx_prof_scope_t ps(LVX_PROF_SINK_ROPE, (hipStream_t)stream);
        st = lvx_launch_rope_to_packed_k(rope, c->sink_src + (size_t)l0 * c->sink_keys * d, d, c->sink_keys, t_sink,
                                         (bf16_t *)lvx_cache_k(c, l0), c->cap_keys, l1 - l0, (int64_t)c->sink_keys * d,
                                         (int64_t)c->layer_k_elems, (hipStream_t)stream);
    }
    if (st != LVX_OK) return st;
    for (int l = l0; l < l1; ++l) c->sink_t[l] = t_sink;
    return LVX_OK;
}

extern "C" lvx_status_t lvx_kvcache_get_sink_index(const lvx_kvcache_t *c, int32_t layer, int32_t *out) {
    LVX_REQUIRE(c != nullptr && out != nullptr, LVX_ERR_INVALID_ARG, "cache handle or out is NULL");
    LVX_REQUIRE(layer >= 0 && layer < c->desc.n_layers, LVX_ERR_INVALID_ARG, "layer %d out of range [0,%d)", layer, c->desc.n_layers);
    *out = c->sink_t[layer];
    return LVX_OK;
}

extern "C" lvx_status_t lvx_kvcache_set_sink_index(lvx_kvcache_t *c, int32_t layer, int32_t t_sink) {
    LVX_REQUIRE(c != nullptr, LVX_ERR_INVALID_ARG, "cache handle is NULL");
    LVX_REQUIRE(layer >= 0 && layer < c->desc.n_layers, LVX_ERR_INVALID_ARG, "layer %d out of range [0,%d)", layer, c->desc.n_layers);
    LVX_REQUIRE(t_sink >= LVX_SINK_STATIC, LVX_ERR_INVALID_ARG, "t_sink %d: -2 (static), -1 (stale) or a temporal index", t_sink);
    LVX_REQUIRE(t_sink == LVX_SINK_STATIC || c->sink_src != nullptr, LVX_ERR_STATE, "no sink source storage attached");
    c->sink_t[layer] = t_sink;
    return LVX_OK;
}

extern "C" lvx_status_t lvx_kvcache_gather_sink_source(const lvx_kvcache_t *c, int32_t layer, void *dev_k_src_out, int64_t ld,
                                                       lvx_stream_t stream) {
    LVX_REQUIRE(c != nullptr && dev_k_src_out != nullptr, LVX_ERR_INVALID_ARG, "cache handle or output is NULL");
    LVX_REQUIRE(layer >= 0 && layer < c->desc.n_layers, LVX_ERR_INVALID_ARG, "layer %d out of range [0,%d)", layer, c->desc.n_layers);
    LVX_REQUIRE(c->sink_src != nullptr && c->sink_t[layer] != LVX_SINK_STATIC, LVX_ERR_STATE, "layer %d has no sink source", layer);
    const int d = c->desc.n_heads * c->desc.head_dim;
    LVX_REQUIRE(lvx_aligned16(dev_k_src_out) && ld >= d && ld % 8 == 0, LVX_ERR_INVALID_ARG, "output must be 16-byte aligned, ld a multiple of 8 >= d");
    // fp32 rows copied as pairs of bf16-sized elements
    return lvx_launch_copy_rows((const bf16_t *)(c->sink_src + (size_t)layer * c->sink_keys * d), 2 * (int64_t)d, (bf16_t *)dev_k_src_out,
                                2 * ld, c->sink_keys, 2 * d, (hipStream_t)stream);
}

lvx_status_t lvx_cache_append_begin(const lvx_kvcache *c, int layer, int64_t chunk_index, lvx_slot_info_t *info) {
    const lvx_ring_state_t &s = c->state[layer];
    LVX_REQUIRE(chunk_index == s.last_chunk + 1, LVX_ERR_STATE, "layer %d expects chunk %lld, got %lld", layer,
                (long long)(s.last_chunk + 1), (long long)chunk_index);
    LVX_REQUIRE(c->sink_keys == 0 || s.sink_set, LVX_ERR_STATE, "layer %d: sink not set before the first append", layer);
    return lvx_ring_slot(&c->desc, chunk_index, info);
}

void lvx_cache_append_commit(lvx_kvcache *c, int layer, int64_t chunk_index, const lvx_slot_info_t *info) {
    lvx_ring_state_t &s = c->state[layer];
    s.last_chunk = chunk_index;
    s.slot_chunk[info->slot] = chunk_index;
    s.n_valid_chunks = info->n_valid_chunks;
    s.key_count = info->key_count;
}

extern "C" lvx_status_t lvx_chunk_append_evict(lvx_kvcache_t *c, int32_t layer, const void *dev_k, const void *dev_v, int64_t ld,
                                               int64_t chunk_index, lvx_slot_info_t *out, lvx_stream_t stream) {
    lvx_status_t st = check_layer_and_rows(c, layer, dev_k, dev_v, ld);
    if (st != LVX_OK) return st;
    lvx_slot_info_t info;
    st = lvx_cache_append_begin(c, layer, chunk_index, &info);
    if (st != LVX_OK) return st;
    st = lvx_launch_pack_kv((const bf16_t *)dev_k, (const bf16_t *)dev_v, ld, c->chunk_keys, c->desc.n_heads, c->desc.head_dim,
                            c->cap_keys, info.key_offset, (bf16_t *)lvx_cache_k(c, layer), (bf16_t *)lvx_cache_vt(c, layer),
                            (hipStream_t)stream);
    if (st != LVX_OK) return st;
    lvx_cache_append_commit(c, layer, chunk_index, &info);
    if (out) *out = info;
    return LVX_OK;
}

extern "C" lvx_status_t lvx_kvcache_get_state(const lvx_kvcache_t *c, int32_t layer, lvx_ring_state_t *out) {
    LVX_REQUIRE(c != nullptr && out != nullptr, LVX_ERR_INVALID_ARG, "cache handle or out is NULL");
    LVX_REQUIRE(layer >= 0 && layer < c->desc.n_layers, LVX_ERR_INVALID_ARG, "layer %d out of range [0,%d)", layer, c->desc.n_layers);
    *out = c->state[layer];
    return LVX_OK;
}

extern "C" lvx_status_t lvx_kvcache_set_state(lvx_kvcache_t *c, int32_t layer, const lvx_ring_state_t *in) {
    LVX_REQUIRE(c != nullptr && in != nullptr, LVX_ERR_INVALID_ARG, "cache handle or state is NULL");
    LVX_REQUIRE(layer >= 0 && layer < c->desc.n_layers, LVX_ERR_INVALID_ARG, "layer %d out of range [0,%d)", layer, c->desc.n_layers);
    LVX_REQUIRE(in->n_slots == c->n_slots, LVX_ERR_SHAPE, "state has %d slots, cache has %d", in->n_slots, c->n_slots);
    LVX_REQUIRE(in->last_chunk >= -1, LVX_ERR_STATE, "state.last_chunk %lld invalid", (long long)in->last_chunk);
    // the bookkeeping must be what the ring arithmetic yields for last_chunk
    const int64_t n_valid = in->last_chunk + 1 < c->n_slots ? in->last_chunk + 1 : c->n_slots;
    LVX_REQUIRE(in->n_valid_chunks == n_valid, LVX_ERR_STATE, "state.n_valid_chunks %d inconsistent with last_chunk", in->n_valid_chunks);
    LVX_REQUIRE(in->key_count == (in->sink_set ? c->sink_keys : 0) + (int)n_valid * c->chunk_keys, LVX_ERR_STATE,
                "state.key_count %d inconsistent", in->key_count);
    for (int sl = 0; sl < c->n_slots; ++sl) {
        int64_t want = -1;
        for (int64_t j = in->last_chunk; j >= 0 && j > in->last_chunk - c->n_slots; --j)
            if (j % c->n_slots == sl) want = j;
        LVX_REQUIRE(in->slot_chunk[sl] == want, LVX_ERR_STATE, "state.slot_chunk[%d] = %lld, ring arithmetic gives %lld", sl,
                    (long long)in->slot_chunk[sl], (long long)want);
    }
    c->state[layer] = *in;
    return LVX_OK;
}

extern "C" lvx_status_t lvx_kvcache_gather(const lvx_kvcache_t *c, int32_t layer, int32_t first_key, int32_t n_keys, void *dev_k_out,
                                           void *dev_v_out, int64_t ld, lvx_stream_t stream) {
    lvx_status_t st = check_layer_and_rows(c, layer, dev_k_out, dev_v_out, ld);
    if (st != LVX_OK) return st;
    LVX_REQUIRE(first_key >= 0 && n_keys >= 0 && (int64_t)first_key + n_keys <= c->cap_keys, LVX_ERR_SHAPE,
                "key range [%d,%d) outside the cache (%d keys)", first_key, first_key + n_keys, c->cap_keys);
    return lvx_launch_gather_kv(lvx_cache_k(c, layer), lvx_cache_vt(c, layer), c->cap_keys, c->desc.n_heads, c->desc.head_dim, first_key, n_keys,
                                (bf16_t *)dev_k_out, (bf16_t *)dev_v_out, ld, (hipStream_t)stream);
}

lvx_status_t lvx_launch_gather_kv(const bf16_t *k_packed, const bf16_t *vt_packed, int cap, int H, int D, int first_key, int n_keys,
                                  bf16_t *k_out, bf16_t *v_out, int64_t ld, hipStream_t stream) {
    if (n_keys == 0) return LVX_OK;
    const size_t total = (size_t)n_keys * H * (D / 8);
    if (D == 128)
        hipLaunchKernelGGL(lvx_gather_kv_kernel<128>, dim3(grid_for(total)), dim3(256), 0, stream, k_packed, vt_packed, cap, H, first_key, n_keys,
                           k_out, v_out, ld);
    else if (D == 64)
        hipLaunchKernelGGL(lvx_gather_kv_kernel<64>, dim3(grid_for(total)), dim3(256), 0, stream, k_packed, vt_packed, cap, H, first_key, n_keys,
                           k_out, v_out, ld);
    else
        return lvx_fail(LVX_ERR_UNSUPPORTED, "head_dim %d not supported (64 or 128)", D);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}
