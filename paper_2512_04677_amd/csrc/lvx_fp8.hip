// FP8 (E4M3) linears with per-tensor dynamic scaling (paper Appendix C, "FP8 Quantization": every linear projection of the
// DiT takes FP8 operands; embeddings and heads, which are outside the stage, do not).
//
//   amax   = max |x| over the whole tensor                                   (lvx_fp8_amax_kernel, atomic max on the bit pattern)
//   code   = E4M3(x * (448 / amax)), round to nearest even, saturating       (lvx_fp8_quant_kernel, v_cvt_pk_fp8_f32)
//   C      = (amax_a / 448) * (amax_w / 448) * (code_a . code_w)             (lvx_gemm_fp8_kernel, fp32 accumulate)
//
// The two scale factors and the product x * (448/amax) are formed in fp32: that product is what decides the 8-bit code.
// gfx950 converts to and multiplies the OCP form of E4M3 (bias 7, largest finite value 448, no infinities).
//
// The GEMM is the direct-to-LDS design of the bf16 kernel with one-byte elements: a 128 x 256 tile, 8 waves of 64 x 64,
// K walked in slabs of 128 elements (again 128-byte LDS rows, XOR-swizzled, three 48 KB stages), and
// v_mfma_f32_32x32x64_f8f6f4 (64 clocks for 131072 flop: twice the bf16 rate; the older 32x32x16 fp8 form runs at the bf16
// rate on this chip).  A fragment is 32 bytes per lane: row l%32, k = 32*(l/32) .. +31 of the 64-wide k-step.
#include "lvx_internal.h"

#include <mutex>

// Scratch of lvx_fp8_quantize_static: the amax slot array that lvx_fp8_quantize takes from its caller, here owned by the
// library.  One copy per GPU the library runs on, resident until the process ends.  In host code this name only stands for
// the symbol: the device address is resolved per device with hipGetSymbolAddress (static_scratch() below) and only that
// pointer is ever handed to a kernel.
static __device__ __align__(256) uint32_t scratch[LVX_AMAX_SLOTS];

namespace {

constexpr int GROUP_M = 8;
constexpr float E4M3_MAX = 448.0f;

constexpr int MAX_DEVICES = 64;
uint32_t *g_scratch_ptr[MAX_DEVICES];  // device address of `scratch` on each device, resolved on first use
std::mutex g_scratch_mutex;

// Device address of this device's copy of `scratch`.  No allocation: the array is part of the code object's data.
lvx_status_t static_scratch(uint32_t **out) {
    int dev = -1;
    LVX_CHECK_HIP(hipGetDevice(&dev));
    LVX_REQUIRE(dev >= 0 && dev < MAX_DEVICES, LVX_ERR_UNSUPPORTED, "device ordinal %d outside [0,%d)", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        LVX_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        LVX_REQUIRE(p != nullptr && (((uintptr_t)p) & 255u) == 0, LVX_ERR_HIP, "address of the static scratch array is NULL or misaligned");
        g_scratch_ptr[dev] = (uint32_t *)p;
    }
    *out = g_scratch_ptr[dev];
    return LVX_OK;
}

typedef __attribute__((__vector_size__(8 * sizeof(int)))) int i32x8_t;

// ---- quantisation ---------------------------------------------------------------------------------------------------
// amax_slots: LVX_AMAX_SLOTS fp32 bit patterns whose maximum is max|x| (non-negative floats order like their bit patterns),
// zeroed before the producers run.  Producers spread their atomic maxima over the slots (thousands of atomics on ONE address
// would serialise in L2 and cost more than the pass itself); the quantisation kernel reduces the slots.
__global__ void __launch_bounds__(256) lvx_fp8_amax_kernel(const bf16_t *__restrict__ x, int64_t ld, int rows, int chunks_per_row,
                                                           uint32_t *amax_slots) {
    const size_t total = (size_t)rows * chunks_per_row;
    uint32_t m = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t r = i / chunks_per_row, c = i % chunks_per_row;
        const uint4 v = reinterpret_cast<const uint4 *>(x + r * ld)[c];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t lo = w[e] & 0x7fffu, hi = (w[e] >> 16) & 0x7fffu;
            m = m > lo ? m : lo;
            m = m > hi ? m : hi;
        }
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)m, s);
        m = m > o ? m : o;
    }
    __shared__ uint32_t wave_max[4];
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = wave_max[0];
#pragma unroll
        for (int w = 1; w < 4; ++w) m = m > wave_max[w] ? m : wave_max[w];
        if (m != 0) atomicMax(amax_slots + (blockIdx.x & (LVX_AMAX_SLOTS - 1)), m << 16);
    }
}

// 16 bf16 -> 16 codes per thread; also publishes the dequantisation scale amax/448 (1 for an all-zero tensor)
// zero_slots (may be NULL): another slot array, not in use by any kernel in flight, that this kernel clears for the next
// producer (the arrays alternate, so no separate clearing launch is needed between quantisations).
__global__ void __launch_bounds__(256) lvx_fp8_quant_kernel(const bf16_t *__restrict__ x, int64_t ld, int rows, int chunks_per_row,
                                                            const uint32_t *__restrict__ amax_slots, uint32_t *__restrict__ zero_slots,
                                                            uint8_t *__restrict__ q, int64_t ldq, float *__restrict__ scale_out) {
    uint32_t mb = amax_slots[threadIdx.x & (LVX_AMAX_SLOTS - 1)];
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)mb, s);
        mb = mb > o ? mb : o;
    }
    if (zero_slots != nullptr && blockIdx.x == 0 && threadIdx.x < LVX_AMAX_SLOTS) zero_slots[threadIdx.x] = 0;
    const float amax = __uint_as_float(mb);
    const float inv = amax > 0.f ? E4M3_MAX / amax : 0.f;
    if (blockIdx.x == 0 && threadIdx.x == 0) *scale_out = amax > 0.f ? amax / E4M3_MAX : 1.0f;
    const size_t total = (size_t)rows * chunks_per_row;  // chunks of 16 elements
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t r = i / chunks_per_row, c = i % chunks_per_row;
        const uint4 *src = reinterpret_cast<const uint4 *>(x + r * ld) + 2 * c;
        const uint4 v0 = src[0], v1 = src[1];
        const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // |x * inv| <= 448 (1 + 2^-23): far below the midpoint to the next (non-existent) grid value, the clamp only
            // guards the conversion's out-of-range behaviour
            float a = fminf(fmaxf(bf16_lo(w[2 * e]) * inv, -E4M3_MAX), E4M3_MAX);
            float b = fminf(fmaxf(bf16_hi(w[2 * e]) * inv, -E4M3_MAX), E4M3_MAX);
            float c2 = fminf(fmaxf(bf16_lo(w[2 * e + 1]) * inv, -E4M3_MAX), E4M3_MAX);
            float d = fminf(fmaxf(bf16_hi(w[2 * e + 1]) * inv, -E4M3_MAX), E4M3_MAX);
            int p = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
            p = __builtin_amdgcn_cvt_pk_fp8_f32(c2, d, p, true);
            o[e] = (uint32_t)p;
        }
        *reinterpret_cast<uint4 *>(q + r * ldq + 16 * c) = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

int grid_for(size_t n_items) {
    size_t g = (n_items + 255) / 256;
    if (g > 256 * 16) g = 256 * 16;
    return (int)(g ? g : 1);
}

// ---- GEMM -------------------------------------------------------------------------------------------------------------
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
    lvx_gemm_fp8_kernel(const uint8_t *__restrict__ A, int64_t lda, const uint8_t *__restrict__ W, int64_t ldw,
                        const float *__restrict__ scale_a, const float *__restrict__ scale_w, bf16_t *C, int64_t ldc, int M, int N, int K,
                        const bf16_t *R, int64_t ldr, const float *__restrict__ gate, int tiles_m, int tiles_n, int per_xcd,
                        uint32_t *amax_slots) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int FM = WTM / 32, FN = WTN / 32;
    constexpr int ROW_B = 128;  // bytes = elements per LDS row = K extent of a slab
    constexpr int A_B = BM * ROW_B, STAGE_B = (BM + BN) * ROW_B;
    constexpr int NSTAGE = 3;
    constexpr int N_INSTR = (BM + BN) / 8;  // DMA wave-instructions per slab (8 rows each)
    static_assert(N_INSTR % NW == 0 && (BM / 8) % NW == 0, "DMA instructions must divide over the waves, A and W separately");
    constexpr int QPW = N_INSTR / NW;
    constexpr int A_Q = (BM / 8) / NW;

    __shared__ __attribute__((aligned(1024))) char lds[NSTAGE * STAGE_B];

    const int total = tiles_m * tiles_n;
    const int widx = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);  // consecutive ids go to consecutive XCDs
    if (widx >= total) return;
    const int band = widx / (GROUP_M * tiles_n);
    const int first_m = band * GROUP_M;
    const int band_m = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
    const int in_band = widx - band * GROUP_M * tiles_n;
    const int tm = first_m + in_band % band_m;
    const int tn = in_band / band_m;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // DMA instruction q of this wave covers stage rows 8*(wave + NW*q) .. +7 (A rows first, then W rows); rows past the
    // matrix edge are clamped (their results are never stored)
    uint32_t doff[QPW];
#pragma unroll
    for (int q = 0; q < QPW; ++q) {
        const int row_s = 8 * (wave + NW * q) + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row_s >> 1) & 7);
        if (q < A_Q) {
            int r = tm * BM + row_s;
            if (r > M - 1) r = M - 1;
            doff[q] = (uint32_t)((size_t)r * lda + chunk * 16);
        } else {
            int r = tn * BN + (row_s - BM);
            if (r > N - 1) r = N - 1;
            doff[q] = (uint32_t)((size_t)r * ldw + chunk * 16);
        }
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds_base + wave * 1024);
#define LVX8_DMA_ISSUE(stage_, kt_, q_)                                                                                      \
    lvx_dma16(reinterpret_cast<const char *>((q_) < A_Q ? (const void *)A : (const void *)W) + (size_t)(kt_) * ROW_B, doff[q_], \
              lds_wave + (uint32_t)((stage_) * STAGE_B + (q_) * NW * 1024))

    // fragment of k-step kk (64 elements): lane (l32, hh) reads row l32, bytes 64*kk + 32*hh .. +31 = 16-byte chunks
    // 4kk + 2hh and 4kk + 2hh + 1 at their swizzled positions
    const int swz = (l32 >> 1) & 7;
    const char *a_rd = lds + (wm * WTM + l32) * ROW_B;
    const char *w_rd = lds + A_B + (wn * WTN + l32) * ROW_B;
    i32x8_t af[2][FM], wf[2][FN];
#define LVX8_READ_ONE(dst_, base_)                                                                    \
    {                                                                                                 \
        const u32x4_t lo_ = *reinterpret_cast<const u32x4_t *>((base_) + c0_);                        \
        const u32x4_t hi_ = *reinterpret_cast<const u32x4_t *>((base_) + c1_);                        \
        dst_[0] = (int)lo_[0], dst_[1] = (int)lo_[1], dst_[2] = (int)lo_[2], dst_[3] = (int)lo_[3];   \
        dst_[4] = (int)hi_[0], dst_[5] = (int)hi_[1], dst_[6] = (int)hi_[2], dst_[7] = (int)hi_[3];   \
    }
#define LVX8_READ_FRAGS(stage_, kk_)                                                                  \
    {                                                                                                 \
        const int c0_ = (((kk_) * 4 + 2 * hh) ^ swz) * 16 + (stage_) * STAGE_B;                        \
        const int c1_ = (((kk_) * 4 + 2 * hh + 1) ^ swz) * 16 + (stage_) * STAGE_B;                    \
        _Pragma("unroll") for (int i = 0; i < FM; ++i) LVX8_READ_ONE(af[(kk_) & 1][i], a_rd + i * 32 * ROW_B); \
        _Pragma("unroll") for (int j = 0; j < FN; ++j) LVX8_READ_ONE(wf[(kk_) & 1][j], w_rd + j * 32 * ROW_B); \
    }
#define LVX8_MFMAS(kk_)                                                                                          \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) _Pragma("unroll") for (int j = 0; j < FN; ++j)                \
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(af[(kk_) & 1][i], wf[(kk_) & 1][j], acc[i][j], 0, 0, 0, 0, 0, 0);

    f32x16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // fp32 residual epilogue: this lane's part of the residual tile is fetched before the main loop and held in registers, so
    // that only the write is left for the end (all workgroups finish their tiles at the same time and would otherwise read
    // and write the residual with 256 CUs at once).  Rows / columns past the matrix edge are clamped (values unused).
    const int m0 = tm * BM + wm * WTM + 4 * hh, n0 = tn * BN + wn * WTN + l32;
    f32x16_t rres[FM][FN];
    if (EPI == LVX_EPI_RESID_GATE_F32) {
        const float *Rf = reinterpret_cast<const float *>(R);
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int col = n0 + j * 32 < N ? n0 + j * 32 : N - 1;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    int row = m0 + i * 32 + 8 * (e >> 2) + (e & 3);
                    row = row < M ? row : M - 1;
                    rres[i][j][e] = Rf[(size_t)row * ldr + col];
                }
        }
    }

    const int n_k = K / ROW_B;
    const int last = n_k - 1;
#pragma unroll
    for (int q = 0; q < QPW; ++q) LVX8_DMA_ISSUE(0, 0, q);
#pragma unroll
    for (int q = 0; q < QPW; ++q) LVX8_DMA_ISSUE(1, (last < 1 ? last : 1), q);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(QPW) : "memory");
    __syncthreads();
    LVX8_READ_FRAGS(0, 0);

    // Slab t is in stage t % 3.  Per slab: the first k-step's MFMAs run while the second k-step's fragments are read and the
    // DMA for slab t+2 is issued (into the stage that was last read during slab t-1, before that slab's barrier); then this
    // wave's DMA for slab t+1 must have landed, one workgroup barrier, and the second k-step's MFMAs run while k-step 0 of
    // slab t+1 is read.
    int cur = 0, nxt = 1, nx2 = 2;
    for (int t = 0; t < n_k; ++t) {
        const int kt_load = t + 2 < last ? t + 2 : last;
        LVX8_READ_FRAGS(cur, 1);
        __builtin_amdgcn_sched_barrier(0);
        LVX8_MFMAS(0);
#pragma unroll
        for (int q = 0; q < QPW; ++q) LVX8_DMA_ISSUE(nx2, kt_load, q);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(QPW) : "memory");
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        LVX8_READ_FRAGS(nxt, 0);
        __builtin_amdgcn_sched_barrier(0);
        LVX8_MFMAS(1);
        __builtin_amdgcn_sched_barrier(0);
        const int tmp = cur;
        cur = nxt;
        nxt = nx2;
        nx2 = tmp;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no DMA may still be in flight when the workgroup releases its LDS

    // Epilogue.  Accumulator register 4g+r of fragment (i,j) holds row m0 + 32i + 8g + r and column n0 + 32j.
    const float alpha = scale_a[0] * scale_w[0];
    uint32_t amax_b = 0;  // largest magnitude among the bf16 values this lane stores (bit pattern without sign)
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int n = n0 + j * 32;
        if (n >= N) continue;
        float gt = 1.f;
        if ((EPI == LVX_EPI_RESID_GATE || EPI == LVX_EPI_RESID_GATE_F32) && gate != nullptr) gt = gate[n];
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const size_t row0 = (size_t)(m0 + i * 32);
            bf16_t *cp = C + row0 * ldc + n;
            float *cpf = reinterpret_cast<float *>(C) + row0 * ldc + n;
            const bf16_t *rp = R + row0 * ldr + n;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int dm = 8 * (e >> 2) + (e & 3);
                if (m0 + i * 32 + dm >= M) continue;
                float v = acc[i][j][e] * alpha;
                if (EPI == LVX_EPI_GELU_TANH) v = gelu_tanh_f32(v);
                if (EPI == LVX_EPI_RESID_GATE) v = bf16_bits_to_f32(rp[(size_t)dm * ldr]) + gt * v;
                if (EPI == LVX_EPI_RESID_GATE_F32)
                    cpf[(size_t)dm * ldc] = rres[i][j][e] + gt * v;
                else {
                    const uint32_t b = pack_bf16x2(v, 0.f) & 0xffffu;
                    cp[(size_t)dm * ldc] = (bf16_t)b;
                    amax_b = amax_b > (b & 0x7fffu) ? amax_b : (b & 0x7fffu);
                }
            }
        }
    }
    // the output feeds another FP8 linear: hand its amax to that linear's quantisation
    if (amax_slots != nullptr) {
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)amax_b, s);
            amax_b = amax_b > o ? amax_b : o;
        }
        if (lane == 0 && amax_b != 0) atomicMax(amax_slots + ((widx * NW + wave) & (LVX_AMAX_SLOTS - 1)), amax_b << 16);
    }
}

}  // namespace

lvx_status_t lvx_launch_fp8_amax(const bf16_t *x, int64_t ld, int rows, int cols, uint32_t *amax_slots, hipStream_t stream) {
    if (rows == 0) return LVX_OK;
    int amax_grid = grid_for((size_t)rows * (cols / 8));
    if (amax_grid > 1024) amax_grid = 1024;  // 4 workgroups per CU, one atomic each
    hipLaunchKernelGGL(lvx_fp8_amax_kernel, dim3(amax_grid), dim3(256), 0, stream, x, ld, rows, cols / 8, amax_slots);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

lvx_status_t lvx_launch_fp8_quant(const bf16_t *x, int64_t ld, int rows, int cols, uint8_t *q, int64_t ldq, const uint32_t *amax_slots,
                                  uint32_t *zero_slots, float *scale, hipStream_t stream) {
    if (rows == 0) return LVX_OK;
    hipLaunchKernelGGL(lvx_fp8_quant_kernel, dim3(grid_for((size_t)rows * (cols / 16))), dim3(256), 0, stream, x, ld, rows, cols / 16,
                       amax_slots, zero_slots, q, ldq, scale);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

lvx_status_t lvx_launch_fp8_quantize(const bf16_t *x, int64_t ld, int rows, int cols, uint8_t *q, int64_t ldq, uint32_t *amax_slots,
                                     float *scale, hipStream_t stream) {
    if (rows == 0) return LVX_OK;
    LVX_TRY(lvx_launch_fill_zero(amax_slots, LVX_AMAX_SLOTS * sizeof(uint32_t), stream));
    LVX_TRY(lvx_launch_fp8_amax(x, ld, rows, cols, amax_slots, stream));
    return lvx_launch_fp8_quant(x, ld, rows, cols, q, ldq, amax_slots, nullptr, scale, stream);
}

extern "C" lvx_status_t lvx_fp8_quantize(const void *dev_x, int64_t ld, int32_t rows, int32_t cols, void *dev_q, int64_t ldq,
                                         void *dev_scratch256, float *dev_scale, lvx_stream_t stream) {
    LVX_REQUIRE(dev_x != nullptr && dev_q != nullptr && dev_scratch256 != nullptr && dev_scale != nullptr, LVX_ERR_INVALID_ARG,
                "x, q, scratch or scale is NULL");
    LVX_REQUIRE(lvx_aligned16(dev_x) && lvx_aligned16(dev_q) && lvx_aligned16(dev_scratch256) && (((uintptr_t)dev_scale) & 3u) == 0,
                LVX_ERR_INVALID_ARG, "x, q and scratch must be 16-byte aligned, scale 4-byte aligned");
    LVX_REQUIRE(rows >= 0 && cols > 0 && cols % 16 == 0, LVX_ERR_SHAPE, "rows %d, cols %d (cols must be a positive multiple of 16)", rows, cols);
    LVX_REQUIRE(ld >= cols && ld % 8 == 0 && ldq >= cols && ldq % 16 == 0, LVX_ERR_SHAPE,
                "row strides: ld a multiple of 8 and ldq a multiple of 16, both >= cols");
    return lvx_launch_fp8_quantize((const bf16_t *)dev_x, ld, rows, cols, (uint8_t *)dev_q, ldq, (uint32_t *)dev_scratch256, dev_scale,
                                   (hipStream_t)stream);
}

extern "C" lvx_status_t lvx_fp8_quantize_static(const void *dev_x, int64_t ld, int32_t rows, int32_t cols, void *dev_q, int64_t ldq,
                                                float *dev_scale, lvx_stream_t stream) {
    LVX_REQUIRE(dev_x != nullptr && dev_q != nullptr && dev_scale != nullptr, LVX_ERR_INVALID_ARG, "x, q or scale is NULL");
    LVX_REQUIRE(lvx_aligned16(dev_x) && lvx_aligned16(dev_q) && (((uintptr_t)dev_scale) & 3u) == 0, LVX_ERR_INVALID_ARG,
                "x and q must be 16-byte aligned, scale 4-byte aligned");
    LVX_REQUIRE(rows >= 0 && cols > 0 && cols % 16 == 0, LVX_ERR_SHAPE, "rows %d, cols %d (cols must be a positive multiple of 16)", rows, cols);
    LVX_REQUIRE(ld >= cols && ld % 8 == 0 && ldq >= cols && ldq % 16 == 0, LVX_ERR_SHAPE,
                "row strides: ld a multiple of 8 and ldq a multiple of 16, both >= cols");
    LVX_REQUIRE((uint64_t)rows * (uint64_t)cols <= (uint64_t)LVX_FP8_QUANTIZE_STATIC_MAX_ELEMS, LVX_ERR_SHAPE,
                "tensor of %d x %d elements exceeds the %lld elements lvx_fp8_quantize_static accepts (use lvx_fp8_quantize)", rows, cols,
                (long long)LVX_FP8_QUANTIZE_STATIC_MAX_ELEMS);
    uint32_t *slots = nullptr;
    LVX_TRY(static_scratch(&slots));
    // the array keeps the previous call's maxima: lvx_launch_fp8_quantize clears it (by kernel) before collecting
    return lvx_launch_fp8_quantize((const bf16_t *)dev_x, ld, rows, cols, (uint8_t *)dev_q, ldq, slots, dev_scale, (hipStream_t)stream);
}

lvx_status_t lvx_launch_linear_fp8(const void *dev_aq, int64_t lda, const float *dev_scale_a, const void *dev_wq, int64_t ldw,
                                   const float *dev_scale_w, void *dev_c, int64_t ldc, int32_t M, int32_t N, int32_t K, lvx_epilogue_t epi,
                                   const void *dev_resid, int64_t ldr, const float *dev_gate, uint32_t *amax_slots, hipStream_t stream) {
    LVX_REQUIRE(dev_aq != nullptr && dev_wq != nullptr && dev_c != nullptr && dev_scale_a != nullptr && dev_scale_w != nullptr,
                LVX_ERR_INVALID_ARG, "A, W, C or a scale pointer is NULL");
    LVX_REQUIRE(lvx_aligned16(dev_aq) && lvx_aligned16(dev_wq) && lvx_aligned16(dev_c) && lvx_aligned16(dev_resid), LVX_ERR_INVALID_ARG,
                "pointers must be 16-byte aligned");
    LVX_REQUIRE(M >= 0 && N > 0 && K > 0, LVX_ERR_SHAPE, "M %d, N %d, K %d", M, N, K);
    LVX_REQUIRE(K % 128 == 0, LVX_ERR_SHAPE, "K %d must be a multiple of 128", K);
    LVX_REQUIRE(N % 8 == 0, LVX_ERR_SHAPE, "N %d must be a multiple of 8", N);
    LVX_REQUIRE(lda >= K && lda % 16 == 0 && ldw >= K && ldw % 16 == 0 && ldc >= N, LVX_ERR_SHAPE, "bad leading dimension");
    LVX_REQUIRE((uint64_t)M * (uint64_t)lda < (1ull << 32) && (uint64_t)N * (uint64_t)ldw < (1ull << 32), LVX_ERR_SHAPE,
                "operand larger than 4 GiB (32-bit byte offsets inside the kernel)");
    LVX_REQUIRE(epi == LVX_EPI_STORE || epi == LVX_EPI_GELU_TANH || epi == LVX_EPI_RESID_GATE || epi == LVX_EPI_RESID_GATE_F32,
                LVX_ERR_INVALID_ARG, "unknown epilogue %d", (int)epi);
    if (epi == LVX_EPI_RESID_GATE || epi == LVX_EPI_RESID_GATE_F32) {
        LVX_REQUIRE(dev_resid != nullptr, LVX_ERR_INVALID_ARG, "residual epilogue needs a residual pointer");
        LVX_REQUIRE(ldr >= N, LVX_ERR_SHAPE, "bad residual leading dimension");
    }
    if (M == 0) return LVX_OK;
    constexpr int BM = 128, BN = 256;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const dim3 grid(per_xcd * 8), block(512);
#define LVX8_LAUNCH(EPI_)                                                                                                         \
    hipLaunchKernelGGL((lvx_gemm_fp8_kernel<BM, BN, 2, 4, EPI_>), grid, block, 0, (hipStream_t)stream, (const uint8_t *)dev_aq, lda, \
                       (const uint8_t *)dev_wq, ldw, dev_scale_a, dev_scale_w, (bf16_t *)dev_c, ldc, M, N, K, (const bf16_t *)dev_resid, \
                       ldr, dev_gate, tiles_m, tiles_n, per_xcd, amax_slots)
    if (epi == LVX_EPI_STORE) {
        LVX8_LAUNCH(LVX_EPI_STORE);
    } else if (epi == LVX_EPI_GELU_TANH) {
        LVX8_LAUNCH(LVX_EPI_GELU_TANH);
    } else if (epi == LVX_EPI_RESID_GATE) {
        LVX8_LAUNCH(LVX_EPI_RESID_GATE);
    } else {
        LVX8_LAUNCH(LVX_EPI_RESID_GATE_F32);
    }
#undef LVX8_LAUNCH
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

extern "C" lvx_status_t lvx_linear_fp8(const void *dev_aq, int64_t lda, const float *dev_scale_a, const void *dev_wq, int64_t ldw,
                                       const float *dev_scale_w, void *dev_c, int64_t ldc, int32_t M, int32_t N, int32_t K,
                                       lvx_epilogue_t epi, const void *dev_resid, int64_t ldr, const float *dev_gate, lvx_stream_t stream) {
    return lvx_launch_linear_fp8(dev_aq, lda, dev_scale_a, dev_wq, ldw, dev_scale_w, dev_c, ldc, M, N, K, epi, dev_resid, ldr, dev_gate, nullptr,
                                 (hipStream_t)stream);
}
