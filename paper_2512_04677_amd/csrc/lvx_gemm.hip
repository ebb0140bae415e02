// bf16 MFMA GEMM for the DiT linears:  C[M][N] = epilogue(A[M][K] * W[N][K]^T), fp32 accumulate.
// (The paper's "all linear projections in the DiT", Appendix C; shapes are the workload's.)
//
// Both operands have the contraction index contiguous in memory (activations [token][in], weights [out][in]), so both
// stream into LDS with 16-byte loads and are read back as direct v_mfma_f32_32x32x16_bf16 operands with 16-byte
// ds_reads.  One workgroup owns a BM x BN tile of C, K is walked in 64-wide slabs double-buffered in LDS (rows padded
// by 16 bytes: 16 consecutive lanes hit disjoint banks).  The A operand of the MFMA is the activation tile, so an
// accumulator register holds 32 consecutive output columns across lanes: stores are 64-byte contiguous runs and the
// per-column gate of the residual epilogue is a per-lane scalar.
// Workgroup ids are dealt to XCDs round-robin by hardware; each XCD gets a contiguous range of tiles, walked in
// column-major order inside bands of 8 row tiles, so concurrently running workgroups of one XCD share A and W slabs in
// that XCD's L2.
#include "lvx_internal.h"

namespace {

constexpr int BK = 64;
constexpr int LDT = BK + 8;  // padded LDS row (bf16)
constexpr int GROUP_M = 8;

__device__ __forceinline__ float gelu_tanh_f32(float x) {
    // 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3)
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    const float e = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * u);
    return x * __builtin_amdgcn_rcpf(1.0f + e);
}

// Scheduling hint for one half of a slab step: MFMA number I is followed by one LDS fragment read (while I < NDSR), by
// QW LDS stores (while any of the NDSW are left) and by QV global loads (while any of the NVM are left), so that the matrix
// core, the LDS and the texture address unit work at the same time instead of in turns.
template <int I, int NM, int NDSR, int NDSW, int QW, int NVM, int QV>
struct sgb_half {
    static __device__ __forceinline__ void emit() {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (I < NDSR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        constexpr int w = NDSW - I * QW < 0 ? 0 : (NDSW - I * QW < QW ? NDSW - I * QW : QW);
        if (w > 0) __builtin_amdgcn_sched_group_barrier(0x200, w, 0);
        constexpr int v = NVM - I * QV < 0 ? 0 : (NVM - I * QV < QV ? NVM - I * QV : QV);
        if (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);
        sgb_half<I + 1, NM, NDSR, NDSW, QW, NVM, QV>::emit();
    }
};
template <int NM, int NDSR, int NDSW, int QW, int NVM, int QV>
struct sgb_half<NM, NM, NDSR, NDSW, QW, NVM, QV> {
    static __device__ __forceinline__ void emit() {}
};

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
    lvx_gemm_kernel(const bf16_t *__restrict__ A, int64_t lda, const bf16_t *__restrict__ W, int64_t ldw, bf16_t *C, int64_t ldc, int M,
                    int N, int K, const bf16_t *R, int64_t ldr, const float *__restrict__ gate, int tiles_m, int tiles_n, int per_xcd) {
    constexpr int NT = 64 * WAVES_M * WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int FM = WTM / 32, FN = WTN / 32;
    constexpr int A_STAGE = BM * LDT, W_STAGE = BN * LDT;
    constexpr int A_CH = BM * (BK / 8), W_CH = BN * (BK / 8);
    static_assert(A_CH % NT == 0 && W_CH % NT == 0, "tile chunks must divide over the threads");
    constexpr int A_CPT = A_CH / NT, W_CPT = W_CH / NT;
    constexpr int NKK = BK / 16;

    __shared__ __attribute__((aligned(16))) bf16_t as[2 * A_STAGE];
    __shared__ __attribute__((aligned(16))) bf16_t ws[2 * W_STAGE];

    const int total = tiles_m * tiles_n;
    const int widx = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
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

    // byte offsets of this thread's 16-byte chunks from the (uniform) tile-column base; rows are clamped so that tail
    // tiles read valid memory (their results are never stored)
    uint32_t a_off[A_CPT], w_off[W_CPT];
#pragma unroll
    for (int i = 0; i < A_CPT; ++i) {
        const int g = tid + i * NT;
        int r = tm * BM + g / (BK / 8);
        if (r > M - 1) r = M - 1;
        a_off[i] = (uint32_t)(((size_t)r * lda + (g % (BK / 8)) * 8) * sizeof(bf16_t));
    }
#pragma unroll
    for (int i = 0; i < W_CPT; ++i) {
        const int g = tid + i * NT;
        int r = tn * BN + g / (BK / 8);
        if (r > N - 1) r = N - 1;
        w_off[i] = (uint32_t)(((size_t)r * ldw + (g % (BK / 8)) * 8) * sizeof(bf16_t));
    }

    // two register sets: the slab two steps ahead is in flight while the slab one step ahead waits to enter LDS
    u32x4_t ra0[A_CPT], rw0[W_CPT], ra1[A_CPT], rw1[W_CPT];
#define LVX_GEMM_GLOAD(kt_, RA, RW)                                                                                          \
    {                                                                                                                        \
        const char *ab_ = reinterpret_cast<const char *>(A + (size_t)(kt_) * BK);                                            \
        const char *wb_ = reinterpret_cast<const char *>(W + (size_t)(kt_) * BK);                                            \
        _Pragma("unroll") for (int i = 0; i < A_CPT; ++i) RA[i] = *reinterpret_cast<const u32x4_t *>(ab_ + a_off[i]);        \
        _Pragma("unroll") for (int i = 0; i < W_CPT; ++i) RW[i] = *reinterpret_cast<const u32x4_t *>(wb_ + w_off[i]);        \
    }
#define LVX_GEMM_LSTORE(buf_, RA, RW)                                                                              \
    {                                                                                                              \
        _Pragma("unroll") for (int i = 0; i < A_CPT; ++i) {                                                        \
            const int g = tid + i * NT;                                                                            \
            *reinterpret_cast<u32x4_t *>(&as[(buf_) * A_STAGE + (g / (BK / 8)) * LDT + (g % (BK / 8)) * 8]) = RA[i]; \
        }                                                                                                          \
        _Pragma("unroll") for (int i = 0; i < W_CPT; ++i) {                                                        \
            const int g = tid + i * NT;                                                                            \
            *reinterpret_cast<u32x4_t *>(&ws[(buf_) * W_STAGE + (g / (BK / 8)) * LDT + (g % (BK / 8)) * 8]) = RW[i]; \
        }                                                                                                          \
    }

    f32x16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // ---- main loop ------------------------------------------------------------------------------------------------
    // Slab kt lives in LDS buffer kt&1; each slab is NKK = 4 MFMA k-steps; one workgroup barrier per slab.
    //   hazards: the other buffer was last read (k-step 3 of slab kt-1) before the previous barrier; the stores into it are
    //   fenced by this slab's barrier, after which they are read.
    bf16x8_t af[2][FM], wf[2][FN];  // fragment sets, indexed by k-step parity
    constexpr int NMH = (NKK / 2) * FM * FN;    // MFMAs per half
    constexpr int NRH = (NKK / 2) * (FM + FN);  // fragment reads per half
    constexpr int NST = A_CPT + W_CPT;          // staging chunks per thread
    constexpr int QST = (NST + NMH - 1) / NMH;
#define LVX_GEMM_READ_FRAGS(buf_, kk_)                                                                                      \
    {                                                                                                                       \
        const bf16_t *ap_ = &as[(buf_) * A_STAGE + (wm * WTM + l32) * LDT + hh * 8 + (kk_) * 16];                           \
        const bf16_t *wp_ = &ws[(buf_) * W_STAGE + (wn * WTN + l32) * LDT + hh * 8 + (kk_) * 16];                           \
        _Pragma("unroll") for (int i = 0; i < FM; ++i) af[(kk_) & 1][i] = *reinterpret_cast<const bf16x8_t *>(ap_ + i * 32 * LDT); \
        _Pragma("unroll") for (int j = 0; j < FN; ++j) wf[(kk_) & 1][j] = *reinterpret_cast<const bf16x8_t *>(wp_ + j * 32 * LDT); \
    }
#define LVX_GEMM_MFMAS(kk_)                                                                                  \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) _Pragma("unroll") for (int j = 0; j < FN; ++j)            \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[(kk_) & 1][i], wf[(kk_) & 1][j], acc[i][j], 0, 0, 0);
    // Staging chunk c (0 .. NST-1; the first A_CPT are A chunks, the rest W chunks) of register set (RA, RW).
#define LVX_GEMM_LSTORE_CH(buf_, RA, RW, c_)                                                                                  \
    {                                                                                                                         \
        if ((c_) < A_CPT) {                                                                                                   \
            const int g = tid + (c_) * NT;                                                                                    \
            *reinterpret_cast<u32x4_t *>(&as[(buf_) * A_STAGE + (g / (BK / 8)) * LDT + (g % (BK / 8)) * 8]) = RA[(c_) < A_CPT ? (c_) : 0]; \
        } else {                                                                                                              \
            const int g = tid + ((c_) - A_CPT) * NT;                                                                          \
            *reinterpret_cast<u32x4_t *>(&ws[(buf_) * W_STAGE + (g / (BK / 8)) * LDT + (g % (BK / 8)) * 8]) = RW[(c_) >= A_CPT ? (c_) - A_CPT : 0]; \
        }                                                                                                                     \
    }
#define LVX_GEMM_GLOAD_CH(kt_, RA, RW, c_)                                                                                    \
    {                                                                                                                         \
        if ((c_) < A_CPT)                                                                                                     \
            RA[(c_) < A_CPT ? (c_) : 0] = *reinterpret_cast<const u32x4_t *>(reinterpret_cast<const char *>(A + (size_t)(kt_) * BK) + a_off[(c_) < A_CPT ? (c_) : 0]); \
        else                                                                                                                  \
            RW[(c_) >= A_CPT ? (c_) - A_CPT : 0] = *reinterpret_cast<const u32x4_t *>(reinterpret_cast<const char *>(W + (size_t)(kt_) * BK) + w_off[(c_) >= A_CPT ? (c_) - A_CPT : 0]); \
    }
    // One slab step in four MFMA groups (one per k-step); sched_barrier(0) pins the order of the groups, the compiler
    // schedules inside one.  Group g issues the MFMAs of k-step g while it reads the fragments of the NEXT k-step into the
    // other fragment set; the barrier sits between groups 2 and 3, so a wave arrives at it with group 3's fragments already
    // in registers and reads k-step 0 of the next slab (other buffer) right after it.  The next slab's staging chunks go to
    // LDS in groups 0..2 (before the barrier); the global loads that refill those registers are spread over all four groups
    // (never before their store), so the texture address unit (64 B/clk: 16 cycles per 16-byte wave load) works in the
    // background instead of all waves queueing on it at once.
#define LVX_GEMM_GROUP(g_, rbuf_, rkk_, mkk_, sbuf_, RA, RW, kt_load_)                                      \
    {                                                                                                       \
        LVX_GEMM_READ_FRAGS(rbuf_, rkk_);                                                                   \
        LVX_GEMM_MFMAS(mkk_);                                                                               \
        _Pragma("unroll") for (int c = 0; c < NST; ++c) {                                                   \
            if ((g_) < 3 && (c * 3) / NST == (g_)) LVX_GEMM_LSTORE_CH(sbuf_, RA, RW, c);                    \
        }                                                                                                   \
        _Pragma("unroll") for (int c = 0; c < NST; ++c) {                                                   \
            if ((c * 4) / NST == (g_)) LVX_GEMM_GLOAD_CH(kt_load_, RA, RW, c);                              \
        }                                                                                                   \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
    }
#define LVX_GEMM_STEP(buf_, RA, RW, kt_load_)                                                   \
    {                                                                                           \
        LVX_GEMM_GROUP(0, buf_, 1, 0, (buf_) ^ 1, RA, RW, kt_load_);                            \
        LVX_GEMM_GROUP(1, buf_, 2, 1, (buf_) ^ 1, RA, RW, kt_load_);                            \
        LVX_GEMM_GROUP(2, buf_, 3, 2, (buf_) ^ 1, RA, RW, kt_load_);                            \
        __syncthreads();                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                      \
        LVX_GEMM_GROUP(3, (buf_) ^ 1, 0, 3, (buf_) ^ 1, RA, RW, kt_load_);                      \
    }

    const int n_k = K / BK;
    const int last = n_k - 1;
    // slab j is staged in register set j&1; loads past the last slab re-read the last slab (never consumed)
    LVX_GEMM_GLOAD(0, ra0, rw0);
    LVX_GEMM_GLOAD(last < 1 ? last : 1, ra1, rw1);
    LVX_GEMM_LSTORE(0, ra0, rw0);
    LVX_GEMM_GLOAD(last < 2 ? last : 2, ra0, rw0);
    __syncthreads();
    LVX_GEMM_READ_FRAGS(0, 0);

    int kt = 0;
    for (; kt + 1 < n_k; kt += 2) {
        LVX_GEMM_STEP(0, ra1, rw1, (kt + 3 < last ? kt + 3 : last));
        LVX_GEMM_STEP(1, ra0, rw0, (kt + 4 < last ? kt + 4 : last));
    }
    if (kt < n_k) LVX_GEMM_STEP(0, ra1, rw1, last);

    // accumulator register 4g+r of fragment (i,j): row m = 32i + 8g + 4hh + r, column n = 32j + l32
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int n = tn * BN + wn * WTN + j * 32 + l32;
        if (n >= N) continue;
        float gt = 1.f;
        if ((EPI == LVX_EPI_RESID_GATE || EPI == LVX_EPI_RESID_GATE_F32) && gate != nullptr) gt = gate[n];
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = tm * BM + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * hh + (e & 3);
                if (m >= M) continue;
                float v = acc[i][j][e];
                if (EPI == LVX_EPI_GELU_TANH) v = gelu_tanh_f32(v);
                if (EPI == LVX_EPI_RESID_GATE) v = bf16_bits_to_f32(R[(size_t)m * ldr + n]) + gt * v;
                if (EPI == LVX_EPI_RESID_GATE_F32) {
                    const float *rf = reinterpret_cast<const float *>(R);
                    reinterpret_cast<float *>(C)[(size_t)m * ldc + n] = rf[(size_t)m * ldr + n] + gt * v;
                } else {
                    C[(size_t)m * ldc + n] = (bf16_t)(pack_bf16x2(v, 0.f) & 0xffffu);
                }
            }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
lvx_status_t launch(const bf16_t *A, int64_t lda, const bf16_t *W, int64_t ldw, bf16_t *C, int64_t ldc, int M, int N, int K, int epi,
                    const bf16_t *R, int64_t ldr, const float *gate, hipStream_t stream) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const dim3 grid(per_xcd * 8), block(64 * WAVES_M * WAVES_N);
#define LVX_GEMM_LAUNCH(EPI_)                                                                                                      \
    hipLaunchKernelGGL((lvx_gemm_kernel<BM, BN, WAVES_M, WAVES_N, EPI_>), grid, block, 0, stream, A, lda, W, ldw, C, ldc, M, N, K, R, ldr, \
                       gate, tiles_m, tiles_n, per_xcd)
    if (epi == LVX_EPI_STORE)
        LVX_GEMM_LAUNCH(LVX_EPI_STORE);
    else if (epi == LVX_EPI_GELU_TANH)
        LVX_GEMM_LAUNCH(LVX_EPI_GELU_TANH);
    else if (epi == LVX_EPI_RESID_GATE)
        LVX_GEMM_LAUNCH(LVX_EPI_RESID_GATE);
    else
        LVX_GEMM_LAUNCH(LVX_EPI_RESID_GATE_F32);
#undef LVX_GEMM_LAUNCH
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

}  // namespace

extern "C" lvx_status_t lvx_linear(const void *dev_a, int64_t lda, const void *dev_w, int64_t ldw, void *dev_c, int64_t ldc, int32_t M,
                                   int32_t N, int32_t K, lvx_epilogue_t epi, const void *dev_resid, int64_t ldr, const float *dev_gate,
                                   lvx_stream_t stream) {
    LVX_REQUIRE(dev_a != nullptr && dev_w != nullptr && dev_c != nullptr, LVX_ERR_INVALID_ARG, "A, W or C is NULL");
    LVX_REQUIRE(lvx_aligned16(dev_a) && lvx_aligned16(dev_w) && lvx_aligned16(dev_c) && lvx_aligned16(dev_resid), LVX_ERR_INVALID_ARG,
                "pointers must be 16-byte aligned");
    LVX_REQUIRE(M >= 0 && N > 0 && K > 0, LVX_ERR_SHAPE, "M %d, N %d, K %d", M, N, K);
    LVX_REQUIRE(K % BK == 0, LVX_ERR_SHAPE, "K %d must be a multiple of %d", K, BK);
    LVX_REQUIRE(N % 8 == 0, LVX_ERR_SHAPE, "N %d must be a multiple of 8", N);
    LVX_REQUIRE(lda >= K && lda % 8 == 0 && ldw >= K && ldw % 8 == 0 && ldc >= N, LVX_ERR_SHAPE, "bad leading dimension");
    LVX_REQUIRE((uint64_t)M * (uint64_t)lda * 2 < (1ull << 32) && (uint64_t)N * (uint64_t)ldw * 2 < (1ull << 32), LVX_ERR_SHAPE,
                "operand larger than 4 GiB (32-bit byte offsets inside the kernel)");
    LVX_REQUIRE(epi == LVX_EPI_STORE || epi == LVX_EPI_GELU_TANH || epi == LVX_EPI_RESID_GATE || epi == LVX_EPI_RESID_GATE_F32,
                LVX_ERR_INVALID_ARG, "unknown epilogue %d", (int)epi);
    if (epi == LVX_EPI_RESID_GATE || epi == LVX_EPI_RESID_GATE_F32) {
        LVX_REQUIRE(dev_resid != nullptr, LVX_ERR_INVALID_ARG, "residual epilogue needs a residual pointer");
        LVX_REQUIRE(ldr >= N, LVX_ERR_SHAPE, "bad residual leading dimension");
    }
    if (M == 0) return LVX_OK;
    return launch<128, 256, 2, 4>((const bf16_t *)dev_a, lda, (const bf16_t *)dev_w, ldw, (bf16_t *)dev_c, ldc, M, N, K, (int)epi,
                                  (const bf16_t *)dev_resid, ldr, dev_gate, (hipStream_t)stream);
}
