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

    // global source rows, clamped so that tail tiles read valid memory (their results are never stored)
    const bf16_t *a_ptr[A_CPT];
    const bf16_t *w_ptr[W_CPT];
#pragma unroll
    for (int i = 0; i < A_CPT; ++i) {
        const int g = tid + i * NT;
        int r = tm * BM + g / (BK / 8);
        if (r > M - 1) r = M - 1;
        a_ptr[i] = A + (size_t)r * lda + (g % (BK / 8)) * 8;
    }
#pragma unroll
    for (int i = 0; i < W_CPT; ++i) {
        const int g = tid + i * NT;
        int r = tn * BN + g / (BK / 8);
        if (r > N - 1) r = N - 1;
        w_ptr[i] = W + (size_t)r * ldw + (g % (BK / 8)) * 8;
    }

    u32x4_t areg[A_CPT], wreg[W_CPT];
#define LVX_GEMM_GLOAD(k0_)                                                                                       \
    {                                                                                                             \
        _Pragma("unroll") for (int i = 0; i < A_CPT; ++i) areg[i] = *reinterpret_cast<const u32x4_t *>(a_ptr[i] + (k0_)); \
        _Pragma("unroll") for (int i = 0; i < W_CPT; ++i) wreg[i] = *reinterpret_cast<const u32x4_t *>(w_ptr[i] + (k0_)); \
    }
#define LVX_GEMM_LSTORE(buf_)                                                                                     \
    {                                                                                                             \
        _Pragma("unroll") for (int i = 0; i < A_CPT; ++i) {                                                       \
            const int g = tid + i * NT;                                                                           \
            *reinterpret_cast<u32x4_t *>(&as[(buf_) * A_STAGE + (g / (BK / 8)) * LDT + (g % (BK / 8)) * 8]) = areg[i]; \
        }                                                                                                         \
        _Pragma("unroll") for (int i = 0; i < W_CPT; ++i) {                                                       \
            const int g = tid + i * NT;                                                                           \
            *reinterpret_cast<u32x4_t *>(&ws[(buf_) * W_STAGE + (g / (BK / 8)) * LDT + (g % (BK / 8)) * 8]) = wreg[i]; \
        }                                                                                                         \
    }

    f32x16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int n_k = K / BK;
    LVX_GEMM_GLOAD(0);
    LVX_GEMM_LSTORE(0);
    __syncthreads();

    for (int kt = 0; kt < n_k; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < n_k) LVX_GEMM_GLOAD((kt + 1) * BK);
        const bf16_t *ap = &as[buf * A_STAGE + (wm * WTM + l32) * LDT + hh * 8];
        const bf16_t *wp = &ws[buf * W_STAGE + (wn * WTN + l32) * LDT + hh * 8];
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8_t af[FM], wf[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) af[i] = *reinterpret_cast<const bf16x8_t *>(ap + i * 32 * LDT + kk * 16);
#pragma unroll
            for (int j = 0; j < FN; ++j) wf[j] = *reinterpret_cast<const bf16x8_t *>(wp + j * 32 * LDT + kk * 16);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < n_k) LVX_GEMM_LSTORE(buf ^ 1);
        __syncthreads();
    }

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
    LVX_REQUIRE(epi == LVX_EPI_STORE || epi == LVX_EPI_GELU_TANH || epi == LVX_EPI_RESID_GATE || epi == LVX_EPI_RESID_GATE_F32,
                LVX_ERR_INVALID_ARG, "unknown epilogue %d", (int)epi);
    if (epi == LVX_EPI_RESID_GATE || epi == LVX_EPI_RESID_GATE_F32) {
        LVX_REQUIRE(dev_resid != nullptr, LVX_ERR_INVALID_ARG, "residual epilogue needs a residual pointer");
        LVX_REQUIRE(ldr >= N, LVX_ERR_SHAPE, "bad residual leading dimension");
    }
    if (M == 0) return LVX_OK;
    return launch<128, 256, 2, 2>((const bf16_t *)dev_a, lda, (const bf16_t *)dev_w, ldw, (bf16_t *)dev_c, ldc, M, N, K, (int)epi,
                                  (const bf16_t *)dev_resid, ldr, dev_gate, (hipStream_t)stream);
}
