// bf16 MFMA GEMM for the DiT linears:  C[M][N] = epilogue(A[M][K] * W[N][K]^T), fp32 accumulate.
// (The linears of the DiT blocks, Appendix C; shapes are the workload's.)
//
// Both operands have the contraction index contiguous in memory (activations [token][in], weights [out][in]), so both
// stream global -> LDS as 16-byte chunks (direct-to-LDS loads, three 64-wide K slabs in flight) and are read back as direct
// v_mfma_f32_16x16x32_bf16 operands with 16-byte ds_reads (the 16 x 16 x 32 form moves a fifth less through the register
// file per flop than 32 x 32 x 16 and runs 1-5 % faster here, the chip being power-limited).  One workgroup owns a BM x BN
// tile of C.  The A operand of the MFMA is the activation tile, so an accumulator register holds 16 consecutive output
// columns of one row per 16 lanes: stores are 32-byte (fp32: 64-byte) runs and the per-column gate / bias of the epilogue
// is a per-lane scalar.
// Workgroup ids are dealt to XCDs round-robin by hardware; each XCD gets a contiguous range of tiles, walked in
// column-major order inside bands of 8 row tiles, so concurrently running workgroups of one XCD share A and W slabs in
// that XCD's L2.
// The same kernel serves the decoder's 3x3x3 convolution as an implicit GEMM (CONV): its A rows are gathered from a
// zero-padded volume, a tap being a constant shift of the row addresses.
#include "lvx_internal.h"

namespace {

constexpr int BK = 64;
constexpr int GROUP_M = 8;

// Epilogue.  Accumulator register e of 16 x 16 block (i,j) holds row m0 + 16i + e and column n0 + 16j of C (m0, n0 already
// include the lane's 4*q4 / l16 offsets): for a fixed register, each group of 16 lanes writes 16 consecutive columns of one
// row.  Interior tiles take the branch-free path; only tiles on the M or N edge check every element.
template <int FM, int FN, int EPI>
__device__ __forceinline__ void lvx_gemm_epilogue(f32x4_t (&acc)[FM][FN], f32x4_t (&rres)[FM][FN], bf16_t *C, int64_t ldc, const bf16_t *R,
                                                  int64_t ldr, const float *__restrict__ gate, int M, int N, int m0, int n0) {
    const bool interior = (m0 - (m0 & 12) + FM * 16 <= M) && (n0 - (n0 & 15) + FN * 16 <= N);
    float gt[FN];  // per column block: the gate (residual epilogues) or the bias of this lane's column
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int n = n0 + j * 16 < N ? n0 + j * 16 : N - 1;
        gt[j] = 1.f;
        if ((EPI == LVX_EPI_RESID_GATE || EPI == LVX_EPI_RESID_GATE_F32) && gate != nullptr) gt[j] = gate[n];
        if (EPI == LVX_EPI_BIAS || EPI == LVX_EPI_BIAS_SILU) gt[j] = gate != nullptr ? gate[n] : 0.f;
    }
    // rows outermost, column blocks innermost: the FN stores of one row follow each other, so neighbouring 32-byte (fp32:
    // 64-byte) runs of a cache line reach L2 together
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int m = m0 + i * 16 + e;
            if (!interior && m >= M) continue;
            bf16_t *cp = C + (size_t)m * ldc + n0;
            float *cpf = reinterpret_cast<float *>(C) + (size_t)m * ldc + n0;
            const bf16_t *rp = R + (size_t)m * ldr + n0;
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                if (!interior && n0 + j * 16 >= N) continue;
                float v = acc[i][j][e];
                if (EPI == LVX_EPI_GELU_TANH) v = gelu_tanh_f32(v);
                if (EPI == LVX_EPI_BIAS || EPI == LVX_EPI_BIAS_SILU) v += gt[j];
                if (EPI == LVX_EPI_BIAS_SILU) v = v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * v));
                if (EPI == LVX_EPI_RESID_GATE) v = bf16_bits_to_f32(rp[j * 16]) + gt[j] * v;
                if (EPI == LVX_EPI_RESID_GATE_F32)
                    cpf[j * 16] = rres[i][j][e] + gt[j] * v;
                else if (EPI == LVX_EPI_STORE_F32)
                    cpf[j * 16] = v;
                else
                    cp[j * 16] = (bf16_t)(pack_bf16x2(v, 0.f) & 0xffffu);
            }
        }
    }
}

// Sum of squares of this wave's FN * 16 columns for each of its rows (fp32 accumulators), one float per row at out[m * ld + part].
template <int FM, int FN>
__device__ __forceinline__ void lvx_gemm_row_sumsq(const f32x4_t (&acc)[FM][FN], float *out, int64_t ld, int part, int M, int m0, int l16) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float ss = 0.f;
#pragma unroll
            for (int j = 0; j < FN; ++j) ss += acc[i][j][e] * acc[i][j][e];
            ss += __shfl_xor(ss, 1);
            ss += __shfl_xor(ss, 2);
            ss += __shfl_xor(ss, 4);
            ss += __shfl_xor(ss, 8);
            const int m = m0 + i * 16 + e;
            if (l16 == 0 && m < M) out[(size_t)m * ld + part] = ss;
        }
}

// gfx950's global_load_lds_dwordx4 moves 16 bytes per lane from
// global memory straight into LDS (LDS byte address = M0 + 16*lane), so a slab needs no staging registers, no ds_write
// and no trip through the register file; the pipeline depth is set by LDS stages (three 48 KB stages for a 128x256 tile)
// instead of by registers.  A DMA wave-instruction fills 1024 contiguous LDS bytes = 8 rows of 64 bf16, so rows cannot be
// padded; bank conflicts are avoided by an XOR swizzle instead: the 16-byte chunk c of LDS row r holds global chunk
// c ^ ((r >> 1) & 7) (the lane simply fetches that chunk), and a fragment read of k-chunk c goes to position
// c ^ ((r >> 1) & 7): 16 consecutive rows then cover 16 distinct 16-byte units of the 256-byte bank row.
// The loads are issued through inline asm with explicit s_waitcnt vmcnt(n): the compiler would otherwise wait for ALL
// outstanding DMA before any LDS read that might alias, which would undo the multi-stage pipeline.
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, bool CONV>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
    lvx_gemm_dma_kernel(const bf16_t *__restrict__ A, int64_t lda, const bf16_t *__restrict__ W, int64_t ldw, bf16_t *C, int64_t ldc,
                        int M, int N, int K, const bf16_t *R, int64_t ldr, const float *__restrict__ gate, int tiles_m, int tiles_n,
                        int per_xcd, lvx_gemm_segs_t segs, lvx_conv_map_t cm) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int FM = WTM / 16, FN = WTN / 16;  // 16 x 16 accumulator blocks per wave
    constexpr int NKS = BK / 32;                 // 32-wide MFMA k-steps per slab
    constexpr int ROW_B = BK * 2;  // bytes per LDS row (unpadded)
    constexpr int A_B = BM * ROW_B, STAGE_B = (BM + BN) * ROW_B;
    constexpr int NSTAGE = 3;
    constexpr int N_INSTR = (BM + BN) / 8;  // DMA wave-instructions per slab (8 rows each)
    static_assert(N_INSTR % NW == 0 && (BM / 8) % NW == 0, "DMA instructions must divide over the waves, A and W separately");
    constexpr int QPW = N_INSTR / NW;   // per wave
    constexpr int A_Q = (BM / 8) / NW;  // of which the first A_Q fetch A rows
    static_assert(NKS == 2 && FM % 2 == 0, "the grouping below assumes 2 k-steps per slab, each issued as two halves");

    __shared__ __attribute__((aligned(1024))) char lds[NSTAGE * STAGE_B];

    const int total = tiles_m * tiles_n;
#ifdef LVX_GEMM_NPART
    // experiment: XCD x owns the column tiles [x * tn_per, (x + 1) * tn_per) and walks all row tiles of them, bands of 8 row tiles
    const int tn_per = (tiles_n + 7) / 8;
    const int tn_lo = (blockIdx.x & 7) * tn_per;
    const int tn_cnt = tiles_n - tn_lo < tn_per ? tiles_n - tn_lo : tn_per;
    const int kx = blockIdx.x >> 3;
    if (tn_cnt <= 0 || kx >= tiles_m * tn_cnt) return;
    const int band = kx / (GROUP_M * tn_cnt);
    const int first_m = band * GROUP_M;
    const int band_m = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
    const int in_band = kx - band * GROUP_M * tn_cnt;
    const int tm = first_m + in_band % band_m;
    int tn = tn_lo + in_band / band_m;
    const int widx = tm * tiles_n + tn;
#else
    const int widx = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (widx >= total) return;
    const int band = widx / (GROUP_M * tiles_n);
    const int first_m = band * GROUP_M;
    const int band_m = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
    const int in_band = widx - band * GROUP_M * tiles_n;
    const int tm = first_m + in_band % band_m;
    int tn = in_band / band_m;
#endif
    // several projections of the same activations in one launch (tiles_n counts all of them): the column tile's segment gives
    // the weight matrix, the output, its width, its row stride and whether it is stored in fp32 (workgroup-uniform)
    bool seg_f32 = false;
    float *seg_sumsq = nullptr;
    int seg_ld_sumsq = 0;
    if (EPI == LVX_EPI_SEGMENTS) {
        int sg = 0;
        for (int i = 1; i < segs.n; ++i)
            if (tn >= segs.s[i].tn_begin) sg = i;
        tn -= segs.s[sg].tn_begin;
        W = segs.s[sg].W;
        C = reinterpret_cast<bf16_t *>(segs.s[sg].C);
        ldc = segs.s[sg].ldc;
        N = segs.s[sg].N;
        seg_f32 = segs.s[sg].f32 != 0;
        seg_sumsq = segs.s[sg].sumsq;
        seg_ld_sumsq = segs.s[sg].ld_sumsq;
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, q4 = lane >> 4;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // DMA instruction q of this wave covers stage rows 8*(wave + NW*q) .. +7 (A rows first, then W rows); lane -> (row, position)
    uint32_t doff[QPW];
#pragma unroll
    for (int q = 0; q < QPW; ++q) {
        const int row_s = 8 * (wave + NW * q) + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row_s >> 1) & 7);
        if (q < A_Q) {
            int r = tm * BM + row_s;
            if (r > M - 1) r = M - 1;
            size_t e = (size_t)r * lda;
            if (CONV) {  // output pixel r = (t, y, x) -> its position in the padded volume (tap (0,0,0))
                const int hw = cm.H * cm.W;
                const int t = r / hw, rem = r - t * hw;
                const int y = rem / cm.W, x = rem - y * cm.W;
                e = (size_t)t * cm.frame_pitch + (size_t)y * cm.row_pitch + (size_t)x * cm.C;
            }
            doff[q] = (uint32_t)((e + chunk * 8) * sizeof(bf16_t));
        } else {
            int r = tn * BN + (row_s - BM);
            if (r > N - 1) r = N - 1;
            doff[q] = (uint32_t)(((size_t)r * ldw + chunk * 8) * sizeof(bf16_t));
        }
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds_base + wave * 1024);
    // byte offset of K slab kt in the A operand: plain GEMM kt * 128; convolution: the tap's shift in the padded volume plus
    // the slab's channel offset inside the tap (wave-uniform scalar arithmetic)
    auto a_slab = [&](int kt) -> size_t {
        if (!CONV) return (size_t)kt * ROW_B;
        const int tap = kt / cm.slabs_per_tap, kc = kt - tap * cm.slabs_per_tap;
        const int dt = tap / 9, dy = (tap - dt * 9) / 3, dx = tap - dt * 9 - dy * 3;
        return ((size_t)dt * cm.frame_pitch + (size_t)dy * cm.row_pitch + (size_t)dx * cm.C) * sizeof(bf16_t) + (size_t)kc * ROW_B;
    };
#define LVX_DMA_ISSUE(stage_, kt_, q_)                                                                                      \
    lvx_dma16((q_) < A_Q ? reinterpret_cast<const char *>(A) + a_off_ : reinterpret_cast<const char *>(W) + (size_t)(kt_) * ROW_B, \
              doff[q_], lds_wave + (uint32_t)((stage_) * STAGE_B + (q_) * NW * 1024))

    // fragment reads for v_mfma_f32_16x16x32_bf16: lane (l16, q4) reads row l16 of a 16-row block, k-chunk 4*ks + q4 of the
    // slab's 8, at its swizzled position
    const int swz = (l16 >> 1) & 7;
    const char *a_rd = lds + (wm * WTM + l16) * ROW_B;
    const char *w_rd = lds + A_B + (wn * WTN + l16) * ROW_B;
    bf16x8_t af[2][FM], wf[2][FN];
#define LVX_DMA_READ_A(stage_, ks_, i0_, i1_)                                                                               \
    {                                                                                                                       \
        const int co_ = (((ks_) * 4 + q4) ^ swz) * 16 + (stage_) * STAGE_B;                                                 \
        _Pragma("unroll") for (int i = i0_; i < i1_; ++i) af[(ks_) & 1][i] = *reinterpret_cast<const bf16x8_t *>(a_rd + i * 16 * ROW_B + co_); \
    }
#define LVX_DMA_READ_W(stage_, ks_, j0_, j1_)                                                                               \
    {                                                                                                                       \
        const int co_ = (((ks_) * 4 + q4) ^ swz) * 16 + (stage_) * STAGE_B;                                                 \
        _Pragma("unroll") for (int j = j0_; j < j1_; ++j) wf[(ks_) & 1][j] = *reinterpret_cast<const bf16x8_t *>(w_rd + j * 16 * ROW_B + co_); \
    }
    // MFMAs of k-step ks_ for accumulator rows [i0_, i1_)
#define LVX_DMA_MFMAS(ks_, i0_, i1_)                                                                         \
    _Pragma("unroll") for (int i = i0_; i < i1_; ++i) _Pragma("unroll") for (int j = 0; j < FN; ++j)         \
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[(ks_) & 1][i], wf[(ks_) & 1][j], acc[i][j], 0, 0, 0);

    f32x4_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

    // fp32 residual epilogue: the tile of R this lane will add to is fetched NOW, before the main loop, and held in registers.
    // All workgroups run in lock step (equal tiles, one per CU), so an epilogue that reads and writes the residual would hit
    // HBM with 256 CUs at once while the matrix cores idle; this way only the write is left for the end.  Rows / columns past
    // the matrix edge are clamped (loaded values unused).
    const int m0 = tm * BM + wm * WTM + 4 * q4, n0 = tn * BN + wn * WTN + l16;
    f32x4_t rres[FM][FN];
    if (EPI == LVX_EPI_RESID_GATE_F32) {
        const float *Rf = reinterpret_cast<const float *>(R);
        // rows outermost, column blocks innermost: the FN loads of one row are neighbouring 64-byte runs
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int row = m0 + i * 16 + e;
                row = row < M ? row : M - 1;
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const int col = n0 + j * 16 < N ? n0 + j * 16 : N - 1;
                    rres[i][j][e] = Rf[(size_t)row * ldr + col];
                }
            }
    }

    const int n_k = K / BK;
    const int last = n_k - 1;
    {
        const size_t a_off_ = a_slab(0);
#pragma unroll
        for (int q = 0; q < QPW; ++q) LVX_DMA_ISSUE(0, 0, q);
    }
    {
        const size_t a_off_ = a_slab(last < 1 ? last : 1);
#pragma unroll
        for (int q = 0; q < QPW; ++q) LVX_DMA_ISSUE(1, (last < 1 ? last : 1), q);
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(QPW) : "memory");
    __syncthreads();
    LVX_DMA_READ_A(0, 0, 0, FM);
    LVX_DMA_READ_W(0, 0, 0, FN);

    // Slab t is in stage t % 3.  Per slab four MFMA groups (each k-step as two halves of the accumulator rows): the first three
    // read the fragments still missing for what follows and issue a third of the DMA for slab t+2 each (into the stage that
    // was read during slab t-1); then wait until this wave's DMA for slab t+1 has landed, one workgroup barrier, and the
    // fourth group, which already reads k-step 0 of slab t+1.
    int cur = 0, nxt = 1, nx2 = 2;
    for (int t = 0; t < n_k; ++t) {
        const int kt_load = t + 2 < last ? t + 2 : last;
        const size_t a_off_ = a_slab(kt_load);
        LVX_DMA_READ_W(cur, 1, 0, FN);
        __builtin_amdgcn_sched_barrier(0);
        LVX_DMA_MFMAS(0, 0, FM / 2);
#pragma unroll
        for (int q = 0; q < QPW; ++q)
            if ((q * 3) / QPW == 0) LVX_DMA_ISSUE(nx2, kt_load, q);
        __builtin_amdgcn_sched_barrier(0);
        LVX_DMA_READ_A(cur, 1, 0, FM / 2);
        __builtin_amdgcn_sched_barrier(0);
        LVX_DMA_MFMAS(0, FM / 2, FM);
#pragma unroll
        for (int q = 0; q < QPW; ++q)
            if ((q * 3) / QPW == 1) LVX_DMA_ISSUE(nx2, kt_load, q);
        __builtin_amdgcn_sched_barrier(0);
        LVX_DMA_READ_A(cur, 1, FM / 2, FM);
        __builtin_amdgcn_sched_barrier(0);
        LVX_DMA_MFMAS(1, 0, FM / 2);
#pragma unroll
        for (int q = 0; q < QPW; ++q)
            if ((q * 3) / QPW == 2) LVX_DMA_ISSUE(nx2, kt_load, q);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(QPW) : "memory");
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        LVX_DMA_READ_A(nxt, 0, 0, FM);
        LVX_DMA_READ_W(nxt, 0, 0, FN);
        __builtin_amdgcn_sched_barrier(0);
        LVX_DMA_MFMAS(1, FM / 2, FM);
        __builtin_amdgcn_sched_barrier(0);
        const int tmp = cur;
        cur = nxt;
        nxt = nx2;
        nx2 = tmp;
    }
    // no DMA may still be in flight when the workgroup releases its LDS
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    if (EPI == LVX_EPI_SEGMENTS) {
        if (seg_f32)
            lvx_gemm_epilogue<FM, FN, LVX_EPI_STORE_F32>(acc, rres, C, ldc, R, ldr, gate, M, N, m0, n0);
        else
            lvx_gemm_epilogue<FM, FN, LVX_EPI_STORE>(acc, rres, C, ldc, R, ldr, gate, M, N, m0, n0);
        if (seg_sumsq != nullptr) lvx_gemm_row_sumsq<FM, FN>(acc, seg_sumsq, seg_ld_sumsq, tn * WAVES_N + wn, M, m0, l16);
    } else {
        lvx_gemm_epilogue<FM, FN, EPI>(acc, rres, C, ldc, R, ldr, gate, M, N, m0, n0);
    }
}

// Experiment, compiled only with -DLVX_GEMM_BIG (lvx_linear then uses it for the plain-store and GELU epilogues): 256 x 256 tile,
// 8 waves of 64 x 128 (4 x 2), two 64 KB LDS stages.  Per flop a third fewer bytes go from L2 to LDS and a quarter fewer LDS
// fragment reads than with the 128 x 256 tile.  Slab t lives in stage t & 1.  Per slab one barrier, half-way through the second
// k-step (its fragments are in registers by then); right after it the stage just released takes slab t+2, a whole slab of MFMAs
// ahead of its use, and the first fragments of slab t+1 are read under the remaining MFMAs.  Measured: 5 % faster than the
// 128 x 256 kernel when the tile count is a multiple of 256 (4096 x 16384 x 5120), 7 to 14 % slower on the block's own shapes,
// whose 19 x 60 and 19 x 54 tiles need 5 rounds of the chip where the smaller tile wastes under 4 %.
#ifdef LVX_GEMM_BIG
template <int EPI>
__global__ void __launch_bounds__(512)
    lvx_gemm_big_kernel(const bf16_t *__restrict__ A, int64_t lda, const bf16_t *__restrict__ W, int64_t ldw, bf16_t *C, int64_t ldc,
                        int M, int N, int K, const bf16_t *R, int64_t ldr, const float *__restrict__ gate, int tiles_m, int tiles_n,
                        int per_xcd, lvx_gemm_segs_t segs) {
    constexpr int BM = 256, BN = 256, WAVES_N = 2, NW = 8;
    constexpr int WTM = 64, WTN = 128, FM = 4, FN = 8;
    constexpr int ROW_B = BK * 2;
    constexpr int A_B = BM * ROW_B, STAGE_B = (BM + BN) * ROW_B;
    constexpr int QPW = (BM + BN) / 8 / NW;  // 8 DMA instructions per wave per slab
    constexpr int A_Q = (BM / 8) / NW;       // the first 4 fetch A rows

    __shared__ __attribute__((aligned(1024))) char lds[2 * STAGE_B];

    const int total = tiles_m * tiles_n;
    const int widx = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (widx >= total) return;
    constexpr int GM = 4;  // bands of 4 row tiles: 4 x 8 tiles of an XCD's 32 compute units share 4 A panels and 8 W panels
    const int band = widx / (GM * tiles_n);
    const int first_m = band * GM;
    const int band_m = tiles_m - first_m < GM ? tiles_m - first_m : GM;
    const int in_band = widx - band * GM * tiles_n;
    const int tm = first_m + in_band % band_m;
    int tn = in_band / band_m;
    bool seg_f32 = false;
    if (EPI == LVX_EPI_SEGMENTS) {
        int sg = 0;
        for (int i = 1; i < segs.n; ++i)
            if (tn >= segs.s[i].tn_begin) sg = i;
        tn -= segs.s[sg].tn_begin;
        W = segs.s[sg].W;
        C = reinterpret_cast<bf16_t *>(segs.s[sg].C);
        ldc = segs.s[sg].ldc;
        N = segs.s[sg].N;
        seg_f32 = segs.s[sg].f32 != 0;
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, q4 = lane >> 4;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    uint32_t doff[QPW];
#pragma unroll
    for (int q = 0; q < QPW; ++q) {
        const int row_s = 8 * (wave + NW * q) + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row_s >> 1) & 7);
        if (q < A_Q) {
            int r = tm * BM + row_s;
            if (r > M - 1) r = M - 1;
            doff[q] = (uint32_t)(((size_t)r * lda + chunk * 8) * sizeof(bf16_t));
        } else {
            int r = tn * BN + (row_s - BM);
            if (r > N - 1) r = N - 1;
            doff[q] = (uint32_t)(((size_t)r * ldw + chunk * 8) * sizeof(bf16_t));
        }
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds_base + wave * 1024);
#define LVX_BIG_DMA(stage_, kt_, q_)                                                                                               \
    lvx_dma16(reinterpret_cast<const char *>((q_) < A_Q ? (const void *)A : (const void *)W) + (size_t)(kt_) * ROW_B, doff[q_], \
              lds_wave + (uint32_t)((stage_) * STAGE_B + (q_) * NW * 1024))

    const int swz = (l16 >> 1) & 7;
    const char *a_rd = lds + (wm * WTM + l16) * ROW_B;
    const char *w_rd = lds + A_B + (wn * WTN + l16) * ROW_B;
    bf16x8_t af[2][FM], wf[2][FN];
#define LVX_BIG_READ_A(stage_, ks_, i0_, i1_)                                                                               \
    {                                                                                                                       \
        const int co_ = (((ks_) * 4 + q4) ^ swz) * 16 + (stage_) * STAGE_B;                                                 \
        _Pragma("unroll") for (int i = i0_; i < i1_; ++i) af[(ks_) & 1][i] = *reinterpret_cast<const bf16x8_t *>(a_rd + i * 16 * ROW_B + co_); \
    }
#define LVX_BIG_READ_W(stage_, ks_, j0_, j1_)                                                                               \
    {                                                                                                                       \
        const int co_ = (((ks_) * 4 + q4) ^ swz) * 16 + (stage_) * STAGE_B;                                                 \
        _Pragma("unroll") for (int j = j0_; j < j1_; ++j) wf[(ks_) & 1][j] = *reinterpret_cast<const bf16x8_t *>(w_rd + j * 16 * ROW_B + co_); \
    }
#define LVX_BIG_MFMAS(ks_, i0_, i1_)                                                                         \
    _Pragma("unroll") for (int i = i0_; i < i1_; ++i) _Pragma("unroll") for (int j = 0; j < FN; ++j)         \
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[(ks_) & 1][i], wf[(ks_) & 1][j], acc[i][j], 0, 0, 0);

    f32x4_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

    const int n_k = K / BK;
    const int last = n_k - 1;
#pragma unroll
    for (int q = 0; q < QPW; ++q) LVX_BIG_DMA(0, 0, q);
#pragma unroll
    for (int q = 0; q < QPW; ++q) LVX_BIG_DMA(1, (last < 1 ? last : 1), q);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(QPW) : "memory");
    __syncthreads();
    LVX_BIG_READ_A(0, 0, 0, FM);
    LVX_BIG_READ_W(0, 0, 0, FN);

    for (int t = 0; t < n_k; ++t) {
        const int cur = t & 1, nxt = cur ^ 1;
        const int kt_load = t + 2 < last ? t + 2 : last;  // past the end: a harmless reload of the last slab
        LVX_BIG_READ_W(cur, 1, 0, FN);
        __builtin_amdgcn_sched_barrier(0);
        LVX_BIG_MFMAS(0, 0, 2);
        __builtin_amdgcn_sched_barrier(0);
        LVX_BIG_READ_A(cur, 1, 0, FM);
        __builtin_amdgcn_sched_barrier(0);
        LVX_BIG_MFMAS(0, 2, 4);
        __builtin_amdgcn_sched_barrier(0);
        LVX_BIG_MFMAS(1, 0, 2);
        __builtin_amdgcn_sched_barrier(0);
        // this wave's part of slab t+1 has landed and every wave has read the last fragment of slab t: one barrier, then stage
        // cur takes slab t+2 (a whole slab of MFMAs ahead of its use) and the first fragments of slab t+1 are read
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < QPW; ++q) LVX_BIG_DMA(cur, kt_load, q);
        LVX_BIG_READ_W(nxt, 0, 0, FN);
        LVX_BIG_READ_A(nxt, 0, 0, FM);
        __builtin_amdgcn_sched_barrier(0);
        LVX_BIG_MFMAS(1, 2, 4);
        __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    const int m0 = tm * BM + wm * WTM + 4 * q4, n0 = tn * BN + wn * WTN + l16;
    f32x4_t rres[FM][FN];
    if (EPI == LVX_EPI_SEGMENTS) {
        if (seg_f32)
            lvx_gemm_epilogue<FM, FN, LVX_EPI_STORE_F32>(acc, rres, C, ldc, R, ldr, gate, M, N, m0, n0);
        else
            lvx_gemm_epilogue<FM, FN, LVX_EPI_STORE>(acc, rres, C, ldc, R, ldr, gate, M, N, m0, n0);
    } else {
        lvx_gemm_epilogue<FM, FN, EPI>(acc, rres, C, ldc, R, ldr, gate, M, N, m0, n0);
    }
#undef LVX_BIG_DMA
#undef LVX_BIG_READ_A
#undef LVX_BIG_READ_W
#undef LVX_BIG_MFMAS
}

lvx_status_t launch_big(const bf16_t *A, int64_t lda, const bf16_t *W, int64_t ldw, bf16_t *C, int64_t ldc, int M, int N, int K, int epi,
                        hipStream_t stream, const lvx_gemm_segs_t *seg_table = nullptr) {
    constexpr int BM = 256, BN = 256;
    lvx_gemm_segs_t segs;
    segs.n = 0;
    int tiles_n = (N + BN - 1) / BN;
    if (seg_table != nullptr) {
        segs = *seg_table;
        tiles_n = 0;
        for (int i = 0; i < segs.n; ++i) {
            segs.s[i].tn_begin = tiles_n;
            tiles_n += (segs.s[i].N + BN - 1) / BN;
        }
    }
    const int tiles_m = (M + BM - 1) / BM;
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const dim3 grid(per_xcd * 8), block(512);
#define LVX_BIG_LAUNCH(EPI_)                                                                                                        \
    hipLaunchKernelGGL((lvx_gemm_big_kernel<EPI_>), grid, block, 0, stream, A, lda, W, ldw, C, ldc, M, N, K, (const bf16_t *)nullptr, \
                       (int64_t)0, (const float *)nullptr, tiles_m, tiles_n, per_xcd, segs)
    if (epi == LVX_EPI_STORE) {
        LVX_BIG_LAUNCH(LVX_EPI_STORE);
    } else if (epi == LVX_EPI_GELU_TANH) {
        LVX_BIG_LAUNCH(LVX_EPI_GELU_TANH);
    } else if (epi == LVX_EPI_SEGMENTS) {
        LVX_BIG_LAUNCH(LVX_EPI_SEGMENTS);
    } else {
        return lvx_fail(LVX_ERR_UNSUPPORTED, "256 x 256 tiles: epilogue %d not built", epi);
    }
#undef LVX_BIG_LAUNCH
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}
#endif  // LVX_GEMM_BIG

template <int BM, int BN, int WAVES_M, int WAVES_N, bool CONV = false>
lvx_status_t launch(const bf16_t *A, int64_t lda, const bf16_t *W, int64_t ldw, bf16_t *C, int64_t ldc, int M, int N, int K, int epi,
                    const bf16_t *R, int64_t ldr, const float *gate, hipStream_t stream, const lvx_gemm_segs_t *seg_table = nullptr,
                    const lvx_conv_map_t *conv = nullptr) {
    lvx_conv_map_t cm = {};
    if (conv != nullptr) cm = *conv;
    lvx_gemm_segs_t segs;
    segs.n = 0;
    int tiles_n = (N + BN - 1) / BN;
    if (seg_table != nullptr) {  // column tiles of all segments, one after the other
        segs = *seg_table;
        tiles_n = 0;
        for (int i = 0; i < segs.n; ++i) {
            segs.s[i].tn_begin = tiles_n;
            tiles_n += (segs.s[i].N + BN - 1) / BN;
        }
    }
    const int tiles_m = (M + BM - 1) / BM;
    const int total = tiles_m * tiles_n;
#ifdef LVX_GEMM_NPART
    const int per_xcd = tiles_m * ((tiles_n + 7) / 8);
#else
    const int per_xcd = (total + 7) / 8;
#endif
    const dim3 grid(per_xcd * 8), block(64 * WAVES_M * WAVES_N);
#define LVX_GEMM_LAUNCH(EPI_)                                                                                                      \
    hipLaunchKernelGGL((lvx_gemm_dma_kernel<BM, BN, WAVES_M, WAVES_N, EPI_, CONV>), grid, block, 0, stream, A, lda, W, ldw, C, ldc, M, N, K, \
                       R, ldr, gate, tiles_m, tiles_n, per_xcd, segs, cm)
    if (epi == LVX_EPI_STORE) {
        LVX_GEMM_LAUNCH(LVX_EPI_STORE);
    } else if (epi == LVX_EPI_GELU_TANH) {
        LVX_GEMM_LAUNCH(LVX_EPI_GELU_TANH);
    } else if (epi == LVX_EPI_RESID_GATE) {
        LVX_GEMM_LAUNCH(LVX_EPI_RESID_GATE);
    } else if (epi == LVX_EPI_RESID_GATE_F32) {
        LVX_GEMM_LAUNCH(LVX_EPI_RESID_GATE_F32);
    } else if (epi == LVX_EPI_BIAS) {
        LVX_GEMM_LAUNCH(LVX_EPI_BIAS);
    } else if (epi == LVX_EPI_STORE_F32) {
        LVX_GEMM_LAUNCH(LVX_EPI_STORE_F32);
    } else if (epi == LVX_EPI_SEGMENTS) {
        LVX_GEMM_LAUNCH(LVX_EPI_SEGMENTS);
    } else {
        LVX_GEMM_LAUNCH(LVX_EPI_BIAS_SILU);
    }
#undef LVX_GEMM_LAUNCH
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

}  // namespace

// C1 = A W1^T ([M][N1]) and C2 = A W2^T ([M][N2]) in one launch (same K and weight row stride).  Two uses: two small-M
// projections of the same input fill the chip together where each alone leaves most of it idle (the context's K and V
// projections: 100 tiles each on 256 CUs); and the fused QKV projection with its q | k columns stored in fp32 (they go on to
// the RMSNorm + RoPE kernel, which rounds to bf16 once, after the rotation) and its v columns in bf16.
static lvx_status_t check_dual(const void *A, int64_t lda, const void *W1, const void *W2, int64_t ldw, const void *C1, int64_t ldc1,
                               const void *C2, int64_t ldc2, int M, int N1, int N2, int K) {
    LVX_REQUIRE(A && W1 && W2 && C1 && C2, LVX_ERR_INVALID_ARG, "linear dual: NULL pointer");
    LVX_REQUIRE(lvx_aligned16(A) && lvx_aligned16(W1) && lvx_aligned16(W2) && lvx_aligned16(C1) && lvx_aligned16(C2), LVX_ERR_INVALID_ARG,
                "pointers must be 16-byte aligned");
    LVX_REQUIRE(M >= 0 && N1 > 0 && N2 > 0 && K > 0 && K % BK == 0 && N1 % 8 == 0 && N2 % 8 == 0, LVX_ERR_SHAPE,
                "linear dual: M %d, N1 %d, N2 %d, K %d (K %% 64 == 0, N %% 8 == 0)", M, N1, N2, K);
    LVX_REQUIRE(lda >= K && lda % 8 == 0 && ldw >= K && ldw % 8 == 0 && ldc1 >= N1 && ldc2 >= N2, LVX_ERR_SHAPE, "bad leading dimension");
    const uint64_t n_max = (uint64_t)(N1 > N2 ? N1 : N2);
    LVX_REQUIRE((uint64_t)M * (uint64_t)lda * 2 < (1ull << 32) && n_max * (uint64_t)ldw * 2 < (1ull << 32), LVX_ERR_SHAPE,
                "operand larger than 4 GiB (32-bit byte offsets inside the kernel)");
    return LVX_OK;
}

lvx_status_t lvx_launch_linear_dual(const bf16_t *A, int64_t lda, const bf16_t *W1, const bf16_t *W2, int64_t ldw, void *C1, int64_t ldc1,
                                    int c1_is_f32, bf16_t *C2, int64_t ldc2, int M, int N1, int N2, int K, hipStream_t stream) {
    LVX_TRY(check_dual(A, lda, W1, W2, ldw, C1, ldc1, C2, ldc2, M, N1, N2, K));
    if (M == 0) return LVX_OK;
    lvx_gemm_segs_t segs;
    segs.n = 2;
    segs.s[0] = {W1, C1, ldc1, N1, 0, c1_is_f32 ? 1 : 0, 0};
    segs.s[1] = {W2, C2, ldc2, N2, 0, 0, 0};
    return launch<128, 256, 2, 4>(A, lda, W1, ldw, (bf16_t *)C1, ldc1, M, N1, K, (int)LVX_EPI_SEGMENTS, nullptr, 0, nullptr, stream, &segs);
}

// Up to LVX_GEMM_MAX_SEGS projections of the same activations in one launch (same K, same weight row stride; each with its own
// weight matrix, output, width and row stride; bf16 or fp32 plain store): the context's K and V projections of several layers.
lvx_status_t lvx_launch_linear_segments(const bf16_t *A, int64_t lda, int64_t ldw, const lvx_gemm_segs_t &segs, int M, int K, hipStream_t stream) {
    LVX_REQUIRE(segs.n >= 1 && segs.n <= LVX_GEMM_MAX_SEGS, LVX_ERR_INVALID_ARG, "linear segments: %d segments (1..%d)", segs.n, LVX_GEMM_MAX_SEGS);
    for (int i = 0; i < segs.n; ++i)
        LVX_TRY(check_dual(A, lda, segs.s[i].W, segs.s[i].W, ldw, segs.s[i].C, segs.s[i].ldc, segs.s[i].C, segs.s[i].ldc, M, segs.s[i].N, segs.s[i].N, K));
    for (int i = 0; i < segs.n; ++i)
        LVX_REQUIRE(segs.s[i].sumsq == nullptr || (segs.s[i].N % 256 == 0 && !segs.s[i].f32 && segs.s[i].ld_sumsq >= LVX_GEMM_SUMSQ_PARTS(segs.s[i].N)),
                    LVX_ERR_SHAPE, "linear segments: row sums of squares need a bf16 segment of N %% 256 == 0 and ld_sumsq >= N / 64");
    if (M == 0) return LVX_OK;
    return launch<128, 256, 2, 4>(A, lda, segs.s[0].W, ldw, (bf16_t *)segs.s[0].C, segs.s[0].ldc, M, segs.s[0].N, K, (int)LVX_EPI_SEGMENTS, nullptr, 0,
                                  nullptr, stream, &segs);
}

extern "C" lvx_status_t lvx_linear_dual(const void *dev_a, int64_t lda, const void *dev_w1, const void *dev_w2, int64_t ldw, void *dev_c1,
                                        int64_t ldc1, int32_t c1_is_f32, void *dev_c2, int64_t ldc2, int32_t M, int32_t N1, int32_t N2,
                                        int32_t K, lvx_stream_t stream) {
    return lvx_launch_linear_dual((const bf16_t *)dev_a, lda, (const bf16_t *)dev_w1, (const bf16_t *)dev_w2, ldw, dev_c1, ldc1, c1_is_f32,
                                  (bf16_t *)dev_c2, ldc2, M, N1, N2, K, (hipStream_t)stream);
}

// Implicit-GEMM 3x3x3 convolution: rows = output pixels, K = 27 taps x C channels gathered from the padded volume P.
// 256 x 128 tiles (C_out is 128 ... 512 in the decoder this serves; 128-wide column tiles waste nothing there).
lvx_status_t lvx_launch_conv_gemm(const bf16_t *P, const lvx_conv_map_t &cm, const bf16_t *Wt, int64_t ldw, const float *bias, int act,
                                  bf16_t *Y, int64_t ldy, int M, int N, hipStream_t stream) {
    const int K = 27 * cm.C;
    return launch<256, 128, 4, 2, true>(P, 0, Wt, ldw, Y, ldy, M, N, K, act ? (int)LVX_EPI_BIAS_SILU : (int)LVX_EPI_BIAS, nullptr, 0, bias, stream,
                                        nullptr, &cm);
}

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
    LVX_REQUIRE((int)epi >= (int)LVX_EPI_STORE && (int)epi <= (int)LVX_EPI_STORE_F32, LVX_ERR_INVALID_ARG, "unknown epilogue %d", (int)epi);
    if (epi == LVX_EPI_RESID_GATE || epi == LVX_EPI_RESID_GATE_F32) {
        LVX_REQUIRE(dev_resid != nullptr, LVX_ERR_INVALID_ARG, "residual epilogue needs a residual pointer");
        LVX_REQUIRE(ldr >= N, LVX_ERR_SHAPE, "bad residual leading dimension");
    }
    if (M == 0) return LVX_OK;
#ifdef LVX_GEMM_BIG
    if (epi == LVX_EPI_STORE || epi == LVX_EPI_GELU_TANH)
        return launch_big((const bf16_t *)dev_a, lda, (const bf16_t *)dev_w, ldw, (bf16_t *)dev_c, ldc, M, N, K, (int)epi, (hipStream_t)stream);
#endif
    return launch<128, 256, 2, 4>((const bf16_t *)dev_a, lda, (const bf16_t *)dev_w, ldw, (bf16_t *)dev_c, ldc, M, N, K, (int)epi,
                                  (const bf16_t *)dev_resid, ldr, dev_gate, (hipStream_t)stream);
}
