// Chunk-to-cache attention for gfx950: O = softmax(scale * Q K^T) V over the visible key prefix, no mask
// (paper Eq. 1 and the mask rule of Sec. 3.2: everything in the cache is visible to the current block).
//
// Design (MI355X-first, not the Hopper kernels the paper names):
//   * one workgroup = one head x (32*NWAVES) queries; each 64-lane wave owns 32 queries and the full head_dim.
//   * scores are produced TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: in that accumulator layout a lane
//     holds scores of ONE query (column lane%32) for 16 keys per 32-key block, so the online-softmax statistics are
//     per-lane scalars (one cross-half exchange per tile) and the exponentiated scores are already in the B-operand
//     layout of the second MFMA, O^T += V^T P^T, with no LDS round trip.
//   * K tiles ([64 keys][D]) and V^T tiles ([D][64 keys], stored transposed in the cache) go global -> LDS directly
//     (global_load_lds_dwordx4, no staging registers) into rings of four tiles each; rows are XOR-swizzled so that 16
//     consecutive lanes reading 16 bytes each hit disjoint banks.
//   * the two waves of each SIMD are run half a period apart (matrix phase against vector phase, see "pipeline" below),
//     so the softmax VALU work of one wave hides under the MFMA work of the other.
//   * K rows are placed in LDS in the order the accumulator layout wants (lane i of the A operand reads LDS row i),
//     which makes each half-wave's 16 scores per block belong to 16 CONSECUTIVE keys, so V^T fragments are
//     contiguous 16-byte reads.
//   * the vector phase competes with the other wave's MFMA issue for the SIMD's one VALU port, so it is kept short: the
//     reference value that online softmax subtracts only has to keep exp2 in range, so no per-tile maximum is taken.  The
//     reference is the first tile's row maximum; a tile whose sum of exponentials reaches 2^64 (or overflows) is redone
//     with its own maximum as the new reference and the O accumulators rescaled (wave-uniform branch, practically never
//     taken after the first tile); the final division by the row sum absorbs whatever reference was used.
//   * workgroup -> (head, query tile) mapping keeps all query tiles of a head on one XCD (hardware deals consecutive
//     workgroup ids round-robin over the 8 XCDs), so a head's K/V stream is fetched into one L2 only.
#include "lvx_internal.h"

namespace {

constexpr int KT = LVX_KEY_TILE;

template <int D, int NWAVES>
__global__ void __launch_bounds__(64 * NWAVES)
    lvx_attention_kernel(const bf16_t *__restrict__ q, int64_t ld_q, int n_q, const bf16_t *__restrict__ kp,
                         const bf16_t *__restrict__ vtp, int cap, int n_keys, float c_exp2, bf16_t *__restrict__ out,
                         int64_t ld_out, int n_qtiles, int total_wg, int per_xcd, uint32_t *amax_slots) {
    constexpr int QT = 32 * NWAVES;
    constexpr int MK = D / 16;  // MFMA k-steps over head_dim
    constexpr int DB = D / 32;  // 32-row blocks of O^T
    constexpr int NV = DB * 4;  // V^T fragments (= PV MFMAs) per 64-key tile
    constexpr int NK = 2 * MK;  // K fragments (= QK MFMAs) per 64-key tile
    constexpr int PD = 6;       // LDS fragment prefetch distance, in MFMAs
    // LDS: a ring of NS K tiles ([64 keys][D], rows of D*2 bytes) and a ring of NS V^T tiles ([D][64 keys], rows of 128 bytes),
    // filled by direct-to-LDS loads.  A DMA wave-instruction writes 1024 contiguous bytes, so rows cannot be padded; a 16-byte
    // chunk c of row r is stored at position c ^ swz(r) instead (the lane fetches the matching global chunk), with
    // swz(r) = r & 15 for 256-byte rows and (r >> 1) & 7 for 128-byte rows: 16 consecutive rows then hit 16 distinct
    // 16-byte units of a 256-byte bank row.
    constexpr int NS = 4;
    constexpr int TILE_B = KT * D * 2;        // bytes per K tile = per V^T tile
    constexpr int K_ROW_B = D * 2;
    constexpr int K_RPI = 1024 / K_ROW_B;     // K rows per DMA instruction (4 or 8)
    constexpr int K_CPR = D / 8;              // 16-byte chunks per K row (16 or 8)
    constexpr int N_DMA = TILE_B / 1024;      // DMA instructions per tile (K and V^T alike)
    static_assert(N_DMA % NWAVES == 0, "DMA instructions must divide over the waves");
    constexpr int DPW = N_DMA / NWAVES;       // per wave, per tile
    constexpr int V_ROW_B = KT * 2;           // 128

    __shared__ __attribute__((aligned(1024))) char ks[NS * TILE_B];
    __shared__ __attribute__((aligned(1024))) char vs[NS * TILE_B];

    // XCD-aware decode: consecutive block ids go to consecutive XCDs; give each XCD a contiguous range of work
    const int xcd = blockIdx.x & 7;
    const int widx = xcd * per_xcd + (blockIdx.x >> 3);
    if (widx >= total_wg) return;
    const int head = widx / n_qtiles;
    const int qtile = widx % n_qtiles;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;

    // Q fragments (B operand of S^T = K Q^T): lane holds Q[query l32][d = 16m + 8hh .. +7]
    bf16x8_t qf[MK];
    {
        int row = qtile * QT + wave * 32 + l32;
        if (row > n_q - 1) row = n_q - 1;
        const bf16_t *qp = q + (size_t)row * ld_q + (size_t)head * D + hh * 8;
#pragma unroll
        for (int m = 0; m < MK; ++m) qf[m] = *reinterpret_cast<const bf16x8_t *>(qp + 16 * m);
    }

    const int n_tiles = (n_keys + KT - 1) / KT;
    const char *k_src = reinterpret_cast<const char *>(kp + (size_t)head * cap * D);   // K tile t at k_src + t * TILE_B
    const char *v_src = reinterpret_cast<const char *>(vtp + (size_t)head * cap * D);  // V^T tile t at v_src + t * TILE_B

    // ---- staging (direct to LDS) -----------------------------------------------------------------------------------------
    // DMA instruction e of this wave covers LDS rows [rows_per_instr * (wave + NWAVES*e), +rows_per_instr) of a tile.
    // K: LDS row rr holds key r(rr) (accumulator-row order: key r = 32*blk + 16h + 4g + r4 sits at LDS row 32*blk + 8g + 4h + r4,
    // which makes each half-wave's 16 scores per block belong to 16 consecutive keys).
    uint32_t kdoff[DPW], vdoff[DPW];
#pragma unroll
    for (int e = 0; e < DPW; ++e) {
        const int j = wave + NWAVES * e;
        {
            const int rr = K_RPI * j + lane / K_CPR;  // LDS row
            const int pos = lane % K_CPR;
            const int key = (rr & 32) | (((rr >> 2) & 1) << 4) | (((rr >> 3) & 3) << 2) | (rr & 3);
            const int swz = K_CPR == 16 ? (rr & 15) : ((rr >> 1) & 7);
            kdoff[e] = (uint32_t)(key * K_ROW_B + (pos ^ swz) * 16);
        }
        {
            const int rr = 8 * j + (lane >> 3);  // LDS row = head-dim index d
            const int pos = lane & 7;
            vdoff[e] = (uint32_t)(rr * V_ROW_B + (pos ^ ((rr >> 1) & 7)) * 16);
        }
    }
    const uint32_t ks_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)ks;
    const uint32_t vs_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)vs;
    const uint32_t ks_wave = __builtin_amdgcn_readfirstlane(ks_base + wave * 1024);
    const uint32_t vs_wave = __builtin_amdgcn_readfirstlane(vs_base + wave * 1024);
    const int last_tile = n_tiles - 1;
#define LVX_ATTN_DMA_K(t_)                                                                                                  \
    {                                                                                                                       \
        const int tt_ = (t_) < last_tile ? (t_) : last_tile;                                                                \
        _Pragma("unroll") for (int e = 0; e < DPW; ++e)                                                                     \
            lvx_dma16(k_src + (size_t)tt_ * TILE_B, kdoff[e], ks_wave + (uint32_t)(((t_) & (NS - 1)) * TILE_B + e * NWAVES * 1024)); \
    }
#define LVX_ATTN_DMA_V(t_)                                                                                                  \
    {                                                                                                                       \
        const int tt_ = (t_) < last_tile ? (t_) : last_tile;                                                                \
        _Pragma("unroll") for (int e = 0; e < DPW; ++e)                                                                     \
            lvx_dma16(v_src + (size_t)tt_ * TILE_B, vdoff[e], vs_wave + (uint32_t)(((t_) & (NS - 1)) * TILE_B + e * NWAVES * 1024)); \
    }
    // stage u = { V^T(u), K(u+1) }: what the matrix phase X(u) reads
#define LVX_ATTN_STAGE_DMA(u_) \
    {                          \
        LVX_ATTN_DMA_V(u_);    \
        LVX_ATTN_DMA_K((u_) + 1); \
    }
#define LVX_ATTN_WAIT_DMA(n_) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n_) : "memory")

    // fragment read offsets inside a tile (bytes): K fragment m of 32-key block kb: row kb*32 + l32, chunk (2m + hh) ^ swz;
    // V^T fragment (db, kb, mm): row db*32 + l32, chunk (4kb + 2hh + mm) ^ swz
    const int k_swz = K_CPR == 16 ? (l32 & 15) : ((l32 >> 1) & 7);
    const int v_swz = (l32 >> 1) & 7;
    int kfo[MK], vfo[4];
#pragma unroll
    for (int m = 0; m < MK; ++m) kfo[m] = l32 * K_ROW_B + (((2 * m + hh) ^ k_swz) * 16);
#pragma unroll
    for (int c = 0; c < 4; ++c) vfo[c] = l32 * V_ROW_B + ((((c >> 1) * 4 + 2 * hh + (c & 1)) ^ v_swz) * 16);

    // ---- pipeline -------------------------------------------------------------------------------------------------
    // A wave alternates between a matrix phase X(t) = { O += V(t)^T P(t) ; S(t+1) = K(t+1) Q^T } (MFMAs fed from LDS)
    // and a vector phase Y(t) = online softmax of S(t) -> P(t).  The two waves that share a SIMD (wave w and
    // w + NWAVES/2) run half a period apart, with a workgroup barrier after every phase: while group 0 is in X the
    // other is in Y, so the matrix core and the vector ALU of each SIMD are busy at the same time.
    //   iteration i, first half :  group 0: X(i-1) (S(0) only before the loop)  group 1: Y(i-1)
    //   iteration i, second half:  group 0: Y(i)                                group 1: X(i-1)
    // Staging: every wave issues the DMA of stage i+2 at the end of the first half of iteration i and, before the second
    // half's barrier, waits until its own DMA of stage i has landed (two younger stages may still be in flight); stage i
    // is first read by group 0 in X(i), right after that barrier.  Stage i-2, whose ring slots stage i+2 overwrites, was
    // last read in the second half of iteration i-1 (group 1's X(i-2)), which ended at a barrier before the issue.
    const int grp = wave / (NWAVES / 2);

    f32x16_t o[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[i][j] = 0.f;
    float mc = 0.f;  // the reference the softmax subtracts (a row maximum, already multiplied by c_exp2); set by the first tile
    float l_run = 0.f;
    f32x16_t s[2];
    bf16x8_t pb[2][2];

    // S(0) = K(0) Q^T from K slot 0 (prologue of the pipeline; the steady state computes S inside LVX_ATTN_X)
#define LVX_ATTN_S0()                                                                                          \
    {                                                                                                          \
        _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) {                                                     \
            _Pragma("unroll") for (int j = 0; j < 16; ++j) s[kb][j] = 0.f;                                     \
            bf16x8_t a[MK];                                                                                    \
            _Pragma("unroll") for (int m = 0; m < MK; ++m)                                                     \
                a[m] = *reinterpret_cast<const bf16x8_t *>(ks + kb * 32 * K_ROW_B + kfo[m]);                   \
            _Pragma("unroll") for (int m = 0; m < MK; ++m)                                                     \
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m], qf[m], s[kb], 0, 0, 0);                  \
        }                                                                                                      \
    }
    // Matrix phase X(j): O^T += V(j)^T P(j)^T from V slot j%NS, then S(j+1) = K(j+1) Q^T from K slot (j+1)%NS (past the last
    // tile the slot holds a copy of the last tile; that S is never used).  One basic block of NV + NK MFMAs, each fed by one
    // 16-byte LDS fragment.  The fragment reads run PD MFMAs ahead of their use through a ring of PD registers, and the
    // scheduler is told to keep that order (PD reads, then MFMA / read pairs, then PD MFMAs), so an MFMA never waits for a
    // read issued just before it.  Consecutive MFMAs target different accumulators (round robin over the DB blocks of O^T,
    // then over the two 32-key blocks of S), so none has to wait for the previous one's result.
    //   fragment f < NV :  r = f / DB: V^T rows 32*(f%DB).., key chunk (r/2, r%2)   -> o[f%DB] += frag * pb[r/2][r%2]
    //   fragment f >= NV:  g = f - NV: K rows 32*(g%2).., dims 16*(g/2) ..          -> s[g%2] += frag * qf[g/2]
#define LVX_ATTN_FRAG(f_)                                                                                              \
    ((f_) < NV ? *reinterpret_cast<const bf16x8_t *>(vr + ((f_) % DB) * 32 * V_ROW_B + vfo[((f_) / DB) & 3])            \
               : *reinterpret_cast<const bf16x8_t *>(kr + (((f_) - NV) & 1) * 32 * K_ROW_B + kfo[(((f_) - NV) >> 1) % MK]))
#define LVX_ATTN_X(j_)                                                                                         \
    {                                                                                                          \
        __builtin_amdgcn_s_setprio(2); /* the matrix phase wins instruction arbitration over the other wave's VALU */ \
        const char *vr = vs + ((j_) & (NS - 1)) * TILE_B;                                                      \
        const char *kr = ks + (((j_) + 1) & (NS - 1)) * TILE_B;                                                \
        bf16x8_t fr[PD];                                                                                       \
        _Pragma("unroll") for (int f = 0; f < PD; ++f) fr[f] = LVX_ATTN_FRAG(f);                               \
        _Pragma("unroll") for (int j = 0; j < 16; ++j) s[0][j] = 0.f;                                          \
        _Pragma("unroll") for (int j = 0; j < 16; ++j) s[1][j] = 0.f;                                          \
        _Pragma("unroll") for (int f = 0; f < NV + NK; ++f) {                                                  \
            const bf16x8_t a = fr[f % PD];                                                                     \
            if (f + PD < NV + NK) fr[f % PD] = LVX_ATTN_FRAG(f + PD);                                          \
            if (f < NV)                                                                                        \
                o[f % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[((f / DB) >> 1) & 1][(f / DB) & 1], o[f % DB], 0, 0, 0); \
            else                                                                                               \
                s[(f - NV) & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[(f - NV) >> 1], s[(f - NV) & 1], 0, 0, 0); \
        }                                                                                                      \
        __builtin_amdgcn_sched_group_barrier(0x100, PD, 0);                                                    \
        _Pragma("unroll") for (int f = 0; f < NV + NK - PD; ++f) {                                             \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                 \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                 \
        }                                                                                                      \
        __builtin_amdgcn_sched_group_barrier(0x008, PD, 0);                                                    \
    }
    // vector phase: accumulator register v of block kb holds key  t*64 + kb*32 + 16*hh + v  for query l32
#define LVX_ATTN_Y(t_)                                                                                         \
    {                                                                                                          \
        __builtin_amdgcn_s_setprio(0); /* the matrix phase's priority is kept through its DMA issue, up to here */ \
        if ((t_) == n_tiles - 1 && (n_keys % KT) != 0) {                                                       \
            int lim_ = n_keys - (t_) * KT - 16 * hh; /* keys of this lane's first block that are valid */      \
            asm volatile("" : "+v"(lim_));           /* keep the 32 compares out of the loop preheader */      \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) _Pragma("unroll") for (int v = 0; v < 16; ++v)    \
                if (kb * 32 + v >= lim_) s[kb][v] = -INFINITY;                                                 \
        }                                                                                                      \
        /* The reference mc only has to keep exp2 inside the fp32 range, so no per-tile maximum is taken: mc is the first     \
           tile's row maximum, and a later tile whose sum of exponentials reaches 2^64 (or overflows) is redone with its own   \
           maximum as the new reference and the accumulators rescaled.  Both half-waves of a query decide together           \
           (wave-wide vote); the final division by the row sum absorbs whatever reference was used. */                     \
        float lsum;                                                                                            \
        bool rebase_ = (t_) == 0;                                                                              \
        for (;;) {                                                                                             \
            if (rebase_) {                                                                                     \
                float tmax = s[0][0];                                                                          \
                _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) _Pragma("unroll") for (int v = 0; v < 16; ++v) \
                    tmax = fmaxf(tmax, s[kb][v]);                                                              \
                {   /* the other half-wave holds the same query's other 32 keys */                             \
                    const auto sw_ = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false); \
                    tmax = fmaxf(__uint_as_float(sw_[0]), __uint_as_float(sw_[1]));                            \
                }                                                                                              \
                const bool first_ = (t_) == 0;                                                                 \
                const float tmc = tmax * c_exp2;                                                               \
                const bool need = first_ || tmc > mc + 6.0f;                                                   \
                const float alpha = (need && !first_) ? __builtin_amdgcn_exp2f(mc - tmc) : 1.0f;               \
                if (need) mc = tmc;                                                                            \
                l_run *= alpha;                                                                                \
                _Pragma("unroll") for (int i = 0; i < DB; ++i) _Pragma("unroll") for (int j = 0; j < 16; ++j)  \
                    o[i][j] *= alpha;                                                                          \
            }                                                                                                  \
            lsum = 0.f;                                                                                        \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) _Pragma("unroll") for (int v = 0; v < 16; ++v) {  \
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][v], c_exp2, -mc));                 \
                lsum += p;                                                                                     \
                pb[kb][v >> 3][v & 7] = (__bf16)p;                                                             \
            }                                                                                                  \
            if (rebase_ || !__any(!(lsum < 0x1p64f))) break;                                                   \
            rebase_ = true;                                                                                    \
        }                                                                                                      \
        l_run += lsum;                                                                                         \
    }

    LVX_ATTN_DMA_K(0);
    LVX_ATTN_STAGE_DMA(0);
    LVX_ATTN_STAGE_DMA(1);
    LVX_ATTN_WAIT_DMA(4 * DPW);  // K(0) landed; stages 0 and 1 may be in flight
    __syncthreads();

    // Each group runs its own straight-line loop; both execute the same number of barriers (2 per iteration) and the same
    // DMA issue / wait sequence (issue in the first half, wait in the second half of every iteration).
    // A wave whose 32 queries all lie past n_q (ragged last query tile: 4680 = 18 x 256 + 72) only keeps up the DMA and
    // barrier protocol: no LDS reads, no MFMAs, no softmax.  Its SIMD partner then has the matrix core to itself, so such a
    // workgroup finishes early and frees its CU, and the padding costs no energy on a chip that is power-limited.
    const bool active = __builtin_amdgcn_readfirstlane(qtile * QT + wave * 32) < n_q;
    if (!active) {
        __syncthreads();
        LVX_ATTN_STAGE_DMA(2);
        LVX_ATTN_WAIT_DMA(4 * DPW);
        __syncthreads();
        for (int i = 1; i < n_tiles; ++i) {
            LVX_ATTN_STAGE_DMA(i + 2);
            __syncthreads();
            LVX_ATTN_WAIT_DMA(4 * DPW);
            __syncthreads();
        }
        __syncthreads();
        __syncthreads();
    } else if (grp == 0) {
        LVX_ATTN_S0();
        __syncthreads();
        LVX_ATTN_Y(0);
        LVX_ATTN_STAGE_DMA(2);
        LVX_ATTN_WAIT_DMA(4 * DPW);  // stage 0 landed
        __syncthreads();
        for (int i = 1; i < n_tiles; ++i) {
            LVX_ATTN_X(i - 1);
            LVX_ATTN_STAGE_DMA(i + 2);
            __syncthreads();
            LVX_ATTN_Y(i);
            LVX_ATTN_WAIT_DMA(4 * DPW);  // stage i landed
            __syncthreads();
        }
        LVX_ATTN_X(n_tiles - 1);
        __syncthreads();
        __syncthreads();
    } else {
        __syncthreads();
        LVX_ATTN_S0();
        LVX_ATTN_STAGE_DMA(2);
        LVX_ATTN_WAIT_DMA(4 * DPW);
        __syncthreads();
        for (int i = 1; i <= n_tiles; ++i) {
            LVX_ATTN_Y(i - 1);
            if (i < n_tiles) LVX_ATTN_STAGE_DMA(i + 2);
            __syncthreads();
            LVX_ATTN_X(i - 1);
            if (i < n_tiles) LVX_ATTN_WAIT_DMA(4 * DPW);
            __syncthreads();
        }
    }
    LVX_ATTN_WAIT_DMA(0);  // no DMA may still be in flight when the workgroup releases its LDS

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.0f / l_tot;
    const int row = qtile * QT + wave * 32 + l32;
    uint32_t amax_b = 0;  // largest magnitude among the bf16 values this lane stores (bit pattern without sign)
    if (row < n_q) {
        bf16_t *op = out + (size_t)row * ld_out + (size_t)head * D;
        // accumulator register 4g+r of block db holds O^T[d = 32db + 8g + 4hh + r][query l32]
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 w;
                w.x = pack_bf16x2(o[db][4 * g + 0] * inv, o[db][4 * g + 1] * inv);
                w.y = pack_bf16x2(o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv);
                *reinterpret_cast<uint2 *>(op + 32 * db + 8 * g + 4 * hh) = w;
                if (amax_slots != nullptr) {
                    const uint32_t a0 = w.x & 0x7fffu, a1 = (w.x >> 16) & 0x7fffu, a2 = w.y & 0x7fffu, a3 = (w.y >> 16) & 0x7fffu;
                    uint32_t m = a0 > a1 ? a0 : a1;
                    m = m > a2 ? m : a2;
                    m = m > a3 ? m : a3;
                    amax_b = amax_b > m ? amax_b : m;
                }
            }
    }
    // the output feeds an FP8 linear: hand its amax to that linear's quantisation (one atomic per wave)
    if (amax_slots != nullptr) {
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) {
            const uint32_t o2 = (uint32_t)__shfl_xor((int)amax_b, s);
            amax_b = amax_b > o2 ? amax_b : o2;
        }
        if (lane == 0 && amax_b != 0) atomicMax(amax_slots + ((widx * NWAVES + wave) & (LVX_AMAX_SLOTS - 1)), amax_b << 16);
    }
}

template <int D, int NWAVES>
lvx_status_t launch(const bf16_t *q, int64_t ld_q, int n_q, int H, const bf16_t *kp, const bf16_t *vtp, int cap, int n_keys,
                    float scale, bf16_t *out, int64_t ld_out, hipStream_t stream, uint32_t *amax_slots) {
    constexpr int QT = 32 * NWAVES;
    const int n_qtiles = (n_q + QT - 1) / QT;
    const int total = n_qtiles * H;
    const int per_xcd = (total + 7) / 8;
    const float c = scale * 1.4426950408889634f;
    hipLaunchKernelGGL((lvx_attention_kernel<D, NWAVES>), dim3(per_xcd * 8), dim3(64 * NWAVES), 0, stream, q, ld_q, n_q, kp, vtp, cap,
                       n_keys, c, out, ld_out, n_qtiles, total, per_xcd, amax_slots);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

}  // namespace

lvx_status_t lvx_launch_attention(const bf16_t *q, int64_t ld_q, int n_q, int H, int D, const bf16_t *k_packed,
                                  const bf16_t *vt_packed, int cap, int n_keys, float scale, bf16_t *out, int64_t ld_out,
                                  hipStream_t stream, uint32_t *amax_slots) {
    LVX_REQUIRE(n_q > 0 && n_keys > 0 && n_keys <= cap && cap % KT == 0, LVX_ERR_SHAPE, "attention: n_q %d, n_keys %d, cap %d", n_q,
                n_keys, cap);
    LVX_REQUIRE(scale > 0.f, LVX_ERR_INVALID_ARG, "attention: scale must be positive");
    if (D == 128) return launch<128, 8>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots);
    if (D == 64) return launch<64, 8>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots);
    return lvx_fail(LVX_ERR_UNSUPPORTED, "head_dim %d not supported (64 or 128)", D);
}

extern "C" lvx_status_t lvx_chunk_attention(const lvx_kvcache_t *c, int32_t layer, const void *dev_q, int64_t ld_q, int32_t n_q,
                                            float scale, void *dev_out, int64_t ld_out, lvx_stream_t stream) {
    LVX_REQUIRE(c != nullptr, LVX_ERR_INVALID_ARG, "cache handle is NULL");
    LVX_REQUIRE(layer >= 0 && layer < c->desc.n_layers, LVX_ERR_INVALID_ARG, "layer %d out of range [0,%d)", layer, c->desc.n_layers);
    LVX_REQUIRE(dev_q != nullptr && dev_out != nullptr, LVX_ERR_INVALID_ARG, "q or out is NULL");
    LVX_REQUIRE(lvx_aligned16(dev_q) && lvx_aligned16(dev_out), LVX_ERR_INVALID_ARG, "q and out must be 16-byte aligned");
    const int64_t d = (int64_t)c->desc.n_heads * c->desc.head_dim;
    LVX_REQUIRE(ld_q >= d && ld_q % 8 == 0 && ld_out >= d && ld_out % 8 == 0, LVX_ERR_SHAPE,
                "row strides must be multiples of 8 and >= n_heads*head_dim");
    LVX_REQUIRE(n_q > 0, LVX_ERR_SHAPE, "n_q %d must be positive", n_q);
    LVX_REQUIRE(scale > 0.f, LVX_ERR_INVALID_ARG, "scale must be positive");
    const lvx_ring_state_t &s = c->state[layer];
    LVX_REQUIRE(s.key_count > 0, LVX_ERR_STATE, "layer %d has no visible keys (set the sink / append a chunk first)", layer);
    LVX_REQUIRE(c->sink_t[layer] != LVX_SINK_STALE, LVX_ERR_STATE,
                "layer %d: the sink was reset and its keys are not rotated yet (lvx_sink_rope_update)", layer);
    return lvx_launch_attention((const bf16_t *)dev_q, ld_q, n_q, c->desc.n_heads, c->desc.head_dim, lvx_cache_k(c, layer),
                                lvx_cache_vt(c, layer), c->cap_keys, s.key_count, scale, (bf16_t *)dev_out, ld_out, (hipStream_t)stream);
}
