// Chunk-to-cache attention for gfx950: O = softmax(scale * Q K^T) V over the visible key prefix, no mask
// (paper Eq. 1 and the mask rule of Sec. 3.2: everything in the cache is visible to the current block).
//
// Design (MI355X-first, not the Hopper kernels the paper names):
//   * one workgroup = one head x (32*NWAVES) queries; each 64-lane wave owns 32 queries (two blocks of 16) and the full
//     head_dim.
//   * scores are produced TRANSPOSED, S^T = K Q^T, with v_mfma_f32_16x16x32_bf16 (a fifth less register-file traffic per
//     flop than 32x32x16 and 4 % faster here, the chip being power-limited): in that accumulator layout a lane holds
//     scores of ONE query per 16-query block (column lane%16) for 4 keys per 16-key block, so the softmax statistics are
//     per-lane scalars (combined across the four lane groups of a query only at the end and in the rare re-base), and the
//     exponentiated scores are already in the B-operand layout of the second MFMA, O^T += V^T P^T, with no LDS round trip.
//   * K tiles ([64 keys][D]) and V^T tiles ([D][64 keys], stored transposed in the cache) go global -> LDS directly
//     (global_load_lds_dwordx4, no staging registers) into rings of four tiles each; rows are XOR-swizzled so that 16
//     consecutive lanes reading 16 bytes each hit disjoint banks.
//   * the two waves of each SIMD are run half a period apart (matrix phase against vector phase, see "pipeline" below),
//     so the softmax VALU work of one wave hides under the MFMA work of the other.
//   * K rows are placed in LDS in the order the accumulator layout wants, which makes the 8 scores a lane group holds per
//     32-key MFMA step belong to 8 CONSECUTIVE keys, so V^T fragments are contiguous 16-byte reads.
//   * the vector phase competes with the other wave's MFMA issue for the SIMD's one VALU port, so it is kept short: the
//     reference value that online softmax subtracts only has to keep exp2 in range, so no per-tile maximum is taken.  The
//     reference is the first tile's row maximum; a tile whose sum of exponentials reaches 2^64 (or overflows) is redone
//     with its own maximum as the new reference and the O accumulators rescaled (wave-uniform branch, practically never
//     taken after the first tile); the final division by the row sum absorbs whatever reference was used.
//   * workgroup -> (head, query tile) mapping keeps all query tiles of a head on one XCD (hardware deals consecutive
//     workgroup ids round-robin over the 8 XCDs), so a head's K/V stream is fetched into one L2 only.
//   * template switches: TP = 64-key tiles per pipeline phase (2 from 1024 visible keys on: half the barriers, pipeline fills and
//     drains per key); PRE = the queries arrive multiplied by scale * log2(e) and the score accumulators start at minus the
//     softmax reference, so a score leaves the MFMA as the exponent (one FMA per score less; used inside a block, where the
//     RoPE kernel applies the factor before its one rounding); QN = the kernel itself applies the queries' RMSNorm, gain and
//     that factor as it loads them (cross-attention inside a block: no norm-only pass over q).
#include "lvx_internal.h"

namespace {

constexpr int KT = LVX_KEY_TILE;
// from this many visible keys on, a phase of the pipeline covers two 64-key tiles instead of one (measured: 3 % slower at 544
// keys, equal at 1560, 3 to 4 % faster from 6240 keys on)
constexpr int TP2_MIN_KEYS = 16 * KT;

template <int D, int NWAVES, int QB = 2, int TP = 1, bool PRE = false, bool QN = false>
__global__ void __launch_bounds__(64 * NWAVES) __attribute__((amdgpu_waves_per_eu(2, 2)))
    lvx_attention_kernel(const bf16_t *__restrict__ q, int64_t ld_q, int n_q, const bf16_t *__restrict__ kp,
                         const bf16_t *__restrict__ vtp, int cap, int n_keys, float c_exp2, bf16_t *__restrict__ out,
                         int64_t ld_out, int n_qtiles, int total_wg, int per_xcd, uint32_t *amax_slots, lvx_attn_qnorm_t qn) {
    constexpr int QT = 16 * QB * NWAVES;  // QB blocks of 16 queries per wave
    constexpr int MK = D / 32;  // MFMA k-steps (32 wide) over head_dim
    constexpr int DB = D / 16;  // 16-row blocks of O^T
    constexpr int NV = DB * 2;  // V^T fragments per 64-key tile (each feeds two PV MFMAs, one per 16-query block)
    constexpr int NK = 4 * MK;  // K fragments per 64-key tile (each feeds two QK MFMAs)
    constexpr int PD = 4;       // LDS fragment prefetch distance, in fragments (2, 3, 6, 8, 10 measured: 4 is best by 1 %)
    // LDS: a ring of NS K tiles ([64 keys][D], rows of D*2 bytes) and a ring of NS V^T tiles ([D][64 keys], rows of 128 bytes),
    // filled by direct-to-LDS loads.  A DMA wave-instruction writes 1024 contiguous bytes, so rows cannot be padded; a 16-byte
    // chunk c of row r is stored at position c ^ swz(r) instead (the lane fetches the matching global chunk), with
    // swz(r) = r & 15 for 256-byte rows and (r >> 1) & 7 for 128-byte rows: 16 consecutive rows then hit 16 distinct
    // 16-byte units of a 256-byte bank row.
    constexpr int NS = NWAVES == 4 ? 2 : 4;  // two stages of TP tiles each (the 8-wave form keeps four slots at TP = 1 as well)
    static_assert(NS >= 2 * TP && (TP == 1 || TP == 2), "two stages of TP tiles must fit the ring");
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
    const int l16 = lane & 15, q4 = lane >> 4;

    // Q fragments (B operand of S^T = K Q^T, v_mfma_f32_16x16x32_bf16): for query block qb, lane (l16, q4) holds
    // Q[query 16qb + l16][d = 32m + 8q4 .. +7]
    bf16x8_t qf[QB][MK];
    float ss_row = 0.f;
    if (QN) {
        // lane L adds one half (L & 1) of the partial sums of query row L / 2 of this wave: contiguous 16-byte loads, all issued
        // before the first add, in a fixed order (the result is bit-reproducible); the two halves meet through one shuffle
        int r = qtile * QT + wave * 32 + (lane >> 1);
        if (r > n_q - 1) r = n_q - 1;
        const int per4 = qn.n_parts / 8;  // float4 loads per lane, at most 16 (d_model <= 8192)
        const float4 *pp = reinterpret_cast<const float4 *>(qn.sumsq + (size_t)r * qn.ld + (lane & 1) * (qn.n_parts / 2));
        float4 part[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) part[i] = i < per4 ? pp[i] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int i = 0; i < 16; ++i) ss_row += (part[i].x + part[i].y) + (part[i].z + part[i].w);
        ss_row += __shfl_xor(ss_row, 1);
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int row = qtile * QT + wave * (16 * QB) + 16 * qb + l16;
        if (row > n_q - 1) row = n_q - 1;
        const bf16_t *qp = q + (size_t)row * ld_q + (size_t)head * D + q4 * 8;
#pragma unroll
        for (int m = 0; m < MK; ++m) qf[qb][m] = *reinterpret_cast<const bf16x8_t *>(qp + 32 * m);
        if (QN) {
            // RMSNorm of the query row over all d_model channels, its gain and the logit scale, applied in fp32 to the bf16
            // projection output and rounded once.  ss_row (computed once per wave, above) holds the sum of squares of query
            // row lane / 2 of this wave in every lane.
            static_assert(!QN || (PRE && QB == 2), "normalised queries are also pre-scaled; 32 query rows per wave");
            const float ss = __shfl(ss_row, 2 * (16 * qb + l16));
            const float rinv = c_exp2 / sqrtf(ss / (float)qn.d_model + qn.eps);
            const float *gp = qn.gain + head * D + q4 * 8;
#pragma unroll
            for (int m = 0; m < MK; ++m) {
                const float4 g0 = *reinterpret_cast<const float4 *>(gp + 32 * m), g1 = *reinterpret_cast<const float4 *>(gp + 32 * m + 4);
                const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
                u32x4_t w = __builtin_bit_cast(u32x4_t, qf[qb][m]);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    w[e] = pack_bf16x2(bf16_lo(w[e]) * rinv * gg[2 * e], bf16_hi(w[e]) * rinv * gg[2 * e + 1]);
                qf[qb][m] = __builtin_bit_cast(bf16x8_t, w);
            }
        }
    }

    const int n_tiles = (n_keys + KT - 1) / KT;
    const int n_ph = (n_tiles + TP - 1) / TP;  // phases: TP consecutive tiles each
    const char *k_src = reinterpret_cast<const char *>(kp + (size_t)head * cap * D);   // K tile t at k_src + t * TILE_B
    const char *v_src = reinterpret_cast<const char *>(vtp + (size_t)head * cap * D);  // V^T tile t at v_src + t * TILE_B

    // ---- staging (direct to LDS) -----------------------------------------------------------------------------------------
    // DMA instruction e of this wave covers LDS rows [rows_per_instr * (wave + NWAVES*e), +rows_per_instr) of a tile.
    // K: LDS row rr = 16 kb + r (row r of 16-key block kb, i.e. accumulator row r of score block kb) holds key
    // 32 (kb >> 1) + 8 (r >> 2) + 4 (kb & 1) + (r & 3): lane group q4 then owns, in blocks 2ks and 2ks + 1 together, the eight
    // CONSECUTIVE keys 32 ks + 8 q4 .. + 7, which is exactly its share of the B operand of the PV MFMA's k-step ks.
    uint32_t kdoff[DPW], vdoff[DPW];
#pragma unroll
    for (int e = 0; e < DPW; ++e) {
        const int j = wave + NWAVES * e;
        {
            const int rr = K_RPI * j + lane / K_CPR;  // LDS row
            const int pos = lane % K_CPR;
            const int key = (rr & 32) | (((rr >> 2) & 3) << 3) | (((rr >> 4) & 1) << 2) | (rr & 3);
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
    // stage u = { V^T(TP u + i), K(TP (u+1) + i), i < TP }: what the matrix phase X(u) reads
#define LVX_ATTN_STAGE_DMA(u_)                                   \
    {                                                            \
        _Pragma("unroll") for (int i_ = 0; i_ < TP; ++i_) {      \
            LVX_ATTN_DMA_V(TP * (u_) + i_);                      \
            LVX_ATTN_DMA_K(TP * ((u_) + 1) + i_);                \
        }                                                        \
    }
#define LVX_ATTN_WAIT_DMA(n_) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n_) : "memory")

    // fragment read offsets inside a tile (bytes): K fragment (kb, m): row 16 kb + l16, chunk (4m + q4) ^ swz;
    // V^T fragment (db, ks): row 16 db + l16, chunk (4 ks + q4) ^ swz
    const int k_swz = K_CPR == 16 ? l16 : ((l16 >> 1) & 7);
    const int v_swz = (l16 >> 1) & 7;
    int kfo[MK], vfo[2];
#pragma unroll
    for (int m = 0; m < MK; ++m) kfo[m] = l16 * K_ROW_B + (((4 * m + q4) ^ k_swz) * 16);
#pragma unroll
    for (int c = 0; c < 2; ++c) vfo[c] = l16 * V_ROW_B + (((4 * c + q4) ^ v_swz) * 16);

    // ---- pipeline -------------------------------------------------------------------------------------------------
    // A wave alternates between a matrix phase X(t) = { O += V(t)^T P(t) ; S(t+1) = K(t+1) Q^T } (MFMAs fed from LDS)
    // and a vector phase Y(t) = online softmax of S(t) -> P(t).  The two waves that share a SIMD (wave w and
    // w + NWAVES/2) run half a period apart, with a workgroup barrier after every phase: while group 0 is in X the
    // other is in Y, so the matrix core and the vector ALU of each SIMD are busy at the same time.
    //   iteration i, first half :  group 0: X(i-1) (S(0) only before the loop)  group 1: Y(i-1)
    //   iteration i, second half:  group 0: Y(i)                                group 1: X(i-1)
    // A phase covers TP consecutive tiles (TP = 2: 128 keys), which halves the barriers, the pipeline fills at a phase's start
    // and the drains at its end per key.
    // Staging: tile t lives in ring slot t % 4, so two stages fit.  Every wave issues the DMA of stage i at the start of
    // iteration i, into the slots of stage i-2, whose last reader (group 1's X(i-2), second half of iteration i-1) ended at
    // the barrier just passed, and waits for its own part before the barrier that ends iteration i; stage i is first read
    // by group 0 in X(i), right after that barrier: a whole iteration of both groups' work covers the load.
    const int grp = wave / (NWAVES / 2);

    // o[db][qb][e] = O^T[d = 16 db + 4 q4 + e][query 16 qb + l16];  s[kb][qb][e] = score of key row 4 q4 + e of block kb
    f32x4_t o[DB][QB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int e = 0; e < 4; ++e) o[i][qb][e] = 0.f;
    // per query block: the reference the softmax subtracts (a row maximum, already multiplied by c_exp2; set by the first
    // tile) and this lane's share of the row sum
    float mc[QB], l_run[QB];
    // PRE: the queries arrive multiplied by scale * log2(e) (before their rounding to bf16), and the score MFMAs start their
    // accumulators at -mc, so a score leaves the matrix phase as the exponent itself and the vector phase saves one FMA per
    // score.  sub = what the accumulators of the scores at hand were started at; it differs from mc only in the first phase and
    // after a re-base, where the difference is added explicitly.
    float sub[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) mc[qb] = l_run[qb] = sub[qb] = 0.f;
    f32x4_t s[4 * TP][QB];
    bf16x8_t pb[QB][2 * TP];  // [qb][ks]: P^T for keys 32 ks + 8 q4 .. + 7, query 16 qb + l16

    // S(0) = K(0) Q^T from K slot 0 (prologue of the pipeline; the steady state computes S inside LVX_ATTN_X)
#define LVX_ATTN_S0()                                                                                          \
    {                                                                                                          \
        _Pragma("unroll") for (int kb = 0; kb < 4 * TP; ++kb) {                                                \
            _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) _Pragma("unroll") for (int e = 0; e < 4; ++e) s[kb][qb][e] = 0.f; \
            bf16x8_t a[MK];                                                                                    \
            _Pragma("unroll") for (int m = 0; m < MK; ++m)                                                     \
                a[m] = *reinterpret_cast<const bf16x8_t *>(ks + (kb >> 2) * TILE_B + (kb & 3) * 16 * K_ROW_B + kfo[m]); \
            _Pragma("unroll") for (int m = 0; m < MK; ++m) _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)   \
                s[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], qf[qb][m], s[kb][qb], 0, 0, 0);      \
        }                                                                                                      \
    }
    // Matrix phase X(j): O^T += V(j)^T P(j)^T from V slot j%NS, then S(j+1) = K(j+1) Q^T from K slot (j+1)%NS (past the last
    // tile the slot holds a copy of the last tile; that S is never used).  One basic block of NV + NK LDS fragments, each
    // feeding two MFMAs (the two 16-query blocks).  The fragment reads run PD fragments ahead of their use through a ring
    // of PD registers, and the scheduler is told to keep that order (PD reads, then two MFMAs / one read, then 2 PD MFMAs),
    // so an MFMA never waits for a read issued just before it.  Consecutive MFMAs target different accumulators.
    //   fragment f < NV :  V^T rows 16*(f%DB).., keys 32*(f/DB) ..      -> o[f%DB][qb] += frag * pb[qb][f/DB]
    //   fragment f >= NV:  g = f - NV: K rows 16*(g%4).., dims 32*(g/4) ..  -> s[g%4][qb] += frag * qf[qb][g/4]
#define LVX_ATTN_FRAG(f_)                                                                                              \
    ((f_) < NV * TP ? *reinterpret_cast<const bf16x8_t *>(vr[(f_) / NV] + (((f_) % NV) % DB) * 16 * V_ROW_B + vfo[(((f_) % NV) / DB) & 1]) \
                    : *reinterpret_cast<const bf16x8_t *>(kr[(((f_) - NV * TP) / NK) % TP] + (((f_) - NV * TP) & 3) * 16 * K_ROW_B + \
                                                          kfo[((((f_) - NV * TP) % NK) >> 2) % MK]))
#define LVX_ATTN_X(j_)                                                                                         \
    {                                                                                                          \
        __builtin_amdgcn_s_setprio(2); /* the matrix phase wins instruction arbitration over the other wave's VALU */ \
        const char *vr[TP], *kr[TP];                                                                           \
        _Pragma("unroll") for (int i_ = 0; i_ < TP; ++i_) {                                                    \
            vr[i_] = vs + ((TP * (j_) + i_) & (NS - 1)) * TILE_B;                                              \
            kr[i_] = ks + ((TP * ((j_) + 1) + i_) & (NS - 1)) * TILE_B;                                        \
        }                                                                                                      \
        bf16x8_t fr[PD];                                                                                       \
        _Pragma("unroll") for (int f = 0; f < PD; ++f) fr[f] = LVX_ATTN_FRAG(f);                               \
        _Pragma("unroll") for (int kb = 0; kb < 4 * TP; ++kb) _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) \
            _Pragma("unroll") for (int e = 0; e < 4; ++e) s[kb][qb][e] = PRE ? -mc[qb] : 0.f;                  \
        if (PRE) { _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) sub[qb] = mc[qb]; }                       \
        _Pragma("unroll") for (int f = 0; f < (NV + NK) * TP; ++f) {                                           \
            const bf16x8_t a = fr[f % PD];                                                                     \
            if (f + PD < (NV + NK) * TP) fr[f % PD] = LVX_ATTN_FRAG(f + PD);                                   \
            _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                                \
                if (f < NV * TP) {                                                                             \
                    const int u_ = f / NV, ff_ = f % NV;                                                       \
                    o[ff_ % DB][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[qb][2 * u_ + ((ff_ / DB) & 1)], o[ff_ % DB][qb], 0, 0, 0); \
                } else {                                                                                       \
                    const int g_ = f - NV * TP, u_ = g_ / NK, gg_ = g_ % NK;                                   \
                    s[4 * u_ + (gg_ & 3)][qb] =                                                                \
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[qb][(gg_ >> 2) % MK], s[4 * u_ + (gg_ & 3)][qb], 0, 0, 0); \
                }                                                                                              \
            }                                                                                                  \
        }                                                                                                      \
        __builtin_amdgcn_sched_group_barrier(0x100, PD, 0);                                                    \
        _Pragma("unroll") for (int f = 0; f < (NV + NK) * TP - PD; ++f) {                                      \
            __builtin_amdgcn_sched_group_barrier(0x008, QB, 0);                                                \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                 \
        }                                                                                                      \
        __builtin_amdgcn_sched_group_barrier(0x008, QB * PD, 0);                                               \
    }
    // vector phase: s[kb][qb][e] is the score of key  t*64 + 32 (kb >> 1) + 8 q4 + 4 (kb & 1) + e  for query 16 qb + l16
#define LVX_ATTN_Y(t_)                                                                                         \
    {                                                                                                          \
        __builtin_amdgcn_s_setprio(0); /* the matrix phase's priority is kept through its DMA issue, up to here */ \
        if ((t_) == n_ph - 1 && (n_keys % (TP * KT)) != 0) {                                                   \
            int lim_ = n_keys - (t_) * (TP * KT) - 8 * q4; /* valid keys, counted from this lane group's first key */ \
            asm volatile("" : "+v"(lim_));          /* keep the compares out of the loop preheader */          \
            _Pragma("unroll") for (int kb = 0; kb < 4 * TP; ++kb) _Pragma("unroll") for (int e = 0; e < 4; ++e) \
                if (32 * (kb >> 1) + 4 * (kb & 1) + e >= lim_) {                                               \
                    _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) s[kb][qb][e] = -INFINITY;                \
                }                                                                                              \
        }                                                                                                      \
        /* The reference mc only has to keep exp2 inside the fp32 range, so no per-tile maximum is taken: mc is the first     \
           tile's row maximum, and a later tile whose sum of exponentials reaches 2^64 (or overflows) is redone with its own   \
           maximum as the new reference and the accumulators rescaled.  The four lane groups that share a query decide     \
           together (wave-wide vote); the final division by the row sum absorbs whatever reference was used. */            \
        float lsum[QB];                                                                                        \
        bool rebase_ = (t_) == 0;                                                                              \
        for (;;) {                                                                                             \
            if (rebase_) {                                                                                     \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                            \
                    float tmax = s[0][qb][0];                                                                  \
                    _Pragma("unroll") for (int kb = 0; kb < 4 * TP; ++kb) _Pragma("unroll") for (int e = 0; e < 4; ++e) \
                        tmax = fmaxf(tmax, s[kb][qb][e]);                                                      \
                    tmax = fmaxf(tmax, __shfl_xor(tmax, 16));                                                  \
                    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));                                                  \
                    const bool first_ = (t_) == 0;                                                             \
                    const float tmc = PRE ? tmax + sub[qb] : tmax * c_exp2;                                    \
                    const bool need = first_ || tmc > mc[qb] + 6.0f;                                           \
                    const float alpha = (need && !first_) ? __builtin_amdgcn_exp2f(mc[qb] - tmc) : 1.0f;       \
                    if (need) mc[qb] = tmc;                                                                    \
                    l_run[qb] *= alpha;                                                                        \
                    _Pragma("unroll") for (int i = 0; i < DB; ++i) _Pragma("unroll") for (int e = 0; e < 4; ++e) \
                        o[i][qb][e] *= alpha;                                                                  \
                }                                                                                              \
            }                                                                                                  \
            if (PRE) {                                                                                         \
                bool adj_ = false;                                                                             \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) adj_ = adj_ || (sub[qb] != mc[qb]);          \
                if (__any(adj_)) {                                                                             \
                    _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                        \
                        const float d_ = sub[qb] - mc[qb];                                                     \
                        _Pragma("unroll") for (int kb = 0; kb < 4 * TP; ++kb) _Pragma("unroll") for (int e = 0; e < 4; ++e) \
                            s[kb][qb][e] += d_;                                                                \
                        sub[qb] = mc[qb];                                                                      \
                    }                                                                                          \
                }                                                                                              \
            }                                                                                                  \
            bool fits_ = true;                                                                                 \
            _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) lsum[qb] = 0.f;                                  \
            _Pragma("unroll") for (int kb = 0; kb < 4 * TP; ++kb) _Pragma("unroll") for (int e = 0; e < 4; ++e) \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                            \
                    const float p_ = __builtin_amdgcn_exp2f(PRE ? s[kb][qb][e] : __builtin_fmaf(s[kb][qb][e], c_exp2, -mc[qb])); \
                    lsum[qb] += p_;                                                                            \
                    pb[qb][kb >> 1][4 * (kb & 1) + e] = (__bf16)p_;                                            \
                }                                                                                              \
            _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) fits_ = fits_ && (lsum[qb] < 0x1p64f);           \
            if (rebase_ || !__any(!fits_)) break;                                                              \
            rebase_ = true;                                                                                    \
        }                                                                                                      \
        _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) l_run[qb] += lsum[qb];                               \
    }

#pragma unroll
    for (int i = 0; i < TP; ++i) LVX_ATTN_DMA_K(i);
    LVX_ATTN_STAGE_DMA(0);
    LVX_ATTN_WAIT_DMA(0);
    __syncthreads();

    // Each group runs its own straight-line loop; both execute the same number of barriers (2 per iteration) and the same
    // DMA issue / wait sequence (issue at the start, wait at the end of every iteration).
    // A wave whose 32 queries all lie past n_q (ragged last query tile: 4680 = 18 x 256 + 72) only keeps up the DMA and
    // barrier protocol: no LDS reads, no MFMAs, no softmax.  Its SIMD partner then has the matrix core to itself, so such a
    // workgroup finishes early and frees its CU, and the padding costs no energy on a chip that is power-limited.
    const bool active = __builtin_amdgcn_readfirstlane(qtile * QT + wave * (16 * QB)) < n_q;
    if (!active) {
        __syncthreads();
        __syncthreads();
        for (int i = 1; i < n_ph; ++i) {
            LVX_ATTN_STAGE_DMA(i);
            __syncthreads();
            LVX_ATTN_WAIT_DMA(0);
            __syncthreads();
        }
        __syncthreads();
        __syncthreads();
    } else if (grp == 0) {
        LVX_ATTN_S0();
        __syncthreads();
        LVX_ATTN_Y(0);
        __syncthreads();
        for (int i = 1; i < n_ph; ++i) {
            LVX_ATTN_STAGE_DMA(i);
            LVX_ATTN_X(i - 1);
            __syncthreads();
            LVX_ATTN_Y(i);
            LVX_ATTN_WAIT_DMA(0);  // stage i landed
            __syncthreads();
        }
        LVX_ATTN_X(n_ph - 1);
        __syncthreads();
        __syncthreads();
    } else {
        __syncthreads();
        LVX_ATTN_S0();
        __syncthreads();
        for (int i = 1; i <= n_ph; ++i) {
            if (i < n_ph) LVX_ATTN_STAGE_DMA(i);
            LVX_ATTN_Y(i - 1);
            __syncthreads();
            LVX_ATTN_X(i - 1);
            if (i < n_ph) LVX_ATTN_WAIT_DMA(0);
            __syncthreads();
        }
    }
    LVX_ATTN_WAIT_DMA(0);  // no DMA may still be in flight when the workgroup releases its LDS

    uint32_t amax_b = 0;  // largest magnitude among the bf16 values this lane stores (bit pattern without sign)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 16);
        l_tot += __shfl_xor(l_tot, 32);
        const float inv = 1.0f / l_tot;
        const int row = qtile * QT + wave * (16 * QB) + 16 * qb + l16;
        if (row < n_q) {
            bf16_t *op = out + (size_t)row * ld_out + (size_t)head * D;
            // accumulator register e of block (db, qb) holds O^T[d = 16db + 4q4 + e][query 16qb + l16]
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                uint2 w;
                w.x = pack_bf16x2(o[db][qb][0] * inv, o[db][qb][1] * inv);
                w.y = pack_bf16x2(o[db][qb][2] * inv, o[db][qb][3] * inv);
                *reinterpret_cast<uint2 *>(op + 16 * db + 4 * q4) = w;
                if (amax_slots != nullptr) {
                    const uint32_t a0 = w.x & 0x7fffu, a1 = (w.x >> 16) & 0x7fffu, a2 = w.y & 0x7fffu, a3 = (w.y >> 16) & 0x7fffu;
                    uint32_t m = a0 > a1 ? a0 : a1;
                    m = m > a2 ? m : a2;
                    m = m > a3 ? m : a3;
                    amax_b = amax_b > m ? amax_b : m;
                }
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

template <int D, int NWAVES, int QB = 2, int TP = 1, bool PRE = false, bool QN = false>
lvx_status_t launch(const bf16_t *q, int64_t ld_q, int n_q, int H, const bf16_t *kp, const bf16_t *vtp, int cap, int n_keys,
                    float scale, bf16_t *out, int64_t ld_out, hipStream_t stream, uint32_t *amax_slots, const lvx_attn_qnorm_t *qnorm = nullptr) {
    constexpr int QT = 16 * QB * NWAVES;
    const int n_qtiles = (n_q + QT - 1) / QT;
    const int total = n_qtiles * H;
    const int per_xcd = (total + 7) / 8;
    const float c = scale * LVX_LOG2E;
    lvx_attn_qnorm_t qn = {};
    if (qnorm != nullptr) qn = *qnorm;
    hipLaunchKernelGGL((lvx_attention_kernel<D, NWAVES, QB, TP, PRE, QN>), dim3(per_xcd * 8), dim3(64 * NWAVES), 0, stream, q, ld_q, n_q, kp, vtp, cap,
                       n_keys, c, out, ld_out, n_qtiles, total, per_xcd, amax_slots, qn);
    LVX_CHECK_HIP(hipGetLastError());
    return LVX_OK;
}

}  // namespace

lvx_status_t lvx_launch_attention(const bf16_t *q, int64_t ld_q, int n_q, int H, int D, const bf16_t *k_packed,
                                  const bf16_t *vt_packed, int cap, int n_keys, float scale, bf16_t *out, int64_t ld_out,
                                  hipStream_t stream, uint32_t *amax_slots, bool q_prescaled, const lvx_attn_qnorm_t *qnorm) {
    LVX_REQUIRE(n_q > 0 && n_keys > 0 && n_keys <= cap && cap % KT == 0, LVX_ERR_SHAPE, "attention: n_q %d, n_keys %d, cap %d", n_q,
                n_keys, cap);
    LVX_REQUIRE(scale > 0.f, LVX_ERR_INVALID_ARG, "attention: scale must be positive");
#ifdef LVX_ATTN_16W
    if (D == 128) return launch<128, 16, 1>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots);
#endif
#ifdef LVX_ATTN_2WG  // experiment: workgroups of 4 waves (128 queries, 64 KB of LDS), two of them per CU
    if (D == 128) return launch<128, 4, 2, 1>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots);
#endif
    if (qnorm != nullptr) {  // the kernel normalises and scales the queries as it loads them (cross-attention of a bf16 stage)
        LVX_REQUIRE(D == 128 && qnorm->sumsq != nullptr && qnorm->gain != nullptr && qnorm->n_parts > 0 && qnorm->n_parts % 8 == 0 &&
                        qnorm->n_parts <= 128 && qnorm->ld % 4 == 0 && qnorm->d_model == H * D,
                    LVX_ERR_INVALID_ARG,
                    "attention: query norm needs head_dim 128, partial sums and a gain");
        return launch<128, 8, 2, 1, true, true>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots, qnorm);
    }
    if (q_prescaled) {  // q already carries scale * log2(e): see PRE in the kernel
        if (D == 128 && n_keys >= TP2_MIN_KEYS)
            return launch<128, 8, 2, 2, true>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots);
        if (D == 128) return launch<128, 8, 2, 1, true>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots);
        if (D == 64) return launch<64, 8, 2, 1, true>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots);
        return lvx_fail(LVX_ERR_UNSUPPORTED, "head_dim %d not supported (64 or 128)", D);
    }
    if (D == 128 && n_keys >= TP2_MIN_KEYS)
        return launch<128, 8, 2, 2>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots);
    if (D == 128) return launch<128, 8>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots);
    if (D == 64) return launch<64, 8>(q, ld_q, n_q, H, k_packed, vt_packed, cap, n_keys, scale, out, ld_out, stream, amax_slots);
    return lvx_fail(LVX_ERR_UNSUPPORTED, "head_dim %d not supported (64 or 128)", D);
}

static lvx_status_t chunk_attention_entry(const lvx_kvcache_t *c, int32_t layer, const void *dev_q, int64_t ld_q, int32_t n_q, float scale,
                                          void *dev_out, int64_t ld_out, lvx_stream_t stream, bool q_prescaled) {
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
                                lvx_cache_vt(c, layer), c->cap_keys, s.key_count, scale, (bf16_t *)dev_out, ld_out, (hipStream_t)stream, nullptr, q_prescaled);
}

extern "C" lvx_status_t lvx_chunk_attention(const lvx_kvcache_t *c, int32_t layer, const void *dev_q, int64_t ld_q, int32_t n_q,
                                            float scale, void *dev_out, int64_t ld_out, lvx_stream_t stream) {
    return chunk_attention_entry(c, layer, dev_q, ld_q, n_q, scale, dev_out, ld_out, stream, false);
}

extern "C" lvx_status_t lvx_chunk_attention_prescaled(const lvx_kvcache_t *c, int32_t layer, const void *dev_q_scaled, int64_t ld_q,
                                                      int32_t n_q, void *dev_out, int64_t ld_out, lvx_stream_t stream) {
    return chunk_attention_entry(c, layer, dev_q_scaled, ld_q, n_q, 1.0f, dev_out, ld_out, stream, true);
}
