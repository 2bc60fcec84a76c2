// Backward attention kernels for gfx950 (MI355X).
//
//   dV = P^T dO,  dP = dO V^T,  dS = P o (dP - D),  dQ = scale dS K,  dK = scale dS^T Q
// (paper Sec. 2.1) with P recomputed from Q, K and the saved row log-sum-exp.
//
// Three kernels:
//   bwd_prepare : D_i = sum_c dO_ic O_ic (the identity sum_j P_ij dP_ij = dO_i . O_i that
//                 follows from the softmax Jacobian of Sec. 2.1), stored as -D_i, and LSE in
//                 base-2 units.  HBM bound.
//   bwd_dkdv    : one workgroup per KV tile looping over query tiles, dK and dV accumulated
//                 on chip for the whole loop (the loop structure of paper Sec. 3.2.2).
//   bwd_dq      : one workgroup per query tile looping over KV tiles, dQ accumulated on chip.
//
// Why dQ has a kernel of its own.  The paper adds a dQ tile to global memory with atomics
// in every inner iteration (Sec. 3.2.2) and halves their number with CTA pairs (Sec. 3.2.3).
// On MI355X every such fp32 atomic is executed on the memory side of the XCD-private L2s
// (measured: 8.7 GB of write traffic per launch at about 2.4 TB/s for B=2 H=16 N=8192 d=128),
// which alone exceeds the time budget of the whole backward pass, and there is no CTA-pair
// mechanism to halve it.  Recomputing S and dP a second time in a query-stationary kernel
// costs two more MFMA contractions (7 instead of 5) but no atomics, no fp32 accumulator in
// HBM, no dS round trip through LDS, and makes the backward pass deterministic.
//
// MFMA orientations.
//   bwd_dkdv: S = Q K_w^T and dP = dO V_w^T with queries on the MFMA row axis and this wave's
//     32 keys on the column axis, so a lane owns one key column and 16 query rows per 32x32
//     block.  That register layout, converted to bf16, is directly the B operand (contraction
//     over queries) of dV_w^T += dO^T P and dK_w^T += Q^T dS, whose A operands come from the
//     same Q / dO tiles through the transposing LDS read.  This is the "compute the
//     transposed product so that P and dS feed the next MMA from on-chip storage" idea of
//     Sec. 3.2.2 restated for the MFMA register layout.  K_w and V_w stay in registers.
//   bwd_dq: S^T = K Q_w^T and dP^T = V dO_w^T with keys on the row axis and this wave's 32
//     queries on the column axis (as in the forward kernel): LSE and D are one register per
//     lane, and dS^T in registers is the B operand of dQ_w^T += K^T dS^T.
#include "common.h"
#include "launch.h"

namespace attn {

constexpr int BWD_BK = 128;   // dkdv: keys per block
constexpr int BWD_BQ = 64;    // dkdv: queries per step
constexpr int BWD_NT = 256;
constexpr int DQ_BM = 128;    // dq: queries per block
constexpr int DQ_BN = 64;     // dq: keys per step

// ------------------------------------------------------------------------------------------
// bwd_prepare: one group of DV/8 lanes per (b, i, h) row.
template <int DV>
__global__ void __launch_bounds__(256)
bwd_prepare_kernel(const bf16* __restrict__ o, const bf16* __restrict__ d_o, const float* __restrict__ lse,
                   float* __restrict__ D, float* __restrict__ lse2, int H, int N, int64_t nrows)
{
    constexpr int LPR = DV / 8;                 // lanes per row
    constexpr int RPB = 256 / LPR;              // rows per block
    const int sub = threadIdx.x % LPR;
    const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / LPR;   // (b*N + i)*H + h
    if (row >= nrows) return;
    const bf16x8 a = *(const bf16x8*)(o + row * DV + sub * 8);
    const bf16x8 g = *(const bf16x8*)(d_o + row * DV + sub * 8);
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc = fmaf((float)a[e], (float)g[e], acc);
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (sub == 0) {
        const int64_t bi = row / H;             // b*N + i
        const int h = (int)(row - bi * H);
        const int64_t b = bi / N;
        const int i = (int)(bi - b * N);
        const int64_t idx = (b * H + h) * N + i;
        D[idx] = -acc;           // stored negated: the consumers add it (or start an accumulator from it)
        lse2[idx] = lse[idx] * kLog2e;
    }
}

#define ATTN_VARLEN 0
#include "attn_bwd_dkdv_kernel.inc"
#undef ATTN_VARLEN
#define ATTN_VARLEN 1
#include "attn_bwd_dkdv_kernel.inc"
#undef ATTN_VARLEN

// ------------------------------------------------------------------------------------------
// bwd_dkdv, wave-specialised variant (the role split of paper Sec. 3.2.2 -- one set of warps
// computes S, dP and the elementwise stage, another runs the accumulating MMAs and the loads --
// restated for a CU whose registers are divided evenly among its waves).
//
// Block = 8 waves = 128 keys.  Waves 0-3 ("score" waves, 32 keys each) keep K_w and V_w in
// registers and produce P and dS for one query tile per round; waves 4-7 ("gradient" waves, the
// same 32 keys each) keep the dK_w / dV_w accumulators, issue every global->LDS copy and consume
// the P / dS of the previous round.  Each SIMD hosts one wave of each kind, so the exponentials
// of one overlap the MFMAs of the other, and neither needs more than 256 registers.
//
// Round j:   barrier A | score: tile j -> P_j, dS_j in registers     | barrier B | score: P_j, dS_j -> LDS
//                      | gradient: copy tile j+1; dK, dV += tile j-1 |           | gradient: wait for copy
// Query / dO tiles rotate through three LDS stages (tile j is read plainly in round j and
// through the transposing read in round j+1 while tile j+2 is not yet wanted); P / dS pass
// through one 32 KiB buffer: barrier B orders the previous round's readers before the writers.
// Both barriers are plain workgroup barriers that every wave reaches once per round: no wave
// ever spins on another.
constexpr int WS_NT = 512;
constexpr int WS_STAGES = 3;
constexpr int WS_PDS_BYTES = 4 * 8 * 1024;   // 4 key groups x (2 query blocks x (P, dS) x 2 halves) x 64 lanes x 16 B

#define ATTN_VARLEN 0
#include "attn_bwd_dkdv_ws_kernel.inc"
#undef ATTN_VARLEN
#define ATTN_VARLEN 1
#include "attn_bwd_dkdv_ws_kernel.inc"
#undef ATTN_VARLEN

#define ATTN_VARLEN 0
#include "attn_bwd_dq_kernel.inc"
#undef ATTN_VARLEN
#define ATTN_VARLEN 1
#include "attn_bwd_dq_kernel.inc"
#undef ATTN_VARLEN

// Variable-length backward: the prepare kernel sees the packed batch as one sequence of T rows
// (its outputs are then laid out [H, T]); dK/dV and dQ use the plan table.
template <int DQK, int DV, bool CAUSAL>
static int launch_bwd_varlen_t(const BwdArgs& a)
{
    void* st = a.stream;
    const int64_t nrows = (int64_t)a.T * a.H;
    if (a.phases & 1) {
        constexpr int RPB = 256 / (DV / 8);
        if (launch_kernel(bwd_prepare_kernel<DV>, dim3((unsigned)((nrows + RPB - 1) / RPB)), dim3(256), 0, st,
                          (const bf16*)a.o, (const bf16*)a.d_o, a.lse, a.D, a.lse2, a.H, a.T, nrows) != hipSuccess)
            return -3;
    }
    if constexpr (DQK == 128) { if (a.phases & 2) {
        constexpr int smem = WS_STAGES * (BWD_BQ * (DQK + DV) * 2 + 512) + WS_PDS_BYTES;
        auto kern = attn_bwd_dkdv_ws_varlen_kernel<DQK, DV, CAUSAL>;
        static LdsOptIn lds;
        if (!lds.allow(kern, smem)) return -3;
        if (launch_kernel(kern, dim3(a.max_tiles * a.Hkv), dim3(WS_NT), smem, st,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.d_o,
                          (const float*)a.lse2, (const float*)a.D, (bf16*)a.dk, (bf16*)a.dv,
                          a.H, a.Hkv, a.scale, a.scale * kLog2e, (const int4*)a.plan, a.T, a.max_tiles) != hipSuccess)
            return -3;
    } } else if (a.phases & 2) {
        constexpr int smem = 2 * BWD_BQ * (DQK + DV) * 2 + 1024;
        auto kern = attn_bwd_dkdv_varlen_kernel<DQK, DV, CAUSAL>;
        static LdsOptIn lds;
        if (!lds.allow(kern, smem)) return -3;
        if (launch_kernel(kern, dim3(a.max_tiles * a.Hkv), dim3(BWD_NT), smem, st,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.d_o,
                          (const float*)a.lse2, (const float*)a.D, (bf16*)a.dk, (bf16*)a.dv,
                          a.H, a.Hkv, a.scale, a.scale * kLog2e, (const int4*)a.plan, a.T, a.max_tiles) != hipSuccess)
            return -3;
    }
    if (a.phases & 4) {
        constexpr int smem = 2 * DQ_BN * (DQK + DV) * 2;
        auto kern = attn_bwd_dq_varlen_kernel<DQK, DV, CAUSAL>;
        static LdsOptIn lds;
        if (!lds.allow(kern, smem)) return -3;
        if (launch_kernel(kern, dim3(a.max_tiles * a.H), dim3(BWD_NT), smem, st,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.d_o,
                          (const float*)a.lse2, (const float*)a.D, (bf16*)a.dq,
                          a.H, a.Hkv, a.scale, a.scale * kLog2e, (const int4*)a.plan, a.T, a.max_tiles) != hipSuccess)
            return -3;
    }
    return 0;
}

template <int DQK, int DV, bool CAUSAL>
static int launch_bwd_t(const BwdArgs& a)
{
    if (a.plan) return launch_bwd_varlen_t<DQK, DV, CAUSAL>(a);
    void* st = a.stream;
    const int64_t nrows = (int64_t)a.B * a.N * a.H;
    if (a.phases & 1) {
        constexpr int RPB = 256 / (DV / 8);
        if (launch_kernel(bwd_prepare_kernel<DV>, dim3((unsigned)((nrows + RPB - 1) / RPB)), dim3(256), 0, st,
                          (const bf16*)a.o, (const bf16*)a.d_o, a.lse, a.D, a.lse2, a.H, a.N, nrows) != hipSuccess)
            return -3;
    }
#ifndef ATTN_DKDV_WS
#define ATTN_DKDV_WS 1
#endif
    if constexpr (ATTN_DKDV_WS && DQK == 128) { if (a.phases & 2) {
        constexpr int smem = WS_STAGES * (BWD_BQ * (DQK + DV) * 2 + 512) + WS_PDS_BYTES;
        auto kern = attn_bwd_dkdv_ws_kernel<DQK, DV, CAUSAL>;
        static LdsOptIn lds;
        if (!lds.allow(kern, smem)) return -3;
        const int grid = a.B * a.Hkv * (a.N / BWD_BK);
        if (launch_kernel(kern, dim3(grid), dim3(WS_NT), smem, st,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.d_o,
                          (const float*)a.lse2, (const float*)a.D, (bf16*)a.dk, (bf16*)a.dv,
                          a.H, a.Hkv, a.N, a.scale, a.scale * kLog2e) != hipSuccess)
            return -3;
    } } else if (a.phases & 2) {
        constexpr int smem = 2 * BWD_BQ * (DQK + DV) * 2 + 1024;
        auto kern = attn_bwd_dkdv_kernel<DQK, DV, CAUSAL>;
        static LdsOptIn lds;
        if (!lds.allow(kern, smem)) return -3;
        const int grid = a.B * a.Hkv * (a.N / BWD_BK);
        if (launch_kernel(kern, dim3(grid), dim3(BWD_NT), smem, st,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.d_o,
                          (const float*)a.lse2, (const float*)a.D, (bf16*)a.dk, (bf16*)a.dv,
                          a.H, a.Hkv, a.N, a.scale, a.scale * kLog2e) != hipSuccess)
            return -3;
    }
    if (a.phases & 4) {
        constexpr int smem = 2 * DQ_BN * (DQK + DV) * 2;
        auto kern = attn_bwd_dq_kernel<DQK, DV, CAUSAL>;
        static LdsOptIn lds;
        if (!lds.allow(kern, smem)) return -3;
        const int grid = a.B * a.H * (a.N / DQ_BM);
        if (launch_kernel(kern, dim3(grid), dim3(BWD_NT), smem, st,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.d_o,
                          (const float*)a.lse2, (const float*)a.D, (bf16*)a.dq,
                          a.H, a.Hkv, a.N, a.scale, a.scale * kLog2e) != hipSuccess)
            return -3;
    }
    return 0;
}

int launch_bwd(const BwdArgs& a)
{
    if (a.d_qk == 64 && a.d_v == 64)
        return a.causal ? launch_bwd_t<64, 64, true>(a) : launch_bwd_t<64, 64, false>(a);
    if (a.d_qk == 128 && a.d_v == 128)
        return a.causal ? launch_bwd_t<128, 128, true>(a) : launch_bwd_t<128, 128, false>(a);
    if (a.d_qk == 192 && a.d_v == 128)
        return a.causal ? launch_bwd_t<192, 128, true>(a) : launch_bwd_t<192, 128, false>(a);
    return -2;
}

}  // namespace attn
