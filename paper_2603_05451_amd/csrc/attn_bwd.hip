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

template <int DQK, int DV, bool CAUSAL>
__global__ void __launch_bounds__(WS_NT, 1)
attn_bwd_dkdv_ws_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                        const bf16* __restrict__ d_o, const float* __restrict__ lse2, const float* __restrict__ D,
                        bf16* __restrict__ dk, bf16* __restrict__ dv,
                        int H, int Hkv, int N, float scale, float scale_log2e)
{
    constexpr int KSQ = DQK / 16, KSV = DV / 16;
    constexpr int DBQ = DQK / 32, DBV = DV / 32;
    constexpr int QB = BWD_BQ / 32;
    constexpr int Q_BYTES = BWD_BQ * DQK * 2;
    constexpr int DO_BYTES = BWD_BQ * DV * 2;
    constexpr int ST_OFF = WS_STAGES * (Q_BYTES + DO_BYTES);
    constexpr int PDS_OFF = ST_OFF + WS_STAGES * 512;

    extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
    ATTN_LDS char* smem = (ATTN_LDS char*)smem_raw;
    auto q_lds = [&](int stg) { return smem + stg * Q_BYTES; };
    auto do_lds = [&](int stg) { return smem + WS_STAGES * Q_BYTES + stg * DO_BYTES; };
    auto st_lds = [&](int stg) { return smem + ST_OFF + stg * 512; };

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const bool score_wave = wave < 4;
    const int grp = wave & 3;                 // key group of this wave
    const int c = lane & 31, h = lane >> 5;
    ATTN_LDS char* pds = smem + PDS_OFF + grp * 8192 + lane * 16;   // + slot * 1024

    const int ntk = N / BWD_BK;
    const int total = gridDim.x;
    int vid = blockIdx.x;
    if ((total & 7) == 0) vid = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);
    const int bkv = vid / ntk;
    const int kt = vid - bkv * ntk;
    const int b = bkv / Hkv, kvh = bkv - b * Hkv;
    const int G = H / Hkv;
    const int k0 = kt * BWD_BK;
    const int kw0 = k0 + grp * 32;

    const int64_t q_stride = (int64_t)H * DQK, o_stride = (int64_t)H * DV;
    const int64_t k_stride = (int64_t)Hkv * DQK, v_stride = (int64_t)Hkv * DV;

    const int i_first = CAUSAL ? k0 / BWD_BQ : 0;
    const int nq = N / BWD_BQ - i_first;
    const int nsteps = G * nq;
    auto tile_q0 = [&](int step) { return (i_first + step % nq) * BWD_BQ; };

    // Stage rotation: every LDS read address is a lane register that already contains the stage
    // offset, plus an immediate; the registers advance by one stage per round (one vector add
    // each), so the loop body exists once.
    auto stage_step = [](int stg, int bytes) { return stg == WS_STAGES - 1 ? -(WS_STAGES - 1) * bytes : bytes; };

    if (score_wave) {
        // ================= score waves =================
        bf16x8 kf[KSQ], vf[KSV];
        {
            const bf16* krow = k + ((int64_t)b * N * Hkv + kvh) * DQK + (int64_t)(kw0 + c) * k_stride + 8 * h;
            const bf16* vrow = v + ((int64_t)b * N * Hkv + kvh) * DV + (int64_t)(kw0 + c) * v_stride + 8 * h;
#pragma unroll
            for (int ks = 0; ks < KSQ; ++ks) kf[ks] = *(const bf16x8*)(krow + 16 * ks);
#pragma unroll
            for (int ks = 0; ks < KSV; ++ks) vf[ks] = *(const bf16x8*)(vrow + 16 * ks);
#pragma unroll
            for (int ks = 0; ks < KSQ; ++ks) pin_ready(kf[ks]);
#pragma unroll
            for (int ks = 0; ks < KSV; ++ks) pin_ready(vf[ks]);
        }
        // A-operand chunk addresses for query block 0 of the current stage (the swizzle repeats
        // every 16 rows, so the second query block is an immediate away)
        const ATTN_LDS char* aq[KSQ];
        const ATTN_LDS char* ado[KSV];
#pragma unroll
        for (int st = 0; st < KSQ; ++st) aq[st] = q_lds(0) + tile_off<DQK>(c, 2 * st + h);
#pragma unroll
        for (int st = 0; st < KSV; ++st) ado[st] = do_lds(0) + tile_off<DV>(c, 2 * st + h);
        const ATTN_LDS char* stp = st_lds(0) + 16 * h;

        int stg = 0;
        constexpr int GRP = 4, NS = KSQ + KSV, NG = NS / GRP;
        static_assert(KSQ % GRP == 0 && KSV % GRP == 0 && NG == 4,
                      "four MFMA groups per query block, one per elementwise register group");
        for (int j = 0; j <= nsteps; ++j) {
            __syncthreads();                                   // barrier A
            bf16x8 pb[QB][2], dsb[QB][2];
            const bool live = j < nsteps;
            if (live) {
                const int q0 = tile_q0(j);
                const bool diag = CAUSAL && (q0 < k0 + BWD_BK - 1);     // some (query, key) pair is masked
                // Two-stage pipeline over the query blocks of the tile: the MFMAs of block qb are
                // issued in four groups of four, each followed by a quarter of the elementwise work
                // of block qb - 1, which runs in their shadow.
                f32x16 s[QB], dp[QB];
                bf16x8 fr[2][GRP];
                auto load_a = [&](int qb, int g, bf16x8* dst) {
#pragma unroll
                    for (int t = 0; t < GRP; ++t) {
                        const int st = g * GRP + t;
                        dst[t] = st < KSQ ? lds_read_b128(aq[st] + 32 * qb * DQK * 2)
                                          : lds_read_b128(ado[st - KSQ] + 32 * qb * DV * 2);
                    }
                };
                auto mfma_group = [&](int qb, int g) {
#pragma unroll
                    for (int t = 0; t < GRP; ++t) {
                        const int st = g * GRP + t;
                        if (st < KSQ) s[qb] = mfma32(fr[g & 1][t], kf[st], st == 0 ? f32x16{} : s[qb]);
                        else dp[qb] = mfma32(fr[g & 1][t], vf[st - KSQ], dp[qb]);   // starts from -D
                    }
                };
                // LSE of the 4 query rows of register group r4: one 16-byte broadcast read, fetched
                // one group ahead of its use.  -D of the same rows is read straight into the dP
                // accumulator (register r of the accumulator is query row 8(r/4) + 4h + r%4), so
                // the MFMAs deliver dP - D.
                f32x4 Lq[2];
                auto load_stats = [&](int qb, int r4) {
                    Lq[r4 & 1] = *(const ATTN_LDS f32x4*)(stp + (32 * qb + 8 * r4) * 4);
                };
                auto load_negD = [&](int qb) {
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const f32x4 nd = *(const ATTN_LDS f32x4*)(stp + (64 + 32 * qb + 8 * r4) * 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) dp[qb][4 * r4 + e] = nd[e];
                    }
                };
                // P = 2^(c S - LSE2), dS = P o (dP - D) for register group r4 of block qb
                auto elementwise = [&](int qb, int r4) {
                    const f32x4 L = Lq[r4 & 1];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int r = 4 * r4 + e;
                        float p = fast_exp2(fmaf(s[qb][r], scale_log2e, -L[e]));
                        if (diag && (kw0 + c > q0 + 32 * qb + 8 * r4 + 4 * h + e)) p = 0.f;
                        const float ds = p * dp[qb][r];
                        pb[qb][r >> 3][r & 7] = (bf16)p;
                        dsb[qb][r >> 3][r & 7] = (bf16)ds;
                    }
                };
                load_a(0, 0, fr[0]);
#pragma unroll
                for (int qb = 0; qb <= QB; ++qb) {
#pragma unroll
                    for (int g = 0; g < NG; ++g) {
                        if (qb < QB) {
                            if (g + 1 < NG) load_a(qb, g + 1, fr[(g + 1) & 1]);
                            else if (qb + 1 < QB) load_a(qb + 1, 0, fr[(g + 1) & 1]);
                            if (g == 0) load_negD(qb);         // wanted by the first dP MFMA, two groups on
                        }
                        // statistics for the elementwise group after this one
                        if (g + 1 < NG) { if (qb > 0) load_stats(qb - 1, g + 1); }
                        else if (qb < QB) load_stats(qb, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        if (qb < QB) mfma_group(qb, g);
                        if (qb > 0) elementwise(qb - 1, g);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            __syncthreads();                                   // barrier B: last round's P / dS have been read
            if (live) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        *(ATTN_LDS bf16x8*)(pds + (qb * 4 + kk) * 1024) = pb[qb][kk];
                        *(ATTN_LDS bf16x8*)(pds + (qb * 4 + 2 + kk) * 1024) = dsb[qb][kk];
                    }
                }
            }
            const int dq_ = stage_step(stg, Q_BYTES), ddo_ = stage_step(stg, DO_BYTES), dst_ = stage_step(stg, 512);
#pragma unroll
            for (int st = 0; st < KSQ; ++st) aq[st] += dq_;
#pragma unroll
            for (int st = 0; st < KSV; ++st) ado[st] += ddo_;
            stp += dst_;
            stg = stg == WS_STAGES - 1 ? 0 : stg + 1;
        }
        return;
    }

    // ================= gradient waves =================
    const int gtid = tid - 256;
    const int i16 = lane & 15;
    const int tr_row = i16 >> 2;
    const int tr_chunk = 2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1);
    const int tr_half = (i16 & 1) * 8;

    // transposing-read addresses for rows 4h + tr_row (+8) of the stage that holds tile j-1
    // (stage WS_STAGES-1 stands in before the first tile); query block and 16-row group are
    // immediates
    const ATTN_LDS char* tq[2][DBQ];
    const ATTN_LDS char* tdo[2][DBV];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int db = 0; db < DBQ; ++db)
            tq[u][db] = q_lds(WS_STAGES - 1) + tr_half + tile_off<DQK>(4 * h + tr_row + 8 * u, 4 * db + tr_chunk);
#pragma unroll
        for (int db = 0; db < DBV; ++db)
            tdo[u][db] = do_lds(WS_STAGES - 1) + tr_half + tile_off<DV>(4 * h + tr_row + 8 * u, 4 * db + tr_chunk);
    }

    TileCopy<BWD_BQ, DQK, 256> qcopy;
    TileCopy<BWD_BQ, DV, 256> docopy;
    qcopy.init(q_stride, gtid);
    docopy.init(o_stride, gtid);
    auto issue_loads = [&](int step, int stg) {
        const int g = step / nq, i = i_first + (step - g * nq);
        const int hq = kvh * G + g;
        const int64_t row0 = (int64_t)b * N + (int64_t)i * BWD_BQ;
        qcopy.issue_all(q + row0 * q_stride + (int64_t)hq * DQK, q_lds(stg));
        docopy.issue_all(d_o + row0 * o_stride + (int64_t)hq * DV, do_lds(stg));
        if (grp < 2) {
            const float* src = (grp == 0 ? lse2 : D) + ((int64_t)b * H + hq) * N + (int64_t)i * BWD_BQ + lane;
            dma4(src, st_lds(stg) + grp * 256);
        }
    };
    issue_loads(0, 0);

    f32x16 dk_acc[DBQ], dv_acc[DBV];
#pragma unroll
    for (int db = 0; db < DBQ; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dk_acc[db][r] = 0.f;
#pragma unroll
    for (int db = 0; db < DBV; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dv_acc[db][r] = 0.f;

    int pstg = WS_STAGES - 1;                              // stage of tile j-1
    constexpr int NPART = 4 * QB;                          // (query block, 16-query group, dV | dK)
    static_assert(DBV <= DBQ, "fragment buffers are sized by the wider head dim");
    for (int j = 0; j <= nsteps; ++j) {
        wait_async_copies();                               // tile j has landed (this wave's share)
        __syncthreads();                                   // barrier A
        if (j + 1 < nsteps) issue_loads(j + 1, pstg == 0 ? 2 : pstg - 1);   // (pstg + 2) mod 3: stage of tile j+1
        if (j >= 1) {
            bf16x8 pb[QB][2], dsb[QB][2];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    pb[qb][kk] = *(const ATTN_LDS bf16x8*)(pds + (qb * 4 + kk) * 1024);
                    dsb[qb][kk] = *(const ATTN_LDS bf16x8*)(pds + (qb * 4 + 2 + kk) * 1024);
                }
            // transposed fragments run two parts ahead of the MFMAs that consume them
            bf16x4 tfr[3][DBQ][2];
            auto load_t = [&](int part, bf16x4 (*dst)[2]) {
                const int row0 = 16 * (part >> 1);
                if ((part & 1) == 0) {
#pragma unroll
                    for (int db = 0; db < DBV; ++db) {
                        dst[db][0] = lds_read_tr(tdo[0][db] + row0 * DV * 2);
                        dst[db][1] = lds_read_tr(tdo[1][db] + row0 * DV * 2);
                    }
                } else {
#pragma unroll
                    for (int db = 0; db < DBQ; ++db) {
                        dst[db][0] = lds_read_tr(tq[0][db] + row0 * DQK * 2);
                        dst[db][1] = lds_read_tr(tq[1][db] + row0 * DQK * 2);
                    }
                }
            };
            load_t(0, tfr[0]);
            load_t(1, tfr[1]);
#pragma unroll
            for (int part = 0; part < NPART; ++part) {
                if (part + 2 < NPART) load_t(part + 2, tfr[(part + 2) % 3]);
                __builtin_amdgcn_sched_barrier(0);
                const int qb = part >> 2, kk = (part >> 1) & 1;
                if ((part & 1) == 0) {
#pragma unroll
                    for (int db = 0; db < DBV; ++db)
                        dv_acc[db] = mfma32(cat4(tfr[part % 3][db][0], tfr[part % 3][db][1]), pb[qb][kk], dv_acc[db]);
                } else {
#pragma unroll
                    for (int db = 0; db < DBQ; ++db)
                        dk_acc[db] = mfma32(cat4(tfr[part % 3][db][0], tfr[part % 3][db][1]), dsb[qb][kk], dk_acc[db]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();                                   // barrier B
        const int dq_ = stage_step(pstg, Q_BYTES), ddo_ = stage_step(pstg, DO_BYTES);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int db = 0; db < DBQ; ++db) tq[u][db] += dq_;
#pragma unroll
            for (int db = 0; db < DBV; ++db) tdo[u][db] += ddo_;
        }
        pstg = pstg == WS_STAGES - 1 ? 0 : pstg + 1;
    }

    bf16* dkrow = dk + ((int64_t)b * N + kw0 + c) * k_stride + (int64_t)kvh * DQK;
    bf16* dvrow = dv + ((int64_t)b * N + kw0 + c) * v_stride + (int64_t)kvh * DV;
#pragma unroll
    for (int db = 0; db < DBQ; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            bf16x4 out;
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = (bf16)(dk_acc[db][4 * r4 + e] * scale);
            *(bf16x4*)(dkrow + 32 * db + 8 * r4 + 4 * h) = out;
        }
#pragma unroll
    for (int db = 0; db < DBV; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            bf16x4 out;
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = (bf16)dv_acc[db][4 * r4 + e];
            *(bf16x4*)(dvrow + 32 * db + 8 * r4 + 4 * h) = out;
        }
}

#define ATTN_VARLEN 0
#include "attn_bwd_dq_kernel.inc"
#undef ATTN_VARLEN
#define ATTN_VARLEN 1
#include "attn_bwd_dq_kernel.inc"
#undef ATTN_VARLEN

template <typename K>
static bool allow_big_lds(K kern, int smem, bool& done)
{
    if (!done) {   // idempotent; a race only repeats the call
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return false;
        done = true;
    }
    return true;
}

// Variable-length backward: the prepare kernel sees the packed batch as one sequence of T rows
// (its outputs are then laid out [H, T]); dK/dV and dQ use the plan table.  Every head dim uses
// the unspecialised dK/dV kernel here.
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
    if (a.phases & 2) {
        constexpr int smem = 2 * BWD_BQ * (DQK + DV) * 2 + 1024;
        auto kern = attn_bwd_dkdv_varlen_kernel<DQK, DV, CAUSAL>;
        static bool attr_done = false;
        if (!allow_big_lds(kern, smem, attr_done)) return -3;
        if (launch_kernel(kern, dim3(a.max_tiles * a.Hkv), dim3(BWD_NT), smem, st,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.d_o,
                          (const float*)a.lse2, (const float*)a.D, (bf16*)a.dk, (bf16*)a.dv,
                          a.H, a.Hkv, a.scale, a.scale * kLog2e, (const int4*)a.plan, a.T, a.max_tiles) != hipSuccess)
            return -3;
    }
    if (a.phases & 4) {
        constexpr int smem = 2 * DQ_BN * (DQK + DV) * 2;
        auto kern = attn_bwd_dq_varlen_kernel<DQK, DV, CAUSAL>;
        static bool attr_done = false;
        if (!allow_big_lds(kern, smem, attr_done)) return -3;
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
        static bool attr_done = false;
        if (!allow_big_lds(kern, smem, attr_done)) return -3;
        const int grid = a.B * a.Hkv * (a.N / BWD_BK);
        if (launch_kernel(kern, dim3(grid), dim3(WS_NT), smem, st,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.d_o,
                          (const float*)a.lse2, (const float*)a.D, (bf16*)a.dk, (bf16*)a.dv,
                          a.H, a.Hkv, a.N, a.scale, a.scale * kLog2e) != hipSuccess)
            return -3;
    } } else if (a.phases & 2) {
        constexpr int smem = 2 * BWD_BQ * (DQK + DV) * 2 + 1024;
        auto kern = attn_bwd_dkdv_kernel<DQK, DV, CAUSAL>;
        static bool attr_done = false;
        if (!allow_big_lds(kern, smem, attr_done)) return -3;
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
        static bool attr_done = false;
        if (!allow_big_lds(kern, smem, attr_done)) return -3;
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
