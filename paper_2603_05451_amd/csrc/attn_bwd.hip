// Backward attention kernels for gfx950 (MI355X).
//
//   dV = P^T dO,  dP = dO V^T,  dS = P o (dP - D),  dQ = scale dS K,  dK = scale dS^T Q
// (paper Sec. 2.1) with P recomputed from Q, K and the saved row log-sum-exp, one
// workgroup per KV tile looping over query tiles, dK/dV accumulated on chip for the
// whole loop and dQ accumulated across workgroups (paper Sec. 3.2.2).
//
// Three kernels:
//   bwd_prepare : D_i = sum_c dO_ic O_ic (the identity sum_j P_ij dP_ij = dO_i . O_i that
//                 follows from the softmax Jacobian of Sec. 2.1), LSE in base-2 units, and
//                 the fp32 dQ accumulator cleared.  HBM bound.
//   bwd_main    : five MFMA contractions per (query tile, KV tile) pair.
//   bwd_finish  : dq = bf16(scale * dq_acc), from the head-major accumulator.  HBM bound.
//
// bwd_main layout.  Block = 4 waves = 128 keys (32 per wave); query tiles of 64 rows
// stream through LDS (double buffered, direct global->LDS copies); this wave's K and V
// rows stay in registers as MFMA B operands for the whole kernel.
//   S  = Q K_w^T   (queries on the MFMA row axis, this wave's 32 keys on the column axis)
//   dP = dO V_w^T
// so a lane owns one key column and 16 query rows per 32x32 block.  That register layout,
// converted to bf16, is directly the B operand (contraction over queries) of
//   dV_w^T += dO^T P      and      dK_w^T += Q^T dS,
// whose A operands come from the same Q / dO tiles through the transposing LDS read.
// This is the "compute the transposed product so that P and dS feed the next MMA from
// on-chip storage" idea of Sec. 3.2.2 restated for the MFMA register layout.
// dS additionally goes to LDS once (as dS^T, keys x queries) so that the four waves can
// contract over all 128 keys for dQ = dS K; each wave owns whole 32x32 blocks of the
// 64 x d_qk dQ tile and adds them to the fp32 accumulator with hardware float atomics.
#include "common.h"
#include "launch.h"

namespace attn {

constexpr int BWD_BK = 128;   // keys per block
constexpr int BWD_BQ = 64;    // queries per step
constexpr int BWD_NT = 256;

// ------------------------------------------------------------------------------------------
// bwd_prepare: one group of DV/8 lanes per (b, i, h) row.
template <int DQK, int DV>
__global__ void __launch_bounds__(256)
bwd_prepare_kernel(const bf16* __restrict__ o, const bf16* __restrict__ d_o, const float* __restrict__ lse,
                   float* __restrict__ D, float* __restrict__ lse2, float* __restrict__ dq_acc,
                   int H, int N, int64_t nrows)
{
    constexpr int LPR = DV / 8;                 // lanes per row
    constexpr int RPB = 256 / LPR;              // rows per block
    constexpr int ZPL = DQK / 4 / LPR;          // float4 zero-stores per lane
    static_assert(DQK / 4 % LPR == 0, "dq row must split evenly over the row's lanes");
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
    float4* z = (float4*)(dq_acc + row * DQK);
#pragma unroll
    for (int t = 0; t < ZPL; ++t) z[t * LPR + sub] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (sub == 0) {
        const int64_t bi = row / H;             // b*N + i
        const int h = (int)(row - bi * H);
        const int64_t b = bi / N;
        const int i = (int)(bi - b * N);
        const int64_t idx = (b * H + h) * N + i;
        D[idx] = acc;
        lse2[idx] = lse[idx] * kLog2e;
    }
}

// ------------------------------------------------------------------------------------------
// bwd_finish: dq[b, i, h, :] = bf16(scale * dq_acc[b, h, i, :]); one thread per 8 elements.
template <int DQK>
__global__ void __launch_bounds__(256)
bwd_finish_kernel(const float* __restrict__ dq_acc, bf16* __restrict__ dq, float scale, int H, int N, int64_t n8)
{
    constexpr int CPR = DQK / 8;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;   // output chunk index, token-major
    if (t >= n8) return;
    const int ch = (int)(t % CPR);
    const int64_t row = t / CPR;                                  // (b*N + i)*H + h
    const int64_t bi = row / H;
    const int h = (int)(row - bi * H);
    const int64_t b = bi / N;
    const int i = (int)(bi - b * N);
    const float4* src = (const float4*)(dq_acc + (((b * H + h) * N + i) * DQK + ch * 8));
    const float4 x = src[0], y = src[1];
    bf16x8 out;
    out[0] = (bf16)(x.x * scale); out[1] = (bf16)(x.y * scale);
    out[2] = (bf16)(x.z * scale); out[3] = (bf16)(x.w * scale);
    out[4] = (bf16)(y.x * scale); out[5] = (bf16)(y.y * scale);
    out[6] = (bf16)(y.z * scale); out[7] = (bf16)(y.w * scale);
    ((bf16x8*)dq)[t] = out;
}

// ------------------------------------------------------------------------------------------
template <int DQK, int DV, bool CAUSAL>
__global__ void __launch_bounds__(BWD_NT, 1)
attn_bwd_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                const bf16* __restrict__ d_o, const float* __restrict__ lse2, const float* __restrict__ D,
                float* __restrict__ dq_acc, bf16* __restrict__ dk, bf16* __restrict__ dv,
                int H, int Hkv, int N, float scale, float scale_log2e)
{
    constexpr int KSQ = DQK / 16, KSV = DV / 16;       // k-steps over the head dims
    constexpr int DBQ = DQK / 32, DBV = DV / 32;       // 32-wide head-dim blocks
    constexpr int QB = BWD_BQ / 32;                    // 32-query blocks per step (2)
    constexpr int K_BYTES = BWD_BK * DQK * 2;
    constexpr int Q_BYTES = BWD_BQ * DQK * 2;
    constexpr int DO_BYTES = BWD_BQ * DV * 2;
    constexpr int DS_BYTES = BWD_BK * BWD_BQ * 2;
    constexpr int NDQ = QB * DBQ / 4;                  // dQ blocks per wave
    static_assert(QB * DBQ % 4 == 0, "dQ blocks must split evenly over the four waves");

    extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
    ATTN_LDS char* smem = (ATTN_LDS char*)smem_raw;
    ATTN_LDS char* k_lds = smem;
    ATTN_LDS char* q_lds[2] = {smem + K_BYTES, smem + K_BYTES + Q_BYTES};
    ATTN_LDS char* do_lds[2] = {smem + K_BYTES + 2 * Q_BYTES, smem + K_BYTES + 2 * Q_BYTES + DO_BYTES};
    ATTN_LDS char* ds_lds = smem + K_BYTES + 2 * Q_BYTES + 2 * DO_BYTES;
    ATTN_LDS char* st_lds = ds_lds + DS_BYTES;        // [2 buffers][lse2 | D][64] floats

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int c = lane & 31, h = lane >> 5;
    const int i16 = lane & 15;
    // lane-constant parts of transposing-read addresses (4 rows x 32 bytes per 16 lanes)
    const int tr_row = i16 >> 2;                                    // + row base
    const int tr_chunk = 2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1);  // + 4 * (32-column block)
    const int tr_half = (i16 & 1) * 8;

    // ---- block -> (batch, kv head, kv tile); same XCD un-dealing as the forward kernel
    const int ntk = N / BWD_BK;
    const int total = gridDim.x;
    int vid = blockIdx.x;
    if ((total & 7) == 0) vid = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);
    const int bkv = vid / ntk;
    const int kt = vid - bkv * ntk;            // causal: tile 0 has the longest loop and comes first
    const int b = bkv / Hkv, kvh = bkv - b * Hkv;
    const int G = H / Hkv;
    const int k0 = kt * BWD_BK;
    const int kw0 = k0 + wave * 32;

    const int64_t q_stride = (int64_t)H * DQK, o_stride = (int64_t)H * DV;
    const int64_t k_stride = (int64_t)Hkv * DQK, v_stride = (int64_t)Hkv * DV;
    const bf16* kg = k + ((int64_t)b * N * Hkv + kvh) * DQK;
    const bf16* vg = v + ((int64_t)b * N * Hkv + kvh) * DV;

    const int i_first = CAUSAL ? k0 / BWD_BQ : 0;     // first query tile that sees this KV tile
    const int nq = N / BWD_BQ - i_first;
    const int nsteps = G * nq;

    auto issue_loads = [&](int step, int buf) {
        const int g = step / nq, i = i_first + (step - g * nq);
        const int hq = kvh * G + g;
        const int64_t row0 = (int64_t)b * N + (int64_t)i * BWD_BQ;
        tile_load_async<BWD_BQ, DQK, BWD_NT>(q + row0 * q_stride + (int64_t)hq * DQK, q_stride, q_lds[buf], tid);
        tile_load_async<BWD_BQ, DV, BWD_NT>(d_o + row0 * o_stride + (int64_t)hq * DV, o_stride, do_lds[buf], tid);
        if (wave < 2) {   // 64 floats each of lse2 and D
            const float* src = (wave == 0 ? lse2 : D) + ((int64_t)b * H + hq) * N + (int64_t)i * BWD_BQ + lane;
            dma4(src, st_lds + buf * 512 + wave * 256);
        }
    };

    // prologue: K tile -> LDS (for the dQ contraction), first query tile
    tile_load_async<BWD_BK, DQK, BWD_NT>(kg + (int64_t)k0 * k_stride, k_stride, k_lds, tid);
    issue_loads(0, 0);

    // this wave's K and V rows as B operands: lane = key kw0 + c, dims 16*ks + 8h .. +7
    bf16x8 kf[KSQ], vf[KSV];
    {
        const bf16* krow = kg + (int64_t)(kw0 + c) * k_stride + 8 * h;
        const bf16* vrow = vg + (int64_t)(kw0 + c) * v_stride + 8 * h;
#pragma unroll
        for (int ks = 0; ks < KSQ; ++ks) kf[ks] = *(const bf16x8*)(krow + 16 * ks);
#pragma unroll
        for (int ks = 0; ks < KSV; ++ks) vf[ks] = *(const bf16x8*)(vrow + 16 * ks);
#pragma unroll
        for (int ks = 0; ks < KSQ; ++ks) pin_ready(kf[ks]);
#pragma unroll
        for (int ks = 0; ks < KSV; ++ks) pin_ready(vf[ks]);
    }

    f32x16 dk_acc[DBQ], dv_acc[DBV];
#pragma unroll
    for (int db = 0; db < DBQ; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dk_acc[db][r] = 0.f;
#pragma unroll
    for (int db = 0; db < DBV; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dv_acc[db][r] = 0.f;

    // dQ blocks of the previous step.  Their atomic adds are issued one step late, right after
    // the top-of-step wait, so that they drain underneath a whole step of MFMA work instead of
    // being waited for by the next vmcnt(0).
    f32x16 dq_blk[NDQ];
    float* dq_dst = nullptr;
    auto flush_dq = [&]() {
#pragma unroll
        for (int n = 0; n < NDQ; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                unsafeAtomicAdd(dq_dst + acc_row(r, h) * DQK + 64 * n, dq_blk[n][r]);
    };

    for (int step = 0; step < nsteps; ++step) {
        const int buf = step & 1;
        wait_async_copies();
        __syncthreads();           // tiles of this step visible; previous step's dS reads finished
        if (step + 1 < nsteps) issue_loads(step + 1, buf ^ 1);
        if (step > 0) flush_dq();

        const int g = step / nq, i = i_first + (step - g * nq);
        const int hq = kvh * G + g;
        const int q0 = i * BWD_BQ;
        const bool diag = CAUSAL && (q0 < k0 + BWD_BK - 1);     // some (query, key) pair is masked

        bf16x8 pb[QB][2], dsb[QB][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            // ---- S = Q K_w^T and dP = dO V_w^T for 32 queries x 32 keys; LDS reads run one
            // group of 4 fragments ahead of the MFMAs that consume them
            f32x16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
            {
                constexpr int GRP = 4, NS = KSQ + KSV, NG = NS / GRP;
                static_assert(KSQ % GRP == 0 && KSV % GRP == 0, "k-steps must split into whole groups");
                bf16x8 fr[2][GRP];
                auto load_a = [&](int g, bf16x8* dst) {
#pragma unroll
                    for (int t = 0; t < GRP; ++t) {
                        const int st = g * GRP + t;
                        dst[t] = st < KSQ
                            ? lds_read_b128(q_lds[buf] + tile_off<DQK>(32 * qb + c, 2 * st + h))
                            : lds_read_b128(do_lds[buf] + tile_off<DV>(32 * qb + c, 2 * (st - KSQ) + h));
                    }
                };
                load_a(0, fr[0]);
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    if (g + 1 < NG) load_a(g + 1, fr[(g + 1) & 1]);
                    sched_fence();
#pragma unroll
                    for (int t = 0; t < GRP; ++t) {
                        const int st = g * GRP + t;
                        if (st < KSQ) s = mfma32(fr[g & 1][t], kf[st], s);
                        else dp = mfma32(fr[g & 1][t], vf[st - KSQ], dp);
                    }
                    sched_fence();
                }
            }

            // transposed fragments of dO and Q for the first 16 queries: in flight during the
            // elementwise work below
            bf16x4 tfr[2][DBV + DBQ][2];
            auto load_t = [&](int kk, bf16x4 (*dst)[2]) {
                const int row_lo = 32 * qb + 16 * kk + 4 * h + tr_row;   // queries, order 8s + 4h + j
#pragma unroll
                for (int db = 0; db < DBV; ++db) {
                    const ATTN_LDS char* base = do_lds[buf] + tr_half;
                    dst[db][0] = lds_read_tr(base + tile_off<DV>(row_lo, 4 * db + tr_chunk));
                    dst[db][1] = lds_read_tr(base + tile_off<DV>(row_lo + 8, 4 * db + tr_chunk));
                }
#pragma unroll
                for (int db = 0; db < DBQ; ++db) {
                    const ATTN_LDS char* base = q_lds[buf] + tr_half;
                    dst[DBV + db][0] = lds_read_tr(base + tile_off<DQK>(row_lo, 4 * db + tr_chunk));
                    dst[DBV + db][1] = lds_read_tr(base + tile_off<DQK>(row_lo + 8, 4 * db + tr_chunk));
                }
            };
            load_t(0, tfr[0]);
            sched_fence();

            // ---- P = 2^(c S - LSE2), dS = P o (dP - D); the query index is the register row
            const ATTN_LDS float* st = (const ATTN_LDS float*)(st_lds + buf * 512);
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const f32x4 L = *(const ATTN_LDS f32x4*)(st + 32 * qb + 8 * r4 + 4 * h);
                const f32x4 Dr = *(const ATTN_LDS f32x4*)(st + 64 + 32 * qb + 8 * r4 + 4 * h);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = 4 * r4 + e;
                    float p = fast_exp2(fmaf(s[r], scale_log2e, -L[e]));
                    if (diag && (kw0 + c > q0 + 32 * qb + 8 * r4 + 4 * h + e)) p = 0.f;
                    const float ds = p * (dp[r] - Dr[e]);
                    pb[qb][r >> 3][r & 7] = (bf16)p;
                    dsb[qb][r >> 3][r & 7] = (bf16)ds;
                }
            }

            // ---- dS^T (keys x queries) to LDS for the dQ contraction: 4 queries = 8 bytes
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                bf16x4 w4;
#pragma unroll
                for (int e = 0; e < 4; ++e) w4[e] = dsb[qb][r4 >> 1][4 * (r4 & 1) + e];
                *(ATTN_LDS bf16x4*)(ds_lds + tile_off<BWD_BQ>(32 * wave + c, 4 * qb + r4) + 8 * h) = w4;
            }

            // ---- dV_w^T += dO^T P,  dK_w^T += Q^T dS   (contraction over these 32 queries)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                if (kk + 1 < 2) load_t(kk + 1, tfr[(kk + 1) & 1]);
                sched_fence();
#pragma unroll
                for (int db = 0; db < DBV; ++db)
                    dv_acc[db] = mfma32(cat4(tfr[kk & 1][db][0], tfr[kk & 1][db][1]), pb[qb][kk], dv_acc[db]);
#pragma unroll
                for (int db = 0; db < DBQ; ++db)
                    dk_acc[db] = mfma32(cat4(tfr[kk & 1][DBV + db][0], tfr[kk & 1][DBV + db][1]), dsb[qb][kk],
                                        dk_acc[db]);
                sched_fence();
            }
        }

        __syncthreads();           // dS^T of all four waves is in LDS

        // ---- dQ blocks: (32 queries) x (32 dims), contraction over the block's 128 keys
        {
            const int qb = wave & 1;
            constexpr int NKS = BWD_BK / 16;
#pragma unroll
            for (int n = 0; n < NDQ; ++n)
#pragma unroll
                for (int r = 0; r < 16; ++r) dq_blk[n][r] = 0.f;
            bf16x4 fr[2][1 + NDQ][2];
            auto load_dq = [&](int ks, bf16x4 (*dst)[2]) {
                const int row_lo = 16 * ks + 8 * h + tr_row;             // keys, natural order 8h + 4s + j
                const ATTN_LDS char* abase = ds_lds + tr_half;
                dst[0][0] = lds_read_tr(abase + tile_off<BWD_BQ>(row_lo, 4 * qb + tr_chunk));
                dst[0][1] = lds_read_tr(abase + tile_off<BWD_BQ>(row_lo + 4, 4 * qb + tr_chunk));
#pragma unroll
                for (int n = 0; n < NDQ; ++n) {
                    const int db = (wave >> 1) + 2 * n;
                    const ATTN_LDS char* bbase = k_lds + tr_half;
                    dst[1 + n][0] = lds_read_tr(bbase + tile_off<DQK>(row_lo, 4 * db + tr_chunk));
                    dst[1 + n][1] = lds_read_tr(bbase + tile_off<DQK>(row_lo + 4, 4 * db + tr_chunk));
                }
            };
            load_dq(0, fr[0]);
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                if (ks + 1 < NKS) load_dq(ks + 1, fr[(ks + 1) & 1]);
                sched_fence();
                const bf16x8 a = cat4(fr[ks & 1][0][0], fr[ks & 1][0][1]);
#pragma unroll
                for (int n = 0; n < NDQ; ++n)
                    dq_blk[n] = mfma32(a, cat4(fr[ks & 1][1 + n][0], fr[ks & 1][1 + n][1]), dq_blk[n]);
                sched_fence();
            }
            // accumulator is head-major [B, H, N, d_qk]: a dQ tile is one contiguous region;
            // block n of this wave covers dims 32 * (wave/2 + 2n) .. +31
            dq_dst = dq_acc + (((int64_t)b * H + hq) * N + q0 + 32 * qb) * DQK + 32 * (wave >> 1) + c;
        }
    }
    if (nsteps > 0) flush_dq();

    // ---- epilogue: dk = scale * dK, dv = dV; accumulators hold the transposes (dims x keys)
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

template <int DQK, int DV, bool CAUSAL>
static int launch_bwd_t(const BwdArgs& a)
{
    void* st = a.stream;
    const int64_t nrows = (int64_t)a.B * a.N * a.H;
    if (a.phases & 1) {
        constexpr int RPB = 256 / (DV / 8);
        if (launch_kernel(bwd_prepare_kernel<DQK, DV>, dim3((unsigned)((nrows + RPB - 1) / RPB)), dim3(256), 0, st,
                          (const bf16*)a.o, (const bf16*)a.d_o, a.lse, a.D, a.lse2, a.dq_acc, a.H, a.N,
                          nrows) != hipSuccess)
            return -3;
    }
    if (a.phases & 2) {
        constexpr int smem = BWD_BK * DQK * 2 + 2 * BWD_BQ * (DQK + DV) * 2 + BWD_BK * BWD_BQ * 2 + 1024;
        auto kern = attn_bwd_kernel<DQK, DV, CAUSAL>;
        static bool attr_done = false;   // idempotent; a race only repeats the call
        if (!attr_done) {
            if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
                return -3;
            attr_done = true;
        }
        const int grid = a.B * a.Hkv * (a.N / BWD_BK);
        if (launch_kernel(kern, dim3(grid), dim3(BWD_NT), smem, st,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (const bf16*)a.d_o,
                          (const float*)a.lse2, (const float*)a.D, a.dq_acc, (bf16*)a.dk, (bf16*)a.dv,
                          a.H, a.Hkv, a.N, a.scale, a.scale * kLog2e) != hipSuccess)
            return -3;
    }
    if (a.phases & 4) {
        const int64_t n8 = nrows * DQK / 8;
        if (launch_kernel(bwd_finish_kernel<DQK>, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, st,
                          (const float*)a.dq_acc, (bf16*)a.dq, a.scale, a.H, a.N, n8) != hipSuccess)
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
