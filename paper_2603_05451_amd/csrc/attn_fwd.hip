// Forward attention kernel for gfx950 (MI355X).
//
// Computes O = softmax(scale * Q K^T [+ causal mask]) V and the row log-sum-exp
// (paper Sec. 2.1) with the tiled online softmax and thresholded rescaling of
// paper Sec. 3.1.4, in base 2 (scores are multiplied by scale * log2(e) inside the
// exponent's FMA, matching the 2^x formulation of Sec. 3.1.3).
//
// Work decomposition
//   block  = 256 threads = 4 waves, one (batch, query head, 128-query tile);
//   wave w = 32 query rows; it keeps its Q rows in registers for the whole kernel;
//   K/V tiles of BN = 64 keys stream through LDS, double buffered, copied straight
//   from global memory into LDS (no VGPR staging) one tile ahead of the compute.
//
// MFMA orientation.  Scores are computed TRANSPOSED, S^T = K Q^T (keys on the MFMA row
// axis, queries on the column axis).  In the 32x32 accumulator layout a lane then owns
// one query (column lane%32) and 16 keys per 32-key block, so the row max and row sum of
// the softmax are in-lane reductions plus one exchange with the lane 32 apart, and the
// running statistics are one register per lane.  The same registers, converted to bf16,
// are already in the B-operand layout of O^T += V^T P^T (contraction over keys), so P
// never goes through LDS.  V^T fragments come from the row-major V tile in LDS through
// the transposing LDS read.
#include "common.h"
#include "launch.h"

namespace attn {

constexpr int FWD_BM = 128;   // query rows per block
constexpr int FWD_BN = 64;    // keys per tile
constexpr int FWD_NT = 256;

#ifndef ATTN_FWD_OCC192
#define ATTN_FWD_OCC192 2
#endif
template <int DQK, int DV, bool CAUSAL>
__global__ void __launch_bounds__(FWD_NT, (DQK > 128 ? ATTN_FWD_OCC192 : 2))
attn_fwd_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                bf16* __restrict__ o, float* __restrict__ lse,
                int H, int Hkv, int N, float scale_log2e)
{
    constexpr int KS = DQK / 16;            // MFMA k-steps over the head dim (QK^T)
    constexpr int DB = DV / 32;             // 32-wide blocks of the output head dim
    constexpr int KB = FWD_BN / 32;         // 32-key blocks per tile
    constexpr int K_TILE_BYTES = FWD_BN * DQK * 2;
    constexpr int V_TILE_BYTES = FWD_BN * DV * 2;

    extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
    ATTN_LDS char* smem = (ATTN_LDS char*)smem_raw;
    ATTN_LDS char* k_lds[2] = {smem, smem + K_TILE_BYTES};
    ATTN_LDS char* v_lds[2] = {smem + 2 * K_TILE_BYTES, smem + 2 * K_TILE_BYTES + V_TILE_BYTES};

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int c = lane & 31, h = lane >> 5;

    // ---- block -> (batch, head, query tile).  Blocks are dealt to the 8 XCDs round robin
    // by linear id; undo that so that consecutive virtual ids (the query tiles of one head,
    // then the next head of the same KV group) share an XCD and hence an L2.
    const int ntq = N / FWD_BM;
    const int total = gridDim.x;
    int vid = blockIdx.x;
    if ((total & 7) == 0) vid = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);
    const int bh = vid / ntq;
    int qt = vid - bh * ntq;
    if (CAUSAL) qt = ntq - 1 - qt;          // longest tiles first
    const int b = bh / H, hq = bh - b * H;
    const int kvh = hq / (H / Hkv);
    const int q0 = qt * FWD_BM;
    const int qw0 = q0 + wave * 32;         // first query row of this wave

    const int64_t q_stride = (int64_t)H * DQK, o_stride = (int64_t)H * DV;
    const int64_t k_stride = (int64_t)Hkv * DQK, v_stride = (int64_t)Hkv * DV;
    const bf16* kg = k + ((int64_t)b * N * Hkv + kvh) * DQK;
    const bf16* vg = v + ((int64_t)b * N * Hkv + kvh) * DV;

    const int ntiles = CAUSAL ? (q0 + FWD_BM) / FWD_BN : N / FWD_BN;

    // prologue: start the copy of tile 0
    TileCopy<FWD_BN, DQK, FWD_NT> kcopy;
    TileCopy<FWD_BN, DV, FWD_NT> vcopy;
    kcopy.init(k_stride, tid);
    vcopy.init(v_stride, tid);
    kcopy.issue_all(kg, k_lds[0]);
    vcopy.issue_all(vg, v_lds[0]);

    // Q fragments (B operand of S^T = K Q^T): lane holds query qw0 + c, dims 16*ks + 8h .. +7
    bf16x8 qf[KS];
    {
        const bf16* qrow = q + ((int64_t)b * N + qw0 + c) * q_stride + (int64_t)hq * DQK + 8 * h;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(qrow + 16 * ks);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) pin_ready(qf[ks]);
    }

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m_ref = -INFINITY;   // reference maximum actually used (base-2 units), may be stale
    float l_part = 0.f;        // this lane's share of the row sum (its 32 of the 64 keys per tile)

    // lane-constant parts of the LDS read addresses
    // K: row = 32*kb + c, logical chunk = 2*ks + h
    // V (transposing read): row = 16*kk + 8*s + 4*h + i/4, logical chunk = 4*db + 2*((lane/16)&1) + (i%4)/2
    const int i16 = lane & 15;
    const int v_row0 = 4 * h + (i16 >> 2);
    const int v_chunk0 = 2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1);
    const int v_half = (i16 & 1) * 8;

    // One KV tile.  The buffer index is a template constant (the loop below is unrolled by two)
    // so that every LDS read address is "lane register + immediate": no per-tile address
    // arithmetic on the vector ALU.
    auto tile_step = [&](auto bufc, int j) {
        const int buf = bufc;               // compile-time constant in the unrolled variants
        wait_async_copies();
        __syncthreads();                    // tile j visible to all; everyone is done with tile j-1
        if (j + 1 < ntiles) {
            kcopy.issue_all(kg + (int64_t)(j + 1) * FWD_BN * k_stride, k_lds[buf ^ 1]);
            vcopy.issue_all(vg + (int64_t)(j + 1) * FWD_BN * v_stride, v_lds[buf ^ 1]);
        }
        const int key0 = j * FWD_BN;
        if (CAUSAL && key0 > qw0 + 31) return;     // whole tile above this wave's diagonal

        // ---- S^T = K Q^T : KB blocks of 32 keys x 32 queries.  LDS reads run one group of
        // GRP fragments ahead of the MFMAs that consume them.
        f32x16 s[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
        {
            constexpr int GRP = 4, NG = KB * KS / GRP;
            static_assert(KB * KS % GRP == 0, "k-steps must split into whole groups");
            bf16x8 kfr[2][GRP];
            auto load_k = [&](int g, bf16x8* dst) {
#pragma unroll
                for (int t = 0; t < GRP; ++t) {
                    const int st = g * GRP + t, kb = st / KS, ks = st % KS;
                    dst[t] = lds_read_b128(k_lds[buf] + tile_off<DQK>(32 * kb + c, 2 * ks + h));
                }
            };
            load_k(0, kfr[0]);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                if (g + 1 < NG) load_k(g + 1, kfr[(g + 1) & 1]);
                sched_fence();
#pragma unroll
                for (int t = 0; t < GRP; ++t) {
                    const int st = g * GRP + t, kb = st / KS, ks = st % KS;
                    s[kb] = mfma32(kfr[g & 1][t], qf[ks], s[kb]);
                }
                sched_fence();
            }
        }

        // first group of V^T fragments: in flight during the softmax arithmetic
        bf16x4 vfr[2][DB][2];
        auto load_v = [&](int kk, bf16x4 (*dst)[2]) {
            const ATTN_LDS char* base = v_lds[buf] + v_half;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                dst[db][0] = lds_read_tr(base + tile_off<DV>(16 * kk + v_row0, 4 * db + v_chunk0));
                dst[db][1] = lds_read_tr(base + tile_off<DV>(16 * kk + 8 + v_row0, 4 * db + v_chunk0));
            }
        };
        load_v(0, vfr[0]);
        sched_fence();

        // ---- causal mask on tiles that straddle the diagonal
        if (CAUSAL && key0 + FWD_BN - 1 > qw0) {
            const int qi = qw0 + c;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (key0 + 32 * kb + acc_row(r, h) > qi) s[kb][r] = -INFINITY;
        }

        // ---- running maximum with thresholded rescale (paper Sec. 3.1.4)
        float tmax = s[0][0];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[kb][r]);
        tmax = xhalf_max(tmax) * scale_log2e;          // scale > 0, so max and scaling commute
        const float m_new = fmaxf(m_ref, tmax);
        if (__any(m_new - m_ref > kRescaleTau)) {      // wave-uniform vote: no divergence
            const float alpha = fast_exp2(m_ref - m_new);   // 0 on the first tile (m_ref = -inf)
            m_ref = m_new;
            l_part *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
        }

        // ---- P^T = 2^(c S^T - m_ref), row sum in fp32, then bf16
        bf16x8 pf[KB][2];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = fast_exp2(fmaf(s[kb][r], scale_log2e, -m_ref));
                l_part += p;
                pf[kb][r >> 3][r & 7] = (bf16)p;
            }

        // ---- O^T += V^T P^T : contraction over the 64 keys in 4 steps of 16
#pragma unroll
        for (int kk = 0; kk < 2 * KB; ++kk) {
            if (kk + 1 < 2 * KB) load_v(kk + 1, vfr[(kk + 1) & 1]);
            sched_fence();
#pragma unroll
            for (int db = 0; db < DB; ++db)
                oacc[db] = mfma32(cat4(vfr[kk & 1][db][0], vfr[kk & 1][db][1]), pf[kk >> 1][kk & 1], oacc[db]);
            sched_fence();
        }
    };
    if constexpr (DQK <= 128) {
        for (int j = 0; j < ntiles; j += 2) {      // ntiles is even (N and the causal bound are multiples of 128)
            tile_step(std::integral_constant<int, 0>{}, j);
            tile_step(std::integral_constant<int, 1>{}, j + 1);
        }
    } else {                                       // d_qk = 192: the unrolled body does not fit 256 VGPRs
        for (int j = 0; j < ntiles; ++j) tile_step(j & 1, j);
    }

    // ---- epilogue: O = acc / l, LSE = ln2 * (m_ref + log2 l)   (relative to the reference used)
    const float l = xhalf_sum(l_part);
    const float inv_l = 1.0f / l;
    bf16* orow = o + ((int64_t)b * N + qw0 + c) * o_stride + (int64_t)hq * DV;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            bf16x4 out;
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = (bf16)(oacc[db][4 * r4 + e] * inv_l);
            *(bf16x4*)(orow + 32 * db + 8 * r4 + 4 * h) = out;
        }
    if (h == 0) lse[((int64_t)b * H + hq) * N + qw0 + c] = (m_ref + fast_log2(l)) * kLn2;
}

template <int DQK, int DV, bool CAUSAL>
static int launch_fwd_t(const FwdArgs& a)
{
    constexpr int smem = 2 * FWD_BN * (DQK + DV) * 2;
    auto kern = attn_fwd_kernel<DQK, DV, CAUSAL>;
    static bool attr_done = false;   // idempotent; a race only repeats the call
    if (!attr_done) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return -3;
        attr_done = true;
    }
    const int grid = a.B * a.H * (a.N / FWD_BM);
    const hipError_t e = launch_kernel(kern, dim3(grid), dim3(FWD_NT), smem, a.stream,
                                       (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (bf16*)a.o, a.lse,
                                       a.H, a.Hkv, a.N, a.scale * kLog2e);
    return e == hipSuccess ? 0 : -3;
}

int launch_fwd(const FwdArgs& a)
{
    if (a.d_qk == 64 && a.d_v == 64)
        return a.causal ? launch_fwd_t<64, 64, true>(a) : launch_fwd_t<64, 64, false>(a);
    if (a.d_qk == 128 && a.d_v == 128)
        return a.causal ? launch_fwd_t<128, 128, true>(a) : launch_fwd_t<128, 128, false>(a);
    if (a.d_qk == 192 && a.d_v == 128)
        return a.causal ? launch_fwd_t<192, 128, true>(a) : launch_fwd_t<192, 128, false>(a);
    return -2;
}

}  // namespace attn
