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
#define ATTN_VARLEN 0
#include "attn_fwd_kernel.inc"
#undef ATTN_VARLEN
#define ATTN_VARLEN 1
#include "attn_fwd_kernel.inc"
#undef ATTN_VARLEN

template <int DQK, int DV, bool CAUSAL>
static int launch_fwd_t(const FwdArgs& a)
{
    constexpr int smem = 2 * FWD_BN * (DQK + DV) * 2;
    hipError_t e;
    if (a.plan) {
        auto kern = attn_fwd_varlen_kernel<DQK, DV, CAUSAL>;
        static LdsOptIn lds;
        if (!lds.allow(kern, smem)) return -3;
        e = launch_kernel(kern, dim3(a.max_tiles * a.H), dim3(FWD_NT), smem, a.stream,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (bf16*)a.o, a.lse,
                          a.H, a.Hkv, a.scale * kLog2e, (const int4*)a.plan, a.T, a.max_tiles);
    } else {
        auto kern = attn_fwd_kernel<DQK, DV, CAUSAL>;
        static LdsOptIn lds;
        if (!lds.allow(kern, smem)) return -3;
        e = launch_kernel(kern, dim3(a.B * a.H * (a.N / FWD_BM)), dim3(FWD_NT), smem, a.stream,
                          (const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, (bf16*)a.o, a.lse,
                          a.H, a.Hkv, a.N, a.scale * kLog2e);
    }
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
