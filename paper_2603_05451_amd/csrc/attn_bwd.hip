// Backward attention kernels for gfx950 (MI355X).
//
//   dV = P^T dO,  dP = dO V^T,  dS = P o (dP - D),  dQ = scale dS K,  dK = scale dS^T Q
// (paper Sec. 2.1) with P recomputed from Q, K and the saved row log-sum-exp.
//
// Kernels (a backward call launches bwd_dq, then bwd_dkdv):
//   bwd_prepare : D_i = sum_c dO_ic O_ic (the identity sum_j P_ij dP_ij = dO_i . O_i that
//                 follows from the softmax Jacobian of Sec. 2.1), stored as -D_i, and LSE in
//                 base-2 units.  HBM bound.
//   bwd_dkdv    : one workgroup per KV tile looping over query tiles, dK and dV accumulated
//                 on chip for the whole loop (the loop structure of paper Sec. 3.2.2).
//   bwd_dq      : one workgroup per query tile looping over KV tiles, dQ accumulated on chip.
//                 It does the prepare kernel's work for its own rows, runs first and replaces
//                 that kernel (which remains for attn_bwd_phases without the dQ pass).
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

#ifndef ATTN_BWD_VGPR_FORM_PART
#define ATTN_BWD_VGPR_FORM_PART 0     // 1: the pass that compiles only the kernels listed in attn_bwd_all.inc
#endif

namespace attn {

constexpr int BWD_BK = 128;   // dkdv: keys per block
constexpr int BWD_BQ = 64;    // dkdv: queries per step
constexpr int BWD_NT = 256;
constexpr int DQ_BM = 128;    // dq: queries per block
constexpr int DQ_BN = 64;     // dq: keys per step

constexpr int WS_NT = 512;    // wave-specialised dK/dV kernel: threads per block
constexpr int WS_STAGES = 3;  //   LDS stages of the query / dO tiles
constexpr int WS_PDS_BYTES = 4 * 8 * 1024;   // 4 key groups x (2 query blocks x (P, dS) x 2 halves) x 64 lanes x 16 B

// ---- bf16 kernels
#define ATTN_ELEM bf16
#define ATTN_ELEM8 bf16x8
#define ATTN_ELEM4 bf16x4
#include "elem.inc"
#undef ATTN_ELEM
#undef ATTN_ELEM8
#undef ATTN_ELEM4
#include "attn_bwd_all.inc"

// ---- fp16 kernels: the same text, element type _Float16
namespace f16k {
#define ATTN_ELEM f16
#define ATTN_ELEM8 f16x8
#define ATTN_ELEM4 f16x4
#include "elem.inc"
#undef ATTN_ELEM
#undef ATTN_ELEM8
#undef ATTN_ELEM4
#include "attn_bwd_all.inc"
}  // namespace f16k

#if !ATTN_BWD_VGPR_FORM_PART
int launch_bwd(const BwdArgs& a)
{
    // Fixed-length batches at head dims 128, 64 and (192, 128): kernels with one wave per SIMD
    // (attn_bwd_dq_q64.hip), faster than the kernels of this file.  The dK/dV kernel gives the same bits
    // as they do; the dQ kernel differs by the fp32 rounding of dP - D.  The dQ kernel, and with it -D and
    // the base-2 LSE, comes first as in every backward call.
    auto generic = [&](int phases) {
        BwdArgs part = a;
        part.phases = phases;
        return a.f16 ? f16k::launch_bwd_dims(part) : launch_bwd_dims(part);
    };
    const bool d128 = a.d_qk == 128 && a.d_v == 128, d64 = a.d_qk == 64 && a.d_v == 64, d192 = a.d_qk == 192 && a.d_v == 128;
    // below these lengths the 4-wave dQ kernel wins (its blocks are half the size and fill the chip better);
    // at d = 64 the 256-key blocks of the dK/dV kernel are too few on short sequences (measured against the
    // 4-wave kernel: +10 % at N = 512, +1 % at N = 1024, -4 % at N = 2048; under the mask +4 % at N = 4096, -6 % at N = 8192)
    const bool dq_q64 = (a.phases & 4) && !a.plan && a.N % 256 == 0 &&
                        ((d128 && a.N >= (a.causal ? 4096 : 1024)) || (d64 && a.N >= (a.causal ? 8192 : 2048)));
    const bool dkdv_t32 = (a.phases & 2) && !a.plan &&
                          (((d128 || d192) && a.N % 128 == 0) || (d64 && a.N % 256 == 0 && a.N >= (a.causal ? 8192 : 2048)));
    // (192, 128): the 64-query kernel's fragments and accumulators do not fit; 32 queries per wave, pipelined
    const bool dq_t32 = (a.phases & 4) && !a.plan && d192 && a.N % 128 == 0 && a.N >= (a.causal ? 1024 : 512);
    if (!dq_q64 && !dq_t32 && !dkdv_t32) return generic(a.phases);
    if (dq_q64) {
        if (const int rc = launch_bwd_dq_q64(a)) return rc;
    } else if (dq_t32) {
        if (const int rc = launch_bwd_dq_t32(a)) return rc;
    } else if (a.phases & 5) {
        if (const int rc = generic(a.phases & 5)) return rc;
    }
    if (dkdv_t32) return launch_bwd_dkdv_t32(a);
    return (a.phases & 2) ? generic(2) : 0;
}
#endif

}  // namespace attn
