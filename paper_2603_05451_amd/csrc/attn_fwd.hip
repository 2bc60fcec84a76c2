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
//   At d = 128, 64 and (192, 128) and long fixed-length sequences the kernel of attn_fwd_q64.hip runs instead (64
//   queries per wave, one wave per SIMD).
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

// ---- bf16 kernels
#define ATTN_ELEM bf16
#define ATTN_ELEM8 bf16x8
#define ATTN_ELEM4 bf16x4
#include "elem.inc"
#undef ATTN_ELEM
#undef ATTN_ELEM8
#undef ATTN_ELEM4
#define ATTN_VARLEN 0
#include "attn_fwd_kernel.inc"
#undef ATTN_VARLEN
#define ATTN_VARLEN 1
#include "attn_fwd_kernel.inc"
#undef ATTN_VARLEN
#include "attn_fwd_launch.inc"

// ---- fp16 kernels: the same text, element type _Float16 (v_mfma_f32_32x32x16_f16)
namespace f16k {
#define ATTN_ELEM f16
#define ATTN_ELEM8 f16x8
#define ATTN_ELEM4 f16x4
#include "elem.inc"
#undef ATTN_ELEM
#undef ATTN_ELEM8
#undef ATTN_ELEM4
#define ATTN_VARLEN 0
#include "attn_fwd_kernel.inc"
#undef ATTN_VARLEN
#define ATTN_VARLEN 1
#include "attn_fwd_kernel.inc"
#undef ATTN_VARLEN
#include "attn_fwd_launch.inc"
}  // namespace f16k

int launch_fwd(const FwdArgs& a) { return a.f16 ? f16k::launch_fwd_dims(a) : launch_fwd_dims(a); }

}  // namespace attn
