// Forward attention at head dims 128, 64 and (192, 128) with 64 queries per wave (gfx950): the long-sequence,
// fixed-length form of the forward pass.  What is computed is that of attn_fwd.hip (paper
// Sec. 2.1, online softmax with the thresholded rescale of Sec. 3.1.4, base 2); how the work is
// laid out is described at the top of attn_fwd_q64_kernel.inc.  A translation unit of its own:
// the kernel runs one wave per SIMD with accumulators in both halves of the register file, and
// its build flags are chosen for that.
#include "common.h"
#include "launch.h"

namespace attn {

#define ATTN_ELEM bf16
#define ATTN_ELEM8 bf16x8
#define ATTN_ELEM4 bf16x4
#include "elem.inc"
#undef ATTN_ELEM
#undef ATTN_ELEM8
#undef ATTN_ELEM4
#define ATTN_MFMA "v_mfma_f32_32x32x16_bf16"
#define ATTN_Q64_REPAIR 1
typedef bf16x2 elem2;
#include "attn_fwd_q64_kernel.inc"
#undef ATTN_MFMA
#undef ATTN_Q64_REPAIR
#include "attn_fwd_q64_launch.inc"

namespace f16k {
#define ATTN_ELEM f16
#define ATTN_ELEM8 f16x8
#define ATTN_ELEM4 f16x4
#include "elem.inc"
#undef ATTN_ELEM
#undef ATTN_ELEM8
#undef ATTN_ELEM4
#define ATTN_MFMA "v_mfma_f32_32x32x16_f16"
#define ATTN_Q64_REPAIR 0
typedef __attribute__((ext_vector_type(2))) _Float16 elem2;
#include "attn_fwd_q64_kernel.inc"
#undef ATTN_MFMA
#undef ATTN_Q64_REPAIR
#include "attn_fwd_q64_launch.inc"
}  // namespace f16k

int launch_fwd_q64(const FwdArgs& a) { return a.f16 ? f16k::launch_fwd_q64_t(a) : launch_fwd_q64_t(a); }

}  // namespace attn
