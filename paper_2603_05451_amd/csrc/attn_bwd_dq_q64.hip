// The backward kernels with one wave per SIMD (gfx950), fixed-length batches:
//   attn_bwd_dq_q64_kernel    dQ with 64 queries per wave, head dims 128 and 64, long sequences, with or
//                             without the causal mask (attn_bwd_dq_q64_kernel.inc);
//   attn_bwd_dkdv_t32_kernel  dK / dV, its dual: K_w / V_w stationary, 32-query tiles of Q / dO streamed;
//                             head dims 128, (192, 128) with 32 keys per wave and 64 with 64 keys per wave
//                             (attn_bwd_dkdv_t32_kernel.inc).
// What is computed is described in attn_bwd.hip; how, at the top of the two kernel files.  A translation
// unit of its own, like attn_fwd_q64.hip, whose techniques it shares.
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
typedef bf16x2 elem2;
#include "attn_bwd_dq_q64_kernel.inc"
#include "attn_bwd_dkdv_t32_kernel.inc"
#include "attn_bwd_dq_t32_kernel.inc"
#undef ATTN_MFMA
#include "attn_bwd_dq_q64_launch.inc"

namespace f16k {
#define ATTN_ELEM f16
#define ATTN_ELEM8 f16x8
#define ATTN_ELEM4 f16x4
#include "elem.inc"
#undef ATTN_ELEM
#undef ATTN_ELEM8
#undef ATTN_ELEM4
#define ATTN_MFMA "v_mfma_f32_32x32x16_f16"
typedef __attribute__((ext_vector_type(2))) _Float16 elem2;
#include "attn_bwd_dq_q64_kernel.inc"
#include "attn_bwd_dkdv_t32_kernel.inc"
#include "attn_bwd_dq_t32_kernel.inc"
#undef ATTN_MFMA
#include "attn_bwd_dq_q64_launch.inc"
}  // namespace f16k

int launch_bwd_dq_q64(const BwdArgs& a) { return a.f16 ? f16k::launch_bwd_dq_q64_t(a) : launch_bwd_dq_q64_t(a); }
int launch_bwd_dq_t32(const BwdArgs& a) { return a.f16 ? f16k::launch_bwd_dq_t32_t(a) : launch_bwd_dq_t32_t(a); }
int launch_bwd_dkdv_t32(const BwdArgs& a) { return a.f16 ? f16k::launch_bwd_dkdv_t32_t(a) : launch_bwd_dkdv_t32_t(a); }

}  // namespace attn
