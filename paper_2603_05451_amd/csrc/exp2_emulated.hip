// Elementwise 2^x through the polynomial emulation of paper Sec. 3.1.3, built to MEASURE its accuracy
// on gfx950, not to use it: on this hardware v_exp_f32 issues from the same VALU port as the FMAs
// that would emulate it, so the emulation cannot add exponential throughput (the rate probes of
// probes.hip, a library of their own, show that).
#include "../../include/attn.h"
#include "exp2_emulation.h"
#include "launch.h"

namespace attn {

template <int DEG>
__global__ void __launch_bounds__(256) exp2_map_kernel(const float* __restrict__ x, float* __restrict__ y, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    if constexpr (DEG == 0) y[i] = __builtin_amdgcn_exp2f(x[i]);
    else y[i] = exp2_emulated<DEG>(x[i]);
}

}  // namespace attn

extern "C" {

int attn_exp2_emulated(const float* x, float* y, size_t n, int degree, void* stream)
{
    using namespace attn;
    if (!x || !y || n == 0) return ATTN_EINVAL;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    hipError_t e;
    switch (degree) {
        case 0: e = launch_kernel(exp2_map_kernel<0>, grid, block, 0, stream, x, y, n); break;
        case 3: e = launch_kernel(exp2_map_kernel<3>, grid, block, 0, stream, x, y, n); break;
        case 4: e = launch_kernel(exp2_map_kernel<4>, grid, block, 0, stream, x, y, n); break;
        case 5: e = launch_kernel(exp2_map_kernel<5>, grid, block, 0, stream, x, y, n); break;
        default: return ATTN_EUNSUPPORTED;
    }
    return e == hipSuccess ? ATTN_OK : ATTN_ELAUNCH;
}

}  // extern "C"
