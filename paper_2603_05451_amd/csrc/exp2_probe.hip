// Software 2^x on the vector ALU (paper Sec. 3.1.3), built to MEASURE it on gfx950, not to use
// it: on this hardware v_exp_f32 issues from the same VALU port as the FMAs that would emulate
// it, so the emulation cannot add exponential throughput (see the throughput entry point).
//
// Steps of the section: clamp to >= -127; floor (v_floor_f32 here; the section's
// add-and-subtract of 2^23 + 2^22 in round-down mode computes the same function); fractional
// part; polynomial with p0 = 1 by Horner's rule with FMAs; integer part shifted into the exponent
// field and added to the polynomial's bits.  Coefficients: minimax relative error on [0, 1),
// from gen_exp2_coeffs.py (Remez exchange); the section prints none.
#include "../../include/attn.h"
#include "common.h"
#include "launch.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attn {

template <int DEG> struct Exp2Poly;
template <> struct Exp2Poly<3> { static constexpr float p[3] = {6.951167583e-01f, 2.276449949e-01f, 7.706703991e-02f}; };
template <> struct Exp2Poly<4> { static constexpr float p[4] = {6.930448413e-01f, 2.412801981e-01f, 5.224247277e-02f, 1.342668384e-02f}; };
template <> struct Exp2Poly<5> { static constexpr float p[5] = {6.931512952e-01f, 2.401644439e-01f, 5.579991266e-02f, 9.017030708e-03f, 1.867130050e-03f}; };

template <int DEG>
__device__ __forceinline__ float exp2_emulated(float x)
{
    x = fmaxf(x, -127.0f);
    const float fl = __builtin_floorf(x);
    const float f = x - fl;
    float acc = Exp2Poly<DEG>::p[DEG - 1];
#pragma unroll
    for (int i = DEG - 2; i >= 0; --i) acc = __builtin_fmaf(acc, f, Exp2Poly<DEG>::p[i]);
    acc = __builtin_fmaf(acc, f, 1.0f);
    return __int_as_float(__float_as_int(acc) + ((int)fl << 23));
}

template <int DEG>
__global__ void __launch_bounds__(256) exp2_map_kernel(const float* __restrict__ x, float* __restrict__ y, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    if constexpr (DEG == 0) y[i] = __builtin_amdgcn_exp2f(x[i]);
    else y[i] = exp2_emulated<DEG>(x[i]);
}

// ALU throughput: 8 independent evaluations per thread and iteration, arguments kept in [0, 1)
template <int DEG>
__global__ void __launch_bounds__(256) exp2_rate_kernel(float* __restrict__ out, int iters)
{
    float v[8], s[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { v[e] = 0.03f * e + 1e-4f * threadIdx.x; s[e] = 0.f; }
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float r;
            if constexpr (DEG == 0) r = __builtin_amdgcn_exp2f(v[e]);
            else r = exp2_emulated<DEG>(v[e]);
            s[e] += r;
            v[e] = r - 1.0f;              // back into [0, 1): a dependent chain per slot, 8 slots in flight
        }
    float t = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) t += s[e];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = t;
}

// Partial emulation (paper Sec. 3.1.3: a share of every row goes through the polynomial, the rest
// through the hardware unit, so that both work at once): EMU of the 8 evaluation slots of a thread
// use the degree-3 polynomial, the others v_exp_f32.
template <int EMU>
__global__ void __launch_bounds__(256) exp2_rate_partial_kernel(float* __restrict__ out, int iters)
{
    float v[8], s[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { v[e] = 0.03f * e + 1e-4f * threadIdx.x; s[e] = 0.f; }
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float r = e < EMU ? exp2_emulated<3>(v[e]) : __builtin_amdgcn_exp2f(v[e]);
            s[e] += r;
            v[e] = r - 1.0f;
        }
    float t = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) t += s[e];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = t;
}

// Matrix-core ceiling: nothing but v_mfma_f32_32x32x16_bf16 on register operands, two waves per
// SIMD, four accumulation chains per wave.  With random operands the chip's power management
// lowers the shader clock; the rate this kernel sustains is what any bf16 MFMA kernel on such
// data is bounded by, whatever its instruction stream.
__device__ __forceinline__ float hash_gauss(uint32_t s)   // sum of four uniforms, variance 1
{
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s = s * 1664525u + 1013904223u; s ^= s >> 15; s *= 2246822519u; s ^= s >> 13;
        acc += (float)(s >> 8) * (1.0f / 16777216.0f);
    }
    return (acc - 2.0f) * 1.7320508f;
}

__global__ void __launch_bounds__(512) mfma_rate_kernel(float* __restrict__ out, int iters, int random_operands)
{
    typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
    typedef __attribute__((ext_vector_type(16))) float f32x16;
    bf16x8 a[8], b[8];
#pragma unroll
    for (int f = 0; f < 8; ++f)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t id = ((blockIdx.x * 512 + threadIdx.x) * 8 + f) * 8 + e;
            a[f][e] = (__bf16)(random_operands ? hash_gauss(id) : 1.0f);
            b[f][e] = (__bf16)(random_operands ? hash_gauss(id + 0x9e3779b9u) : 0.5f);
        }
    f32x16 c[4] = {{0}, {0}, {0}, {0}};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int m = 0; m < 32; ++m)
            c[m % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m % 8], b[(m / 4) % 8], c[m % 4], 0, 0, 0);
        if ((i & 255) == 255) {   // keep the accumulators finite
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int r = 0; r < 16; ++r) c[m][r] *= 1e-6f;
        }
    }
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = c[0][0] + c[1][1] + c[2][2] + c[3][3];
}

// LDS read rate in the two access patterns of the attention kernels, on a swizzled 64 x 128 tile
// of 16-bit elements: PATTERN 0 = ds_read_b128 of MFMA A-operand fragments (K, Q, dO: lane =
// tile row c, 16-byte chunk 2*ks + h), PATTERN 1 = ds_read_b64_tr_b16 of transposed fragments
// (V^T, K^T, Q^T, dO^T).  Eight reads are kept in flight per wave; the data are never used for
// arithmetic.  256 threads per block, 2 blocks per CU resident (32 KiB of LDS each).
template <int PATTERN>
__global__ void __launch_bounds__(256, 2) lds_rate_kernel(float* __restrict__ out, int iters)
{
    __shared__ __attribute__((aligned(1024))) char tile[4][8192];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 4 * 8192 / 4; i += 256) ((float*)tile)[i] = (float)i;
    __syncthreads();
    const ATTN_LDS char* base = (const ATTN_LDS char*)&tile[0][0] + (wave & 1) * 16384;
    const int h = lane >> 5, c = lane & 31, i16 = lane & 15;
    const ATTN_LDS char* p[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        if (PATTERN == 0) {
            p[u] = base + tile_off<128>(c, 2 * u + h);
        } else {
            const int kk = u >> 2, db = u & 3;
            p[u] = base + tile_off<128>(16 * kk + 4 * h + (i16 >> 2), 4 * db + 2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1)) +
                   (i16 & 1) * 8;
        }
    }
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (PATTERN == 0) {
                f32x4 v;
                asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(7)" : "=v"(v) : "v"(p[u]) : "memory");
                acc += v[0];
            } else {
                float2 v;
                asm volatile("ds_read_b64_tr_b16 %0, %1\n\ts_waitcnt lgkmcnt(7)" : "=v"(v) : "v"(p[u]) : "memory");
                acc += v.x;
            }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    out[(size_t)blockIdx.x * 256 + tid] = acc;
}

}  // namespace attn

extern "C" {

long long attn_lds_rate(float* out, int pattern, int iters, void* stream)
{
    using namespace attn;
    if (!out || iters <= 0) return ATTN_EINVAL;
    hipError_t e;
    if (pattern == 0) e = launch_kernel(lds_rate_kernel<0>, dim3(ATTN_LDS_RATE_BLOCKS), dim3(256), 0, stream, out, iters);
    else if (pattern == 1) e = launch_kernel(lds_rate_kernel<1>, dim3(ATTN_LDS_RATE_BLOCKS), dim3(256), 0, stream, out, iters);
    else return ATTN_EUNSUPPORTED;
    if (e != hipSuccess) return ATTN_ELAUNCH;
    return (long long)ATTN_LDS_RATE_BLOCKS * 4 * iters * 8 * (pattern == 0 ? 1024 : 512);
}

long long attn_mfma_rate(float* out, int random_operands, int iters, void* stream)
{
    using namespace attn;
    if (!out || iters <= 0) return ATTN_EINVAL;
    if (launch_kernel(mfma_rate_kernel, dim3(ATTN_MFMA_RATE_BLOCKS), dim3(512), 0, stream, out, iters,
                      random_operands) != hipSuccess)
        return ATTN_ELAUNCH;
    return (long long)ATTN_MFMA_RATE_BLOCKS * 8 * iters * 32 * (2LL * 32 * 32 * 16);
}

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

long long attn_exp2_rate(float* out, int degree, int iters, void* stream)
{
    using namespace attn;
    if (!out || iters <= 0) return ATTN_EINVAL;
    const dim3 grid(ATTN_EXP2_RATE_BLOCKS), block(256);
    hipError_t e;
    switch (degree) {
        case 0: e = launch_kernel(exp2_rate_kernel<0>, grid, block, 0, stream, out, iters); break;
        case 3: e = launch_kernel(exp2_rate_kernel<3>, grid, block, 0, stream, out, iters); break;
        case 4: e = launch_kernel(exp2_rate_kernel<4>, grid, block, 0, stream, out, iters); break;
        case 5: e = launch_kernel(exp2_rate_kernel<5>, grid, block, 0, stream, out, iters); break;
        default: return ATTN_EUNSUPPORTED;
    }
    if (e != hipSuccess) return ATTN_ELAUNCH;
    return (long long)ATTN_EXP2_RATE_BLOCKS * 256 * 8 * iters;
}

long long attn_exp2_rate_partial(float* out, int emulated_of_8, int iters, void* stream)
{
    using namespace attn;
    if (!out || iters <= 0) return ATTN_EINVAL;
    const dim3 grid(ATTN_EXP2_RATE_BLOCKS), block(256);
    hipError_t e;
    switch (emulated_of_8) {
        case 0: e = launch_kernel(exp2_rate_partial_kernel<0>, grid, block, 0, stream, out, iters); break;
        case 1: e = launch_kernel(exp2_rate_partial_kernel<1>, grid, block, 0, stream, out, iters); break;
        case 2: e = launch_kernel(exp2_rate_partial_kernel<2>, grid, block, 0, stream, out, iters); break;
        case 4: e = launch_kernel(exp2_rate_partial_kernel<4>, grid, block, 0, stream, out, iters); break;
        case 8: e = launch_kernel(exp2_rate_partial_kernel<8>, grid, block, 0, stream, out, iters); break;
        default: return ATTN_EUNSUPPORTED;
    }
    if (e != hipSuccess) return ATTN_ELAUNCH;
    return (long long)ATTN_EXP2_RATE_BLOCKS * 256 * 8 * iters;
}

}  // extern "C"
