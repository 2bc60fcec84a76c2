// Measurement probes (gfx950): rates of the machine's units in the patterns the attention kernels use.
// They are not part of the attention library: this file is built into libattn_probes.so, declared in
// include/attn_probes.h, and only tests and profiles call it.
#include "../../include/attn_probes.h"
#include "common.h"
#include "exp2_emulation.h"
#include "launch.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attn {

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


// Issue cost, inside ONE wave per SIMD, of the instructions that accompany the MFMAs in the kernels
// that run one wave per SIMD: per step {1 MFMA, NV vector instructions (the first a v_exp_f32, the
// rest v_fma_f32), NB ds_read_b128 and NTR pairs of ds_read_b64_tr_b16 whose results feed the MFMA
// RING steps later}, one global->LDS copy instruction every DMA steps (0 = none).  256 blocks of 4
// waves, N(0,1)-like operands.  Thread 0 of block 0 writes the shader cycles and the 100 MHz
// constant-clock ticks the loop took to clk[0], clk[1].
template <int NV, int NB, int NTR, int DMA, int RING>
__global__ void __launch_bounds__(256, 1)
wave_issue_kernel(float* __restrict__ out, int iters, long long* __restrict__ clk)
{
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    extern __shared__ __attribute__((aligned(1024))) char wave_issue_smem[];
    ATTN_LDS char* smem = (ATTN_LDS char*)wave_issue_smem;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 32768; i += 256) ((ATTN_LDS __bf16*)smem)[i] = (__bf16)hash_gauss(i * 2654435761u);
    __syncthreads();
    bf16x8 a0, b0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a0[i] = (__bf16)hash_gauss(tid * 8 + i); b0[i] = (__bf16)hash_gauss(tid * 8 + i + 0x9e3779b9u); }
    f32x16 acc[4] = {{0}, {0}, {0}, {0}};
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = 0.5f + 0.01f * (tid + i);
    bf16x8 ra[RING], rb[RING];
#pragma unroll
    for (int r = 0; r < RING; ++r) { ra[r] = a0; rb[r] = b0; }
    const ATTN_LDS char* pa = smem + lane * 16;                                  // 16 bytes per lane, no bank conflict
    const ATTN_LDS char* pt = smem + (lane & 15) * 8 + (lane >> 4) * 256;
    const uint32_t goff = lane * 16;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(NB ? ra[j % RING] : a0, NTR ? rb[j % RING] : b0, acc[j & 3], 0, 0, 0);
            if (NB >= 1) ra[j % RING] = *(const ATTN_LDS bf16x8*)(pa + j * 1024);
            if (NB >= 2) { const bf16x8 t = *(const ATTN_LDS bf16x8*)(pa + 16384 + j * 1024); ra[j % RING][0] = t[0]; }
            if (NTR >= 1) {
                const s16x4 lo = lds_read_tr_bits(pt + j * 1024);
                const s16x4 hi = lds_read_tr_bits(pt + j * 1024 + 16384);
                rb[j % RING] = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                if (v == 0) asm volatile("v_exp_f32 %0, %0" : "+v"(x[v & 7]));
                else asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(x[v & 7]));
            }
            if (DMA > 0 && (j % DMA) == 0) dma16((const char*)out + goff, smem + 65536 + wave * 4096 + (j & 3) * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (DMA > 0) wait_async_copies();
        if ((it & 255) == 255) {   // keep the accumulators finite
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[m][r] *= 1e-6f;
        }
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    if (blockIdx.x == 0 && tid == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
    float t = 0.f;
#pragma unroll
    for (int m = 0; m < 4; ++m) t += acc[m][m];
#pragma unroll
    for (int i = 0; i < 8; ++i) t += x[i];
    if (t == 123.456f) out[blockIdx.x * 256 + tid] = t + (float)((ATTN_LDS __bf16*)smem)[32768 + tid];   // never true: keeps the work live
}

struct WaveIssueConfig {
    int nv, nb, ntr, dma, ring;
    hipError_t (*launch)(float*, int, long long*, void*);
};
template <int NV, int NB, int NTR, int DMA, int RING>
static hipError_t launch_wave_issue(float* out, int iters, long long* clk, void* stream)
{
    auto kern = wave_issue_kernel<NV, NB, NTR, DMA, RING>;
    static LdsOptIn lds;
    if (!lds.allow(kern, 96 * 1024)) return hipErrorInvalidValue;
    return launch_kernel(kern, dim3(ATTN_PROBE_WAVE_ISSUE_BLOCKS), dim3(256), 96 * 1024, stream, out, iters, clk);
}
#define WI(nv, nb, ntr, dma, ring) {nv, nb, ntr, dma, ring, launch_wave_issue<nv, nb, ntr, dma, ring>}
static const WaveIssueConfig kWaveIssueConfigs[] = {
    WI(0, 0, 0, 0, 4),
    WI(0, 1, 0, 0, 2), WI(0, 1, 0, 0, 4), WI(0, 1, 0, 0, 8), WI(0, 2, 0, 0, 4), WI(0, 2, 0, 0, 8),
    WI(0, 0, 1, 0, 2), WI(0, 0, 1, 0, 4), WI(0, 0, 1, 0, 8), WI(0, 1, 1, 0, 4), WI(0, 1, 1, 0, 8),
    WI(0, 0, 0, 1, 4), WI(0, 0, 0, 2, 4), WI(0, 0, 0, 4, 4), WI(0, 0, 0, 8, 4),
    WI(3, 0, 0, 0, 4), WI(3, 1, 0, 0, 4), WI(3, 0, 1, 0, 4), WI(3, 0, 1, 0, 8), WI(3, 0, 1, 4, 4),
    WI(5, 0, 1, 0, 4), WI(5, 1, 0, 4, 8),
};
#undef WI
}  // namespace attn

extern "C" {

long long attn_lds_rate(float* out, int pattern, int iters, void* stream)
{
    using namespace attn;
    if (!out || iters <= 0) return ATTN_PROBE_EINVAL;
    hipError_t e;
    if (pattern == 0) e = launch_kernel(lds_rate_kernel<0>, dim3(ATTN_LDS_RATE_BLOCKS), dim3(256), 0, stream, out, iters);
    else if (pattern == 1) e = launch_kernel(lds_rate_kernel<1>, dim3(ATTN_LDS_RATE_BLOCKS), dim3(256), 0, stream, out, iters);
    else return ATTN_PROBE_EUNSUPPORTED;
    if (e != hipSuccess) return ATTN_PROBE_ELAUNCH;
    return (long long)ATTN_LDS_RATE_BLOCKS * 4 * iters * 8 * (pattern == 0 ? 1024 : 512);
}

long long attn_mfma_rate(float* out, int random_operands, int iters, void* stream)
{
    using namespace attn;
    if (!out || iters <= 0) return ATTN_PROBE_EINVAL;
    if (launch_kernel(mfma_rate_kernel, dim3(ATTN_MFMA_RATE_BLOCKS), dim3(512), 0, stream, out, iters,
                      random_operands) != hipSuccess)
        return ATTN_PROBE_ELAUNCH;
    return (long long)ATTN_MFMA_RATE_BLOCKS * 8 * iters * 32 * (2LL * 32 * 32 * 16);
}

long long attn_exp2_rate(float* out, int degree, int iters, void* stream)
{
    using namespace attn;
    if (!out || iters <= 0) return ATTN_PROBE_EINVAL;
    const dim3 grid(ATTN_EXP2_RATE_BLOCKS), block(256);
    hipError_t e;
    switch (degree) {
        case 0: e = launch_kernel(exp2_rate_kernel<0>, grid, block, 0, stream, out, iters); break;
        case 3: e = launch_kernel(exp2_rate_kernel<3>, grid, block, 0, stream, out, iters); break;
        case 4: e = launch_kernel(exp2_rate_kernel<4>, grid, block, 0, stream, out, iters); break;
        case 5: e = launch_kernel(exp2_rate_kernel<5>, grid, block, 0, stream, out, iters); break;
        default: return ATTN_PROBE_EUNSUPPORTED;
    }
    if (e != hipSuccess) return ATTN_PROBE_ELAUNCH;
    return (long long)ATTN_EXP2_RATE_BLOCKS * 256 * 8 * iters;
}

long long attn_exp2_rate_partial(float* out, int emulated_of_8, int iters, void* stream)
{
    using namespace attn;
    if (!out || iters <= 0) return ATTN_PROBE_EINVAL;
    const dim3 grid(ATTN_EXP2_RATE_BLOCKS), block(256);
    hipError_t e;
    switch (emulated_of_8) {
        case 0: e = launch_kernel(exp2_rate_partial_kernel<0>, grid, block, 0, stream, out, iters); break;
        case 1: e = launch_kernel(exp2_rate_partial_kernel<1>, grid, block, 0, stream, out, iters); break;
        case 2: e = launch_kernel(exp2_rate_partial_kernel<2>, grid, block, 0, stream, out, iters); break;
        case 4: e = launch_kernel(exp2_rate_partial_kernel<4>, grid, block, 0, stream, out, iters); break;
        case 8: e = launch_kernel(exp2_rate_partial_kernel<8>, grid, block, 0, stream, out, iters); break;
        default: return ATTN_PROBE_EUNSUPPORTED;
    }
    if (e != hipSuccess) return ATTN_PROBE_ELAUNCH;
    return (long long)ATTN_EXP2_RATE_BLOCKS * 256 * 8 * iters;
}

int attn_probe_wave_issue_configs(void)
{
    return (int)(sizeof(attn::kWaveIssueConfigs) / sizeof(attn::kWaveIssueConfigs[0]));
}

long long attn_probe_wave_issue(int config, int* describe5, float* out, long long* clk, int iters, void* stream)
{
    using namespace attn;
    if (config < 0 || config >= attn_probe_wave_issue_configs()) return ATTN_PROBE_EUNSUPPORTED;
    const WaveIssueConfig& c = kWaveIssueConfigs[config];
    if (describe5) { describe5[0] = c.nv; describe5[1] = c.nb; describe5[2] = c.ntr; describe5[3] = c.dma; describe5[4] = c.ring; }
    if (!out || !clk || iters <= 0) return ATTN_PROBE_EINVAL;
    if (c.launch(out, iters, clk, stream) != hipSuccess) return ATTN_PROBE_ELAUNCH;
    return (long long)iters * 16;
}

}  // extern "C"
