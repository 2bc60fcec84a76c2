// Host-side argument bundles handed from the C ABI to the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <tuple>

namespace attn {

struct FwdArgs {
    const void *q, *k, *v;
    void* o;
    float* lse;
    int B, H, Hkv, N, d_qk, d_v;
    float scale;
    int causal;
    void* stream;
    // variable-length mode (plan != nullptr): B and N unused; plan = table of query tiles,
    // max_tiles its size (an upper bound on the number of 128-row query tiles), T = total query rows
    const void* plan = nullptr;
    int T = 0, max_tiles = 0;
    bool f16 = false;   // 16-bit storage type of q, k, v, o: bf16 (default) or IEEE fp16
};

struct BwdArgs {
    const void *q, *k, *v, *o, *d_o;
    const float* lse;
    void *dq, *dk, *dv;
    int B, H, Hkv, N, d_qk, d_v;
    float scale;
    int causal;
    // workspace carved up by the API: -D = -rowsum(dO o O) and the base-2 LSE
    float* D;
    float* lse2;
    void* stream;
    int phases;   // bit mask: 1 prepare, 2 dK/dV kernel, 4 dQ kernel
    const void* plan = nullptr;   // variable-length mode, as in FwdArgs: query-tile table (dQ kernel)
    int T = 0, max_tiles = 0;
    const void* plan_k = nullptr; // key-tile table (dK/dV kernels) and its size
    int max_tiles_k = 0;
    bool f16 = false;             // as in FwdArgs
};

// Launch through hipLaunchKernel so that the status returned belongs to THIS launch (the
// sticky hipGetLastError slot may hold an unrelated earlier error of the host program).
template <typename... KArgs, typename... Args>
inline hipError_t launch_kernel(void (*kern)(KArgs...), dim3 grid, dim3 block, size_t smem, void* stream,
                                Args... args)
{
    std::tuple<KArgs...> vals{static_cast<KArgs>(args)...};
    void* ptrs[sizeof...(KArgs)];
    int n = 0;
    std::apply([&](auto&... v) { ((ptrs[n++] = (void*)&v), ...); }, vals);
    return hipLaunchKernel((const void*)kern, grid, block, ptrs, smem, (hipStream_t)stream);
}

// Raises a kernel's dynamic-LDS limit to `smem` bytes on the current device.  The attribute
// belongs to the (kernel, device) pair, so the "already done" note is kept per device; a race
// between two host threads only repeats the idempotent call.
struct LdsOptIn {
    bool done[64] = {};
    template <typename K>
    bool allow(K kern, int smem)
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return false;
        if (dev >= 0 && dev < 64 && done[dev]) return true;
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return false;
        if (dev >= 0 && dev < 64) done[dev] = true;
        return true;
    }
};

// 0 on success, -2 unsupported head dims, -3 launch failure.
int launch_fwd(const FwdArgs& a);
int launch_bwd(const BwdArgs& a);
// Fills the two plan tables of the variable-length entry points on the device: 0 or -3.
int launch_varlen_plan(const int* cu_q, const int* cu_k, int B, void* plan_q, int max_tiles_q,
                       void* plan_k, int max_tiles_k, void* stream);

}  // namespace attn
