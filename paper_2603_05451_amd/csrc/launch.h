// Host-side argument bundles handed from the C ABI to the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdlib.h>
#include <tuple>

namespace attn {

// Element strides of one tensor in the variable-length kernels: the address of (token t, head h) of
// sequence s is  base + t * row + s * batch + h * head  (+ the position inside the head dim), t
// being the token's index in the packed batch.  Packed tensors have batch = 0; a [B, N, ...]
// tensor whose batch stride is not N rows passes batch = (batch stride) - N * row.
struct Stride3 {
    long long batch, row, head;
};
struct VarlenStrides {
    Stride3 q, k, v, o, d_o, dq, dk, dv;
    long long lse_batch, lse_head;      // lse index = t + s * lse_batch + h * lse_head
};

// Mark of a used entry of the tile tables.  Not 1: a workspace that was never planned, or whose
// tables were overwritten, then holds no entry that a kernel would act on.
constexpr int kPlanUsed = 0x5A17AB1E;

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
    VarlenStrides st = {};   // variable-length mode: q, k, v, o and lse strides
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
    VarlenStrides st = {};        // variable-length mode: strides of every tensor and of lse
    int rows_per_batch = 0;       // variable-length mode, prepare kernel: tokens per sequence when the
                                  // tensors have a batch stride (equal lengths), 0 for packed tensors
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
// The 64-queries-per-wave forward kernel (head dims 128, 64 or (192, 128); fixed length, N % 256 = 0).
int launch_fwd_q64(const FwdArgs& a);
// The dQ kernel with 64 queries per wave (d_qk = d_v = 128 or 64, fixed length, N % 256 = 0); it also
// leaves -D and the base-2 LSE of every row in the workspace.
int launch_bwd_dq_q64(const BwdArgs& a);
// The dK/dV kernel with one wave per SIMD and 32-query tiles (head dims 128, (192, 128): N % 128 = 0; 64:
// N % 256 = 0; fixed length, with or without the causal mask); -D and the base-2 LSE must be in the workspace.
int launch_bwd_dkdv_t32(const BwdArgs& a);
// The dQ kernel with one wave per SIMD and 32 queries per wave (head dims 128 and (192, 128), fixed length,
// N % 128 = 0); it also leaves -D and the base-2 LSE of every row in the workspace.
int launch_bwd_dq_t32(const BwdArgs& a);
// cu[b] = b * N for b = 0 .. B (device): the equal-length batch as a packed one.
int launch_uniform_cu(int* cu, int B, int N, void* stream);
// Fills the two plan tables of the variable-length entry points on the device: 0 or -3.
int launch_varlen_plan(const int* cu_q, const int* cu_k, int B, int Tq, int Tk, void* plan_q, int max_tiles_q,
                       void* plan_k, int max_tiles_k, void* stream);

}  // namespace attn
