// Host-side argument bundles handed from the C ABI to the kernel launchers.
#pragma once
#include <stddef.h>

namespace attn {

struct FwdArgs {
    const void *q, *k, *v;
    void* o;
    float* lse;
    int B, H, Hkv, N, d_qk, d_v;
    float scale;
    int causal;
    void* stream;
};

struct BwdArgs {
    const void *q, *k, *v, *o, *d_o;
    const float* lse;
    void *dq, *dk, *dv;
    int B, H, Hkv, N, d_qk, d_v;
    float scale;
    int causal;
    // workspace carved up by the API: fp32 dQ accumulator, D = rowsum(dO o O), base-2 LSE
    float* dq_acc;
    float* D;
    float* lse2;
    void* stream;
};

// 0 on success, -2 unsupported head dims, -3 launch failure.
int launch_fwd(const FwdArgs& a);
int launch_bwd(const BwdArgs& a);

}  // namespace attn
