// C ABI of the attention library: argument validation, workspace carving, dispatch.
// See include/attn.h for the contract of every entry point.
#include "../../include/attn.h"
#include "launch.h"

#include <stdint.h>

namespace {

bool dims_supported(int d_qk, int d_v)
{
    return (d_qk == 64 && d_v == 64) || (d_qk == 96 && d_v == 96) || (d_qk == 128 && d_v == 128) ||
           (d_qk == 192 && d_v == 128) || (d_qk == 256 && d_v == 256);
}

bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int check_sizes(int B, int H, int Hkv, int N, int d_qk, int d_v)
{
    if (B <= 0 || H <= 0 || Hkv <= 0 || N <= 0 || d_qk <= 0 || d_v <= 0) return ATTN_EINVAL;
    if (H % Hkv != 0) return ATTN_EINVAL;
    if (!dims_supported(d_qk, d_v)) return ATTN_EUNSUPPORTED;
    if (N % 128 != 0) return ATTN_EUNSUPPORTED;
    // element offsets are 64-bit, but the grid index B*H*(N/128) and the byte offsets inside
    // one 128-row tile (row stride H * d * 2 bytes) are 32-bit
    if ((int64_t)B * H * (N / 128) > 0x7fffffffLL) return ATTN_EUNSUPPORTED;
    if ((int64_t)H * (d_qk > d_v ? d_qk : d_v) * 2 * 128 > 0x7fffffffLL) return ATTN_EUNSUPPORTED;
    return ATTN_OK;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct WorkspaceLayout {
    size_t d_off, lse2_off, total;
};

WorkspaceLayout workspace_layout(int B, int H, int N)
{
    WorkspaceLayout w;
    const size_t rows = (size_t)B * H * N;
    w.d_off = 0;
    w.lse2_off = w.d_off + align_up(rows * sizeof(float), 256);
    w.total = w.lse2_off + align_up(rows * sizeof(float), 256);
    return w;
}

}  // namespace

extern "C" {

int attn_fwd_dtype(int dtype, const void* q, const void* k, const void* v, void* o, float* lse,
                   int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                   void* stream)
{
    if (dtype != ATTN_BF16 && dtype != ATTN_F16) return ATTN_EUNSUPPORTED;
    if (!q || !k || !v || !o || !lse) return ATTN_EINVAL;
    if (int rc = check_sizes(B, H, Hkv, N, d_qk, d_v)) return rc;
    if (!(scale > 0.0f) || !(scale < 1e30f)) return ATTN_EINVAL;
    if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(o, 16) ||
        misaligned(lse, 4))
        return ATTN_EINVAL;
    attn::FwdArgs a{q, k, v, o, lse, B, H, Hkv, N, d_qk, d_v, scale, causal != 0, stream};
    a.f16 = dtype == ATTN_F16;
    const int rc = attn::launch_fwd(a);
    return rc == 0 ? ATTN_OK : (rc == -2 ? ATTN_EUNSUPPORTED : ATTN_ELAUNCH);
}

int attn_fwd_ex(const void* q, const void* k, const void* v, void* o, float* lse,
                int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                void* stream)
{
    return attn_fwd_dtype(ATTN_BF16, q, k, v, o, lse, B, H, Hkv, N, d_qk, d_v, scale, causal, stream);
}

int attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
             int B, int H, int Hkv, int N, int d, float scale, int causal, void* stream)
{
    return attn_fwd_ex(q, k, v, o, lse, B, H, Hkv, N, d, d, scale, causal, stream);
}

size_t attn_bwd_workspace_bytes(int B, int H, int Hkv, int N, int d_qk, int d_v)
{
    if (check_sizes(B, H, Hkv, N, d_qk, d_v) != ATTN_OK) return 0;
    return workspace_layout(B, H, N).total;
}

static int bwd_impl(int dtype, const void* q, const void* k, const void* v, const void* o, const void* d_o,
                    const float* lse, void* dq, void* dk, void* dv,
                    int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                    void* workspace, size_t workspace_bytes, void* stream, int phases)
{
    if (dtype != ATTN_BF16 && dtype != ATTN_F16) return ATTN_EUNSUPPORTED;
    if (phases <= 0 || phases > ATTN_BWD_ALL) return ATTN_EINVAL;
    if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv || !workspace) return ATTN_EINVAL;
    if (int rc = check_sizes(B, H, Hkv, N, d_qk, d_v)) return rc;
    if (!(scale > 0.0f) || !(scale < 1e30f)) return ATTN_EINVAL;
    const void* ptrs[] = {q, k, v, o, d_o, dq, dk, dv};
    for (const void* p : ptrs)
        if (misaligned(p, 16)) return ATTN_EINVAL;
    if (misaligned(lse, 4) || misaligned(workspace, 256)) return ATTN_EINVAL;
    const WorkspaceLayout w = workspace_layout(B, H, N);
    if (workspace_bytes < w.total) return ATTN_EINVAL;
    char* ws = static_cast<char*>(workspace);
    attn::BwdArgs a{q, k, v, o, d_o, lse, dq, dk, dv, B, H, Hkv, N, d_qk, d_v, scale, causal != 0,
                    reinterpret_cast<float*>(ws + w.d_off),
                    reinterpret_cast<float*>(ws + w.lse2_off), stream, phases};
    a.f16 = dtype == ATTN_F16;
    const int rc = attn::launch_bwd(a);
    return rc == 0 ? ATTN_OK : (rc == -2 ? ATTN_EUNSUPPORTED : ATTN_ELAUNCH);
}

int attn_bwd_phases(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                    const float* lse, void* dq, void* dk, void* dv,
                    int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                    void* workspace, size_t workspace_bytes, void* stream, int phases)
{
    return bwd_impl(ATTN_BF16, q, k, v, o, d_o, lse, dq, dk, dv, B, H, Hkv, N, d_qk, d_v, scale, causal,
                    workspace, workspace_bytes, stream, phases);
}

int attn_bwd_dtype(int dtype, const void* q, const void* k, const void* v, const void* o, const void* d_o,
                   const float* lse, void* dq, void* dk, void* dv,
                   int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    return bwd_impl(dtype, q, k, v, o, d_o, lse, dq, dk, dv, B, H, Hkv, N, d_qk, d_v, scale, causal,
                    workspace, workspace_bytes, stream, ATTN_BWD_ALL);
}

int attn_bwd_ex(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                const float* lse, void* dq, void* dk, void* dv,
                int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                void* workspace, size_t workspace_bytes, void* stream)
{
    return attn_bwd_phases(q, k, v, o, d_o, lse, dq, dk, dv, B, H, Hkv, N, d_qk, d_v, scale, causal,
                           workspace, workspace_bytes, stream, ATTN_BWD_ALL);
}

int attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* d_o,
             const float* lse, void* dq, void* dk, void* dv,
             int B, int H, int Hkv, int N, int d, float scale, int causal,
             void* workspace, size_t workspace_bytes, void* stream)
{
    return attn_bwd_ex(q, k, v, o, d_o, lse, dq, dk, dv, B, H, Hkv, N, d, d, scale, causal,
                       workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// backward pass without an allocation by anyone: the workspace lives in the library's device image

namespace {

// -D and the base-2 LSE of up to ATTN_NOALLOC_MAX_ROWS rows (B * H * N), laid out as
// workspace_layout() lays out a caller's workspace of that many rows.  Every GPU the library runs
// on holds its own copy, at its own address, until the process ends.
constexpr size_t kScratchBytes = 2 * (size_t)ATTN_NOALLOC_MAX_ROWS * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Device address of `scratch` on the current device (the array's name in host code is only a handle
// for the runtime, not an address a kernel could use).  Looked up once per device; two host threads
// racing here both store the same value.
void* scratch_of_current_device(int* rc)
{
    static void* addr[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { *rc = ATTN_ELAUNCH; return nullptr; }
    if (!addr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { *rc = ATTN_ELAUNCH; return nullptr; }
        addr[dev] = p;
    }
    *rc = ATTN_OK;
    return addr[dev];
}

}  // namespace

int attn_bwd_noalloc(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                     const float* lse, void* dq, void* dk, void* dv,
                     int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                     void* stream)
{
    if (int rc = check_sizes(B, H, Hkv, N, d_qk, d_v)) return rc;
    if ((size_t)B * H * N > (size_t)ATTN_NOALLOC_MAX_ROWS) return ATTN_ETOOLARGE;
    int rc = ATTN_OK;
    void* ws = scratch_of_current_device(&rc);
    if (!ws) return rc;
    return bwd_impl(ATTN_BF16, q, k, v, o, d_o, lse, dq, dk, dv, B, H, Hkv, N, d_qk, d_v, scale, causal,
                    ws, kScratchBytes, stream, ATTN_BWD_ALL);
}

// ---------------------------------------------------------------------------------------------
// variable-length entry points

namespace {

int check_varlen(int B, int Tq, int Tk, int H, int Hkv, int d_qk, int d_v)
{
    if (B <= 0 || Tq <= 0 || Tk <= 0 || H <= 0 || Hkv <= 0) return ATTN_EINVAL;
    if (H % Hkv != 0) return ATTN_EINVAL;
    if (!dims_supported(d_qk, d_v)) return ATTN_EUNSUPPORTED;
    if (((int64_t)Tq / 128 + B) * H > 0x7fffffffLL) return ATTN_EUNSUPPORTED;
    if (((int64_t)Tk / 128 + B) * Hkv > 0x7fffffffLL) return ATTN_EUNSUPPORTED;
    if ((int64_t)H * (d_qk > d_v ? d_qk : d_v) * 2 * 128 > 0x7fffffffLL) return ATTN_EUNSUPPORTED;
    return ATTN_OK;
}

// Workspace of the variable-length calls: table of query tiles | table of key tiles | -D | LSE2
// (forward: the first table only).  A table entry is 32 bytes.
struct VarlenLayout {
    int max_tiles_q, max_tiles_k;
    size_t plan_q_off, plan_k_off, d_off, lse2_off, total_fwd, total_bwd;
};

VarlenLayout varlen_layout(int B, int Tq, int Tk, int H)
{
    VarlenLayout w;
    w.max_tiles_q = Tq / 128 + B;       // sum over sequences of ceil(len / 128) never exceeds this
    w.max_tiles_k = Tk / 128 + B;
    w.plan_q_off = 0;
    w.total_fwd = align_up((size_t)w.max_tiles_q * 32, 256);
    w.plan_k_off = w.total_fwd;
    w.d_off = w.plan_k_off + align_up((size_t)w.max_tiles_k * 32, 256);
    w.lse2_off = w.d_off + align_up((size_t)H * Tq * sizeof(float), 256);
    w.total_bwd = w.lse2_off + align_up((size_t)H * Tq * sizeof(float), 256);
    return w;
}

// Strides of packed [T, heads, d] tensors and of lse [H, Tq].
attn::VarlenStrides packed_strides(int Tq, int H, int Hkv, int d_qk, int d_v)
{
    attn::VarlenStrides st;
    st.q = st.dq = {0, (long long)H * d_qk, d_qk};
    st.k = st.dk = {0, (long long)Hkv * d_qk, d_qk};
    st.v = st.dv = {0, (long long)Hkv * d_v, d_v};
    st.o = st.d_o = {0, (long long)H * d_v, d_v};
    st.lse_batch = 0;
    st.lse_head = Tq;
    return st;
}

int varlen_fwd_run(int dtype, const void* q, const void* k, const void* v, void* o, float* lse,
                   const int* cu_q, const int* cu_k, int B, int Tq, int Tk, int H, int Hkv, int d_qk, int d_v,
                   float scale, int causal, char* ws, const attn::VarlenStrides& st, void* stream)
{
    const VarlenLayout w = varlen_layout(B, Tq, Tk, H);
    if (cu_q && attn::launch_varlen_plan(cu_q, cu_k, B, Tq, Tk, ws + w.plan_q_off, w.max_tiles_q, nullptr, 0, stream) != 0)
        return ATTN_ELAUNCH;
    attn::FwdArgs a{q, k, v, o, lse, B, H, Hkv, 0, d_qk, d_v, scale, causal != 0, stream};
    a.plan = ws + w.plan_q_off;
    a.T = Tq;
    a.max_tiles = w.max_tiles_q;
    a.st = st;
    a.f16 = dtype == ATTN_F16;
    const int rc = attn::launch_fwd(a);
    return rc == 0 ? ATTN_OK : (rc == -2 ? ATTN_EUNSUPPORTED : ATTN_ELAUNCH);
}

int varlen_bwd_run(int dtype, const void* q, const void* k, const void* v, const void* o, const void* d_o,
                   const float* lse, void* dq, void* dk, void* dv,
                   const int* cu_q, const int* cu_k, int B, int Tq, int Tk, int H, int Hkv, int d_qk, int d_v,
                   float scale, int causal, char* ws, const attn::VarlenStrides& st, int rows_per_batch, void* stream)
{
    const VarlenLayout w = varlen_layout(B, Tq, Tk, H);
    if (cu_q && attn::launch_varlen_plan(cu_q, cu_k, B, Tq, Tk, ws + w.plan_q_off, w.max_tiles_q,
                                         ws + w.plan_k_off, w.max_tiles_k, stream) != 0)
        return ATTN_ELAUNCH;
    attn::BwdArgs a{q, k, v, o, d_o, lse, dq, dk, dv, B, H, Hkv, 0, d_qk, d_v, scale, causal != 0,
                    reinterpret_cast<float*>(ws + w.d_off), reinterpret_cast<float*>(ws + w.lse2_off),
                    stream, ATTN_BWD_ALL};
    a.plan = ws + w.plan_q_off;
    a.T = Tq;
    a.max_tiles = w.max_tiles_q;
    a.plan_k = ws + w.plan_k_off;
    a.max_tiles_k = w.max_tiles_k;
    a.st = st;
    a.rows_per_batch = rows_per_batch;
    a.f16 = dtype == ATTN_F16;
    const int rc = attn::launch_bwd(a);
    return rc == 0 ? ATTN_OK : (rc == -2 ? ATTN_EUNSUPPORTED : ATTN_ELAUNCH);
}

}  // namespace

size_t attn_varlen_workspace_bytes(int B, int total_q, int total_k, int H, int Hkv, int d_qk, int d_v, int backward)
{
    if (check_varlen(B, total_q, total_k, H, Hkv, d_qk, d_v) != ATTN_OK) return 0;
    const VarlenLayout w = varlen_layout(B, total_q, total_k, H);
    return backward ? w.total_bwd : w.total_fwd;
}

int attn_varlen_plan(const int* cu_seqlens_q, const int* cu_seqlens_k, int B, int total_q, int total_k,
                     int H, int Hkv, int d_qk, int d_v, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!cu_seqlens_q || !cu_seqlens_k || !workspace) return ATTN_EINVAL;
    if (int rc = check_varlen(B, total_q, total_k, H, Hkv, d_qk, d_v)) return rc;
    if (misaligned(cu_seqlens_q, 4) || misaligned(cu_seqlens_k, 4) || misaligned(workspace, 256)) return ATTN_EINVAL;
    const VarlenLayout w = varlen_layout(B, total_q, total_k, H);
    if (workspace_bytes < w.total_bwd) return ATTN_EINVAL;
    char* ws = static_cast<char*>(workspace);
    return attn::launch_varlen_plan(cu_seqlens_q, cu_seqlens_k, B, total_q, total_k, ws + w.plan_q_off, w.max_tiles_q,
                                    ws + w.plan_k_off, w.max_tiles_k, stream) == 0 ? ATTN_OK : ATTN_ELAUNCH;
}

int attn_varlen_fwd_dtype(int dtype, const void* q, const void* k, const void* v, void* o, float* lse,
                          const int* cu_seqlens_q, const int* cu_seqlens_k, int B, int total_q, int total_k,
                          int H, int Hkv, int d_qk, int d_v,
                          float scale, int causal, void* workspace, size_t workspace_bytes, void* stream)
{
    if (dtype != ATTN_BF16 && dtype != ATTN_F16) return ATTN_EUNSUPPORTED;
    if (!q || !k || !v || !o || !lse || !workspace) return ATTN_EINVAL;
    if ((cu_seqlens_q == nullptr) != (cu_seqlens_k == nullptr)) return ATTN_EINVAL;   // both null: tables kept
    if (int rc = check_varlen(B, total_q, total_k, H, Hkv, d_qk, d_v)) return rc;
    if (!(scale > 0.0f) || !(scale < 1e30f)) return ATTN_EINVAL;
    if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(o, 16) ||
        misaligned(lse, 4) || misaligned(cu_seqlens_q, 4) || misaligned(cu_seqlens_k, 4) || misaligned(workspace, 256))
        return ATTN_EINVAL;
    if (workspace_bytes < varlen_layout(B, total_q, total_k, H).total_fwd) return ATTN_EINVAL;
    return varlen_fwd_run(dtype, q, k, v, o, lse, cu_seqlens_q, cu_seqlens_k, B, total_q, total_k, H, Hkv, d_qk, d_v,
                          scale, causal, static_cast<char*>(workspace), packed_strides(total_q, H, Hkv, d_qk, d_v),
                          stream);
}

int attn_varlen_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                    const int* cu_seqlens_q, const int* cu_seqlens_k, int B, int total_q, int total_k,
                    int H, int Hkv, int d_qk, int d_v,
                    float scale, int causal, void* workspace, size_t workspace_bytes, void* stream)
{
    return attn_varlen_fwd_dtype(ATTN_BF16, q, k, v, o, lse, cu_seqlens_q, cu_seqlens_k, B, total_q, total_k,
                                 H, Hkv, d_qk, d_v, scale, causal, workspace, workspace_bytes, stream);
}

int attn_varlen_bwd_dtype(int dtype, const void* q, const void* k, const void* v, const void* o, const void* d_o,
                          const float* lse, void* dq, void* dk, void* dv,
                          const int* cu_seqlens_q, const int* cu_seqlens_k, int B, int total_q, int total_k,
                          int H, int Hkv, int d_qk, int d_v,
                          float scale, int causal, void* workspace, size_t workspace_bytes, void* stream)
{
    if (dtype != ATTN_BF16 && dtype != ATTN_F16) return ATTN_EUNSUPPORTED;
    if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv || !workspace) return ATTN_EINVAL;
    if ((cu_seqlens_q == nullptr) != (cu_seqlens_k == nullptr)) return ATTN_EINVAL;   // both null: tables kept
    if (int rc = check_varlen(B, total_q, total_k, H, Hkv, d_qk, d_v)) return rc;
    if (!(scale > 0.0f) || !(scale < 1e30f)) return ATTN_EINVAL;
    const void* ptrs[] = {q, k, v, o, d_o, dq, dk, dv};
    for (const void* p : ptrs)
        if (misaligned(p, 16)) return ATTN_EINVAL;
    if (misaligned(lse, 4) || misaligned(cu_seqlens_q, 4) || misaligned(cu_seqlens_k, 4) || misaligned(workspace, 256))
        return ATTN_EINVAL;
    if (workspace_bytes < varlen_layout(B, total_q, total_k, H).total_bwd) return ATTN_EINVAL;
    return varlen_bwd_run(dtype, q, k, v, o, d_o, lse, dq, dk, dv, cu_seqlens_q, cu_seqlens_k, B, total_q, total_k,
                          H, Hkv, d_qk, d_v, scale, causal, static_cast<char*>(workspace),
                          packed_strides(total_q, H, Hkv, d_qk, d_v), 0, stream);
}

int attn_varlen_bwd(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                    const float* lse, void* dq, void* dk, void* dv,
                    const int* cu_seqlens_q, const int* cu_seqlens_k, int B, int total_q, int total_k,
                    int H, int Hkv, int d_qk, int d_v,
                    float scale, int causal, void* workspace, size_t workspace_bytes, void* stream)
{
    return attn_varlen_bwd_dtype(ATTN_BF16, q, k, v, o, d_o, lse, dq, dk, dv, cu_seqlens_q, cu_seqlens_k, B,
                                 total_q, total_k, H, Hkv, d_qk, d_v, scale, causal, workspace, workspace_bytes,
                                 stream);
}

// ---------------------------------------------------------------------------------------------
// strided entry points: equal-length batches (Nq queries and Nk keys per sequence) in any layout
// whose head dim is contiguous, run by the variable-length kernels on generated boundaries
// cu_seqlens_q = {0, Nq, 2 Nq, ...}, cu_seqlens_k = {0, Nk, 2 Nk, ...}

namespace {

size_t cu_bytes(int B) { return align_up((size_t)(B + 1) * sizeof(int), 256); }

int check_strided(int B, int H, int Hkv, int Nq, int Nk, int d_qk, int d_v)
{
    if (B <= 0 || Nq <= 0 || Nk <= 0) return ATTN_EINVAL;
    if ((int64_t)B * Nq > 0x7fffffffLL || (int64_t)B * Nk > 0x7fffffffLL) return ATTN_EUNSUPPORTED;
    return check_varlen(B, B * Nq, B * Nk, H, Hkv, d_qk, d_v);
}

// every stride a multiple of 8 elements (16 bytes: vector loads and the global->LDS copies),
// rows and heads apart (stride 0 only where there is a single one)
bool bad_stride(const attn_strides_t* s, int B, int N, int heads)
{
    if (!s) return true;
    if (s->batch % 8 || s->row % 8 || s->head % 8) return true;
    if (s->batch < 0 || s->row < 0 || s->head < 0) return true;
    if ((B > 1 && s->batch == 0) || (N > 1 && s->row == 0) || (heads > 1 && s->head == 0)) return true;
    if (s->row > (1LL << 23)) return true;     // byte offsets inside a 128-row tile are 32-bit
    return false;
}

attn::Stride3 as_packed(const attn_strides_t* s, int N)
{
    return {s->batch - (long long)N * s->row, s->row, s->head};
}

}  // namespace

size_t attn_strided_workspace_bytes(int B, int H, int Hkv, int Nq, int Nk, int d_qk, int d_v, int backward)
{
    if (check_strided(B, H, Hkv, Nq, Nk, d_qk, d_v) != ATTN_OK) return 0;
    const VarlenLayout w = varlen_layout(B, B * Nq, B * Nk, H);
    return 2 * cu_bytes(B) + (backward ? w.total_bwd : w.total_fwd);
}

int attn_fwd_strided(int dtype, const void* q, const attn_strides_t* sq, const void* k, const attn_strides_t* sk,
                     const void* v, const attn_strides_t* sv, void* o, const attn_strides_t* so, float* lse,
                     int B, int H, int Hkv, int Nq, int Nk, int d_qk, int d_v, float scale, int causal,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (dtype != ATTN_BF16 && dtype != ATTN_F16) return ATTN_EUNSUPPORTED;
    if (!q || !k || !v || !o || !lse || !workspace) return ATTN_EINVAL;
    if (int rc = check_strided(B, H, Hkv, Nq, Nk, d_qk, d_v)) return rc;
    if (causal && Nk < Nq) return ATTN_EINVAL;             // some query would see no key
    if (bad_stride(sq, B, Nq, H) || bad_stride(sk, B, Nk, Hkv) || bad_stride(sv, B, Nk, Hkv) || bad_stride(so, B, Nq, H))
        return ATTN_EINVAL;
    if (!(scale > 0.0f) || !(scale < 1e30f)) return ATTN_EINVAL;
    if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(o, 16) ||
        misaligned(lse, 4) || misaligned(workspace, 256))
        return ATTN_EINVAL;
    if (workspace_bytes < attn_strided_workspace_bytes(B, H, Hkv, Nq, Nk, d_qk, d_v, 0)) return ATTN_EINVAL;
    char* ws = static_cast<char*>(workspace);
    int* cu_q = reinterpret_cast<int*>(ws);
    int* cu_k = reinterpret_cast<int*>(ws + cu_bytes(B));
    if (attn::launch_uniform_cu(cu_q, B, Nq, stream) != 0 || attn::launch_uniform_cu(cu_k, B, Nk, stream) != 0)
        return ATTN_ELAUNCH;
    attn::VarlenStrides st = {};
    st.q = as_packed(sq, Nq);
    st.k = as_packed(sk, Nk);
    st.v = as_packed(sv, Nk);
    st.o = as_packed(so, Nq);
    st.lse_head = Nq;                      // lse [B, H, Nq]
    st.lse_batch = (long long)(H - 1) * Nq;
    return varlen_fwd_run(dtype, q, k, v, o, lse, cu_q, cu_k, B, B * Nq, B * Nk, H, Hkv, d_qk, d_v, scale, causal,
                          ws + 2 * cu_bytes(B), st, stream);
}

int attn_bwd_strided(int dtype, const void* q, const attn_strides_t* sq, const void* k, const attn_strides_t* sk,
                     const void* v, const attn_strides_t* sv, const void* o, const attn_strides_t* so,
                     const void* d_o, const attn_strides_t* sdo, const float* lse,
                     void* dq, const attn_strides_t* sdq, void* dk, const attn_strides_t* sdk,
                     void* dv, const attn_strides_t* sdv,
                     int B, int H, int Hkv, int Nq, int Nk, int d_qk, int d_v, float scale, int causal,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (dtype != ATTN_BF16 && dtype != ATTN_F16) return ATTN_EUNSUPPORTED;
    if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv || !workspace) return ATTN_EINVAL;
    if (int rc = check_strided(B, H, Hkv, Nq, Nk, d_qk, d_v)) return rc;
    if (causal && Nk < Nq) return ATTN_EINVAL;
    if (bad_stride(sq, B, Nq, H) || bad_stride(sk, B, Nk, Hkv) || bad_stride(sv, B, Nk, Hkv) || bad_stride(so, B, Nq, H) ||
        bad_stride(sdo, B, Nq, H) || bad_stride(sdq, B, Nq, H) || bad_stride(sdk, B, Nk, Hkv) || bad_stride(sdv, B, Nk, Hkv))
        return ATTN_EINVAL;
    if (!(scale > 0.0f) || !(scale < 1e30f)) return ATTN_EINVAL;
    const void* ptrs[] = {q, k, v, o, d_o, dq, dk, dv};
    for (const void* p : ptrs)
        if (misaligned(p, 16)) return ATTN_EINVAL;
    if (misaligned(lse, 4) || misaligned(workspace, 256)) return ATTN_EINVAL;
    if (workspace_bytes < attn_strided_workspace_bytes(B, H, Hkv, Nq, Nk, d_qk, d_v, 1)) return ATTN_EINVAL;
    char* ws = static_cast<char*>(workspace);
    int* cu_q = reinterpret_cast<int*>(ws);
    int* cu_k = reinterpret_cast<int*>(ws + cu_bytes(B));
    if (attn::launch_uniform_cu(cu_q, B, Nq, stream) != 0 || attn::launch_uniform_cu(cu_k, B, Nk, stream) != 0)
        return ATTN_ELAUNCH;
    attn::VarlenStrides st = {};
    st.q = as_packed(sq, Nq);
    st.k = as_packed(sk, Nk);
    st.v = as_packed(sv, Nk);
    st.o = as_packed(so, Nq);
    st.d_o = as_packed(sdo, Nq);
    st.dq = as_packed(sdq, Nq);
    st.dk = as_packed(sdk, Nk);
    st.dv = as_packed(sdv, Nk);
    st.lse_head = Nq;
    st.lse_batch = (long long)(H - 1) * Nq;
    return varlen_bwd_run(dtype, q, k, v, o, d_o, lse, dq, dk, dv, cu_q, cu_k, B, B * Nq, B * Nk, H, Hkv, d_qk, d_v,
                          scale, causal, ws + 2 * cu_bytes(B), st, Nq, stream);
}

const char* attn_strerror(int code)
{
    switch (code) {
        case ATTN_OK: return "success";
        case ATTN_EINVAL: return "invalid argument (null or misaligned pointer, bad size, H % Hkv != 0, "
                                 "non-positive scale, or workspace too small)";
        case ATTN_EUNSUPPORTED: return "unsupported shape: (d_qk, d_v) must be (64,64), (96,96), (128,128), "
                                       "(192,128) or (256,256) and N a multiple of 128";
        case ATTN_ELAUNCH: return "HIP kernel launch failed";
        case ATTN_ETOOLARGE: return "B * H * N exceeds ATTN_NOALLOC_MAX_ROWS, the size of the built-in workspace of "
                                    "attn_bwd_noalloc: use attn_bwd_ex with a workspace of your own";
        default: return "unknown error code";
    }
}

int attn_version(void) { return 100; }

}  // extern "C"
