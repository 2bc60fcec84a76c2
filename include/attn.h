/*
 * C ABI of the MI355X (gfx950) fused attention library: exact scaled-dot-product
 * attention, forward and backward, bf16 storage, fp32 accumulation.
 *
 * What is computed (paper Sec. 2.1):
 *   forward   S = scale * Q K^T (+ causal mask), P = softmax_rows(S), O = P V,
 *             LSE_i = ln sum_j exp(S_ij)   (natural log, of the scaled, masked scores)
 *   backward  dV = P^T dO, dP = dO V^T, dS = P o (dP - D), D_i = sum_c dO_ic O_ic,
 *             dQ = scale * dS K, dK = scale * dS^T Q
 * The N x N matrices S, P, dP, dS never reach device memory; the forward pass keeps
 * tiled online-softmax statistics with thresholded rescaling (paper Sec. 3.1.4) and the
 * backward pass recomputes P from Q, K and LSE (paper Sec. 3.2).
 *
 * Conventions shared by every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees or keeps it.  `stream` is a hipStream_t passed as void*
 *     (NULL = the default stream).  Calls only enqueue work on `stream` and return.
 *   - Layouts are contiguous row-major ("token-major"):
 *       q, o, d_o, dq : [B, N, H,   d]   bf16      (d = d_qk for q/dq, d_v for o/d_o)
 *       k, dk         : [B, N, Hkv, d_qk] bf16
 *       v, dv         : [B, N, Hkv, d_v]  bf16
 *       lse           : [B, H, N]         fp32
 *     bf16 = upper 16 bits of an IEEE fp32; outputs are rounded to nearest even.
 *     All pointers must be 16-byte aligned.
 *   - Grouped-query attention: H % Hkv == 0; query head h reads KV head h / (H / Hkv);
 *     dk and dv are summed over the query heads of each group.
 *   - causal != 0: key j is visible to query i iff j <= i.
 *   - Supported shapes: (d_qk, d_v) in {(64,64), (96,96), (128,128), (192,128), (256,256)}; N a positive
 *     multiple of 128 (the attn_varlen_* entry points take any lengths).
 *   - Return value: ATTN_OK, or a negative code.  ATTN_EINVAL, ATTN_EUNSUPPORTED and
 *     ATTN_ETOOLARGE are found before anything is enqueued: no output has been touched.
 *     ATTN_ELAUNCH (the HIP runtime refused a launch or an attribute) can come from any of the
 *     launches of a call that has several (the backward pass: dQ kernel, then dK/dV kernel; the
 *     variable-length and strided calls: a small table kernel first): the launches before the
 *     failed one stay enqueued and write their outputs (dq, the workspace); the outputs of the
 *     failed and later launches are untouched.
 *   - Re-entrant; no global state.  Calls on different streams may run concurrently
 *     as long as their outputs and workspaces do not overlap.
 */
#ifndef PAPER_2603_05451_AMD_ATTN_H
#define PAPER_2603_05451_AMD_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ATTN_OK = 0,
    ATTN_EINVAL = -1,       /* null pointer, non-positive size, H % Hkv != 0, misaligned pointer,
                               workspace too small */
    ATTN_EUNSUPPORTED = -2, /* head dims or N outside the supported set */
    ATTN_ELAUNCH = -3,      /* the HIP runtime refused a launch */
    ATTN_ETOOLARGE = -4     /* attn_bwd_noalloc only: B * H * N above ATTN_NOALLOC_MAX_ROWS */
};

/* Forward pass (paper Sec. 2.1 first display; tiled evaluation per Sec. 3.1.4).
 *   in : q [B,N,H,d_qk], k [B,N,Hkv,d_qk], v [B,N,Hkv,d_v]   bf16, device
 *   out: o [B,N,H,d_v] bf16, lse [B,H,N] fp32                 device
 * attn_fwd is attn_fwd_ex with d_qk = d_v = d. */
int attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
             int B, int H, int Hkv, int N, int d, float scale, int causal, void* stream);
int attn_fwd_ex(const void* q, const void* k, const void* v, void* o, float* lse,
                int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                void* stream);

/* Backward pass (paper Sec. 2.1 second display).
 *   in : q, k, v as above; o, d_o [B,N,H,d_v] bf16; lse [B,H,N] fp32 -- o and lse
 *        must be the outputs of the forward call with the same arguments
 *   out: dq [B,N,H,d_qk], dk [B,N,Hkv,d_qk], dv [B,N,Hkv,d_v]  bf16
 *   workspace: device scratch of at least attn_bwd_workspace_bytes(...) bytes,
 *        256-byte aligned; contents on entry are ignored, contents on exit are
 *        unspecified; may be reused by the next call on the same stream.
 * Two kernels are enqueued, in this order: the dQ kernel (one workgroup per query tile, dQ
 * accumulated on chip over all KV tiles; it also forms D = rowsum(dO o O) and the base-2 LSE of
 * its rows and leaves them in the workspace), then the dK/dV kernel (one workgroup per KV tile,
 * dK and dV accumulated on chip over all query tiles and all query heads of the group: the loop
 * structure of paper Sec. 3.2.2).  The paper
 * accumulates dQ with global atomics inside the dK/dV loop (Sec. 3.2.2-3.2.3); on MI355X
 * those atomics are memory-side and cost more than recomputing S and dP, so dQ has its
 * own pass.  No atomics are used: results are bit-reproducible from run to run (the
 * property paper Sec. 3.2.4 obtains with semaphores). */
int attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* d_o,
             const float* lse, void* dq, void* dk, void* dv,
             int B, int H, int Hkv, int N, int d, float scale, int causal,
             void* workspace, size_t workspace_bytes, void* stream);
int attn_bwd_ex(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                const float* lse, void* dq, void* dk, void* dv,
                int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                void* workspace, size_t workspace_bytes, void* stream);

/* attn_bwd_ex restricted to a subset of its passes, for per-kernel timing and profiling (the
 * backward of paper Sec. 3.2 is one logical step; this splits it at the kernel boundaries).
 * phases is a bit mask: ATTN_BWD_PREPARE (-D and base-2 LSE into the workspace), ATTN_BWD_DKDV
 * (writes dk, dv; reads -D and the base-2 LSE from the workspace), ATTN_BWD_DQ (writes dq).  All
 * arguments as attn_bwd_ex.  The dQ kernel computes -D and the base-2 LSE of its own rows
 * itself (the same values bit for bit as the prepare kernel) and writes them to the workspace,
 * so a call whose mask includes ATTN_BWD_DQ launches no prepare kernel: the dQ kernel runs first
 * and ATTN_BWD_DKDV, of the same or of a later call, reads what it left.  attn_bwd_ex is
 * therefore two kernels; ATTN_BWD_PREPARE has an effect only in a mask without ATTN_BWD_DQ. */
enum { ATTN_BWD_PREPARE = 1, ATTN_BWD_DKDV = 2, ATTN_BWD_DQ = 4, ATTN_BWD_ALL = 7 };
int attn_bwd_phases(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                    const float* lse, void* dq, void* dk, void* dv,
                    int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                    void* workspace, size_t workspace_bytes, void* stream, int phases);

/* attn_bwd_ex for callers that cannot allocate device memory at all: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc (and with it torch's allocator).  The
 * workspace (-D and the base-2 LSE, 8 bytes per row of B * H * N) is an array inside the library's
 * own device image, 8 MiB per GPU the library runs on, held until the process ends; this call and
 * everything it reaches allocates and frees nothing.  Inputs, outputs, layouts and results are
 * those of attn_bwd_ex (bit for bit).
 *   - B * H * N must not exceed ATTN_NOALLOC_MAX_ROWS; beyond that the call returns
 *     ATTN_ETOOLARGE with nothing enqueued.
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (on
 *     different streams, or from different host threads) race on it.  Calls on one stream, or
 *     ordered by events, are fine; nothing needs to be cleared between calls (every row that is
 *     read has been written earlier in the same call). */
#define ATTN_NOALLOC_MAX_ROWS (1 << 20)
int attn_bwd_noalloc(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                     const float* lse, void* dq, void* dk, void* dv,
                     int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                     void* stream);

/* Bytes of workspace attn_bwd(_ex) needs for these sizes (0 if they are invalid):
 * D and the base-2 LSE, [B,H,N] fp32 each (256-byte aligned sections). */
size_t attn_bwd_workspace_bytes(int B, int H, int Hkv, int N, int d_qk, int d_v);

/* Variable sequence lengths (paper Sec. 3.3: a list of query and key/value sequence lengths per
 * batch): B sequences packed back to back, attention inside each sequence only; a sequence's
 * number of queries and number of keys may differ (cross-attention, decoding against a cache).
 *   layouts  q, o, d_o, dq : [Tq, H, d]    k, dk : [Tk, Hkv, d_qk]    v, dv : [Tk, Hkv, d_v]   bf16
 *            lse           : [H, Tq] fp32
 *            cu_seqlens_q  : [B + 1] int32, DEVICE memory, cu[0] = 0, non-decreasing,
 *                            cu[B] = Tq = total_q; sequence b owns query rows cu[b] .. cu[b+1]-1.
 *            cu_seqlens_k  : the same for the key/value rows, cu[B] = Tk = total_k; may be the same
 *                            pointer as cu_seqlens_q (self-attention).
 *                            Any length >= 0 is allowed (no multiple-of-128 requirement), except that
 *                            a sequence with queries must have at least one key, and under a causal
 *                            mask at least as many keys as queries.
 *   causal != 0: the last query of a sequence is aligned with its last key: key j is visible to
 *   query i iff j <= i + (keys - queries) of that sequence; j <= i for self-attention.
 *   The host never reads the lengths: a small kernel turns them into tables of 128-row tiles,
 *   sequences with the longest loop per tile first (the longest-processing-time-first order of
 *   Sec. 3.3), and the attention kernels are launched over upper bounds of total_q/128 + B query
 *   tiles per head and total_k/128 + B key tiles per key/value head.
 *   workspace: attn_varlen_workspace_bytes(..., backward) bytes, 256-byte aligned; the forward
 *   call needs the backward = 0 size, the backward call the backward = 1 size.  Contents on entry
 *   are ignored.  All other conventions (device pointers, stream, alignment, head dims, error
 *   codes) are those of attn_fwd_ex / attn_bwd_ex.  The table kernel checks every sequence's
 *   boundaries on the device against total_q and total_k: a sequence whose rows do not lie inside
 *   the tensors (decreasing boundaries, boundaries past the totals) is left out, i.e. none of its
 *   rows is read or written, and the other sequences are served.  The remaining conditions (a key
 *   for every sequence with queries; keys >= queries under a causal mask) are not checked: rows
 *   that violate them hold unspecified values, nothing outside the tensors is touched. */
size_t attn_varlen_workspace_bytes(int B, int total_q, int total_k, int H, int Hkv, int d_qk, int d_v, int backward);
int attn_varlen_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                    const int* cu_seqlens_q, const int* cu_seqlens_k, int B, int total_q, int total_k,
                    int H, int Hkv, int d_qk, int d_v,
                    float scale, int causal, void* workspace, size_t workspace_bytes, void* stream);
/* The tile tables alone (paper Sec. 3.3: the sort's metadata can be cached).  Fills both tables
 * at the head of a workspace of the backward = 1 size.  A later attn_varlen_fwd / attn_varlen_bwd
 * (or _dtype) call on that workspace with the SAME B, total_q, total_k, H, Hkv and head dims may
 * then pass cu_seqlens_q = cu_seqlens_k = NULL: it skips the plan kernel and uses the tables as
 * they are (a backward call needs tables written by this function or by an earlier backward call;
 * a forward call with non-NULL cu_seqlens writes the query table only).  Calls never modify the
 * tables otherwise; results are bit-identical to those of calls that rebuild them.  Table entries
 * carry a mark and are checked against total_q: on a workspace that was never planned the kernels
 * find nothing to act on and leave the outputs untouched (tables planned for OTHER lengths with
 * the same totals cannot be told apart: that remains the caller's responsibility). */
int attn_varlen_plan(const int* cu_seqlens_q, const int* cu_seqlens_k, int B, int total_q, int total_k,
                     int H, int Hkv, int d_qk, int d_v, void* workspace, size_t workspace_bytes, void* stream);
/* Backward of attn_varlen_fwd (paper Sec. 2.1 second display, per sequence): o and lse must be that
 * call's outputs for the same arguments; dk and dv are summed over the query heads of each group.
 * Every row of dq, dk, dv is written (dk = dv = 0 for the keys of a sequence without queries).
 * No atomics: bit-reproducible like attn_bwd. */
int attn_varlen_bwd(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                    const float* lse, void* dq, void* dk, void* dv,
                    const int* cu_seqlens_q, const int* cu_seqlens_k, int B, int total_q, int total_k,
                    int H, int Hkv, int d_qk, int d_v,
                    float scale, int causal, void* workspace, size_t workspace_bytes, void* stream);

/* The same four operations on IEEE fp16 storage (the paper's benchmarks cover FP16 and BF16
 * inputs, Sec. 5): dtype = ATTN_BF16 is exactly the entry point without the suffix, dtype =
 * ATTN_F16 reads q, k, v, o, d_o and writes o, dq, dk, dv as fp16 (round to nearest even), with
 * fp16 MFMA operands (P and dS are rounded to fp16) and fp32 accumulation, statistics and LSE.
 * Any other dtype: ATTN_EUNSUPPORTED.  All remaining arguments and conventions as in
 * attn_fwd_ex, attn_bwd_ex, attn_varlen_fwd, attn_varlen_bwd. */
enum { ATTN_BF16 = 0, ATTN_F16 = 1 };
int attn_fwd_dtype(int dtype, const void* q, const void* k, const void* v, void* o, float* lse,
                   int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal, void* stream);
int attn_bwd_dtype(int dtype, const void* q, const void* k, const void* v, const void* o, const void* d_o,
                   const float* lse, void* dq, void* dk, void* dv,
                   int B, int H, int Hkv, int N, int d_qk, int d_v, float scale, int causal,
                   void* workspace, size_t workspace_bytes, void* stream);
int attn_varlen_fwd_dtype(int dtype, const void* q, const void* k, const void* v, void* o, float* lse,
                          const int* cu_seqlens_q, const int* cu_seqlens_k, int B, int total_q, int total_k,
                          int H, int Hkv, int d_qk, int d_v,
                          float scale, int causal, void* workspace, size_t workspace_bytes, void* stream);
int attn_varlen_bwd_dtype(int dtype, const void* q, const void* k, const void* v, const void* o, const void* d_o,
                          const float* lse, void* dq, void* dk, void* dv,
                          const int* cu_seqlens_q, const int* cu_seqlens_k, int B, int total_q, int total_k,
                          int H, int Hkv, int d_qk, int d_v,
                          float scale, int causal, void* workspace, size_t workspace_bytes, void* stream);

/* Strided layouts: the same attention on equal-length batches whose tensors are views with
 * arbitrary batch, token and head strides -- [B, H, N, d] tensors, slices of a fused QKV
 * projection, padded buffers -- with Nq >= 1 queries and Nk >= 1 keys per sequence (no
 * multiple-of-128 requirement; Nq != Nk is a prefix held in a cache, a decode step or
 * cross-attention).  The head dim is contiguous.  Element (b, n, h, c) of a tensor x with strides
 * sx (counted in ELEMENTS) is x[b * sx->batch + n * sx->row + h * sx->head + c]; q, o, d_o, dq
 * have Nq tokens and H heads, k, v, dk, dv Nk tokens and Hkv heads.
 * Every stride must be a non-negative multiple of 8 (16-byte vector accesses), non-zero
 * wherever the corresponding extent exceeds 1, and the token stride at most 2^23 elements;
 * outputs must not overlap themselves or any input.  lse is [B, H, Nq] fp32, contiguous.
 * causal != 0: the last query is aligned with the last key, key j is visible to query i iff
 * j <= i + Nk - Nq (the convention of the variable-length calls; the paper is silent on
 * Nq != Nk), and Nk >= Nq is required (ATTN_EINVAL otherwise).
 * Runs the variable-length kernels on the sequence boundaries {0, Nq, 2 Nq, ...} and
 * {0, Nk, 2 Nk, ...} generated on the device; on contiguous [B, N, H, d] tensors with
 * Nq = Nk = N a multiple of 128 the results are bit-identical to attn_fwd_ex / attn_bwd_ex.
 *   workspace: attn_strided_workspace_bytes(..., backward) bytes, 256-byte aligned, contents
 *   ignored on entry.  Other conventions as in attn_fwd_dtype / attn_bwd_dtype. */
typedef struct attn_strides {
    long long batch, row, head;
} attn_strides_t;
size_t attn_strided_workspace_bytes(int B, int H, int Hkv, int Nq, int Nk, int d_qk, int d_v, int backward);
int attn_fwd_strided(int dtype, const void* q, const attn_strides_t* sq, const void* k, const attn_strides_t* sk,
                     const void* v, const attn_strides_t* sv, void* o, const attn_strides_t* so, float* lse,
                     int B, int H, int Hkv, int Nq, int Nk, int d_qk, int d_v, float scale, int causal,
                     void* workspace, size_t workspace_bytes, void* stream);
int attn_bwd_strided(int dtype, const void* q, const attn_strides_t* sq, const void* k, const attn_strides_t* sk,
                     const void* v, const attn_strides_t* sv, const void* o, const attn_strides_t* so,
                     const void* d_o, const attn_strides_t* sdo, const float* lse,
                     void* dq, const attn_strides_t* sdq, void* dk, const attn_strides_t* sdk,
                     void* dv, const attn_strides_t* sdv,
                     int B, int H, int Hkv, int Nq, int Nk, int d_qk, int d_v, float scale, int causal,
                     void* workspace, size_t workspace_bytes, void* stream);

/* Software 2^x of paper Sec. 3.1.3 (range reduction + degree-n minimax polynomial, p0 = 1, Horner
 * with FMAs, exponent splice), provided to measure its accuracy on this hardware; attn_fwd does not
 * use it (v_exp_f32 and the FMAs share one issue port on CDNA4, so emulation cannot add throughput:
 * the rate probes that show this live in a library of their own, include/attn_probes.h).
 *   attn_exp2_emulated: y[i] = 2^x[i] for n fp32 values; degree 3, 4 or 5, or 0 for the hardware
 *       instruction.  x, y: device pointers, 4-byte aligned, may not overlap partially. */
int attn_exp2_emulated(const float* x, float* y, size_t n, int degree, void* stream);

/* Human-readable text for a return code (static storage). */
const char* attn_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int attn_version(void);

#ifdef __cplusplus
}
#endif
#endif
