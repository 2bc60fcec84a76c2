// Plan tables of the variable-length entry points (paper Sec. 3.3: variable sequence lengths are
// served longest first, after a preprocessing kernel that sorts the batch).
//
// Input: cu_q[0..B] and cu_k[0..B] (device), the running token counts of the packed query-side
// and key-side tensors: sequence b owns query rows cu_q[b] .. cu_q[b+1]-1 and key rows
// cu_k[b] .. cu_k[b+1]-1 (cu_k may be the same array: self-attention).
// Output: two tables, one entry per 128-row QUERY tile and one per 128-row KEY tile.  An entry is
// two int4: {first query row, query length, first key row, key length} of the sequence and
// {tile index inside the sequence, kPlanUsed, sequence index, 0}.  Sequences are ordered by the length of the loop one
// of their tiles runs -- the key tile count for query tiles, the query tile count for key tiles --
// longest first (a counting sort over tile counts; ties keep no particular order, which does not
// matter because no result depends on which block computes which tile), and inside a sequence
// from the last tile to the first (under a causal mask the last query tile has the longest key
// loop; the dK/dV kernels read the index backwards for the same reason).  Unused entries up to
// the table size are zero.  The kernels size their grids by the table sizes, host-side upper
// bounds, because the host never reads the lengths; for the same reason the boundaries are checked
// here, on the device, against the row counts the caller stated: a sequence that does not lie
// inside the tensors is left out of both tables.
#include "common.h"
#include "launch.h"

namespace attn {

constexpr int PLAN_NT = 1024;
constexpr int PLAN_BUCKETS = 4096;      // loop lengths 0 .. 4095 tiles; longer ones share the top bucket

// One table.  own/other: the side whose tiles are listed and the side they loop over.
__device__ void plan_build(const int* __restrict__ cu_q, const int* __restrict__ cu_k, int B, int Tq, int Tk, bool own_is_q,
                           int4* __restrict__ plan, int max_tiles, int* hist, int* start, int* part)
{
    static_assert(PLAN_BUCKETS == 4 * PLAN_NT, "four buckets per thread in the scan below");
    const int tid = threadIdx.x;
    for (int i = tid; i < PLAN_BUCKETS; i += PLAN_NT) hist[i] = 0;
    for (int i = tid; i < 2 * max_tiles; i += PLAN_NT) plan[i] = make_int4(0, 0, 0, 0);
    __syncthreads();
    auto tiles = [](int len) { return (len + 127) / 128; };
    auto bucket_of = [](int nt) { return nt < PLAN_BUCKETS ? nt : PLAN_BUCKETS - 1; };
    // a sequence contributes its own tiles; query tiles of a sequence without keys are not listed
    auto own_tiles = [&](int ql, int kl) { return own_is_q ? (kl > 0 ? tiles(ql) : 0) : tiles(kl); };
    auto key_of = [&](int ql, int kl) { return bucket_of(tiles(own_is_q ? kl : ql)); };
    // A sequence whose rows do not lie inside the tensors (boundaries that decrease, or that run past
    // the totals the caller stated) gets no tiles at all: nothing of it is read or written.
    auto inside = [&](int qs, int ql, int ks, int kl) {
        return qs >= 0 && ql >= 0 && qs <= Tq - ql && ks >= 0 && kl >= 0 && ks <= Tk - kl;
    };
    for (int b = tid; b < B; b += PLAN_NT) {
        const int qs = cu_q[b], ql = cu_q[b + 1] - qs, ks = cu_k[b], kl = cu_k[b + 1] - ks;
        const int nt = inside(qs, ql, ks, kl) ? own_tiles(ql, kl) : 0;
        if (nt > 0) atomicAdd(&hist[key_of(ql, kl)], nt);
    }
    __syncthreads();
    // Exclusive prefix sum of the tile counts over the buckets from the longest loop down.
    // Position p = 0 .. PLAN_BUCKETS-1 stands for bucket PLAN_BUCKETS-1-p; every thread owns four
    // consecutive positions.
    int w[4], local = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) { w[e] = hist[PLAN_BUCKETS - 1 - (4 * tid + e)]; local += w[e]; }
    part[tid] = local;
    __syncthreads();
    for (int off = 1; off < PLAN_NT; off <<= 1) {          // inclusive Hillis-Steele scan of the partials
        const int add = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    int run = part[tid] - local;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        start[PLAN_BUCKETS - 1 - (4 * tid + e)] = run;
        run += w[e];
    }
    __syncthreads();
    for (int i = tid; i < PLAN_BUCKETS; i += PLAN_NT) hist[i] = 0;     // becomes the per-bucket tile cursor
    __syncthreads();
    for (int b = tid; b < B; b += PLAN_NT) {
        const int qs = cu_q[b], ql = cu_q[b + 1] - qs, ks = cu_k[b], kl = cu_k[b + 1] - ks;
        const int nt = inside(qs, ql, ks, kl) ? own_tiles(ql, kl) : 0;
        if (nt <= 0) continue;
        const int key = key_of(ql, kl);
        const int first = start[key] + atomicAdd(&hist[key], nt);
        for (int t = 0; t < nt; ++t)
            if (first + t < max_tiles) {
                plan[2 * (first + t)] = make_int4(qs, ql, ks, kl);
                plan[2 * (first + t) + 1] = make_int4(nt - 1 - t, kPlanUsed, b, 0);
            }
    }
    __syncthreads();
}

__global__ void __launch_bounds__(PLAN_NT)
varlen_plan_kernel(const int* __restrict__ cu_q, const int* __restrict__ cu_k, int B, int Tq, int Tk,
                   int4* __restrict__ plan_q, int max_tiles_q, int4* __restrict__ plan_k, int max_tiles_k)
{
    __shared__ int hist[PLAN_BUCKETS];       // tiles per bucket, then next free tile per bucket
    __shared__ int start[PLAN_BUCKETS];      // first table entry of each bucket
    __shared__ int part[PLAN_NT];
    plan_build(cu_q, cu_k, B, Tq, Tk, true, plan_q, max_tiles_q, hist, start, part);
    if (plan_k) plan_build(cu_q, cu_k, B, Tq, Tk, false, plan_k, max_tiles_k, hist, start, part);   // backward only
}

__global__ void uniform_cu_kernel(int* __restrict__ cu, int B, int N)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b <= B) cu[b] = b * N;
}

int launch_uniform_cu(int* cu, int B, int N, void* stream)
{
    return launch_kernel(uniform_cu_kernel, dim3((B + 256) / 256), dim3(256), 0, stream, cu, B, N) == hipSuccess ? 0 : -3;
}

int launch_varlen_plan(const int* cu_q, const int* cu_k, int B, int Tq, int Tk, void* plan_q, int max_tiles_q,
                       void* plan_k, int max_tiles_k, void* stream)
{
    return launch_kernel(varlen_plan_kernel, dim3(1), dim3(PLAN_NT), 0, stream, cu_q, cu_k, B, Tq, Tk,
                         (int4*)plan_q, max_tiles_q, (int4*)plan_k, max_tiles_k) == hipSuccess ? 0 : -3;
}

}  // namespace attn
