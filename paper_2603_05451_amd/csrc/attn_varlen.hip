// Plan table of the variable-length entry points (paper Sec. 3.3: variable sequence lengths are
// served longest first, after a preprocessing kernel that sorts the batch).
//
// Input: cu_seqlens[0..B] (device), the running token count: sequence b owns token rows
// cu[b] .. cu[b+1]-1.  Output: one int4 per 128-row tile, {first row of the sequence, its length,
// tile index inside the sequence, 1}, sequences ordered by their tile count, longest first (a
// counting sort: ties keep no particular order, which does not matter because no result depends
// on which block computes which tile), and inside a sequence from the last tile to the first
// (under a causal mask the last query tile has the longest key loop).  Unused entries up to
// max_tiles are {0, 0, 0, 0}.  The kernels size their grids by max_tiles, a host-side upper
// bound, because the host never reads cu_seqlens.
#include "common.h"
#include "launch.h"

namespace attn {

constexpr int PLAN_NT = 1024;
constexpr int PLAN_BUCKETS = 4096;      // tile counts 0 .. 4095 (sequences up to 524 160 tokens); longer ones share the top bucket

__global__ void __launch_bounds__(PLAN_NT)
varlen_plan_kernel(const int* __restrict__ cu, int B, int4* __restrict__ plan, int max_tiles)
{
    static_assert(PLAN_BUCKETS == 4 * PLAN_NT, "four buckets per thread in the scan below");
    __shared__ int hist[PLAN_BUCKETS];       // sequences per tile count, then next free slot per bucket
    __shared__ int tile_start[PLAN_BUCKETS]; // first plan entry of each bucket
    __shared__ int part[PLAN_NT];
    const int tid = threadIdx.x;
    for (int i = tid; i < PLAN_BUCKETS; i += PLAN_NT) hist[i] = 0;
    for (int i = tid; i < max_tiles; i += PLAN_NT) plan[i] = make_int4(0, 0, 0, 0);
    __syncthreads();
#ifdef ATTN_PLAN_GIVEN_ORDER   // measurement only: the batch order as given, no sort
    if (tid == 0) {
        int run = 0;
        for (int b = 0; b < B; ++b) {
            const int len = cu[b + 1] - cu[b], nt = (len + 127) / 128;
            for (int t = 0; t < nt && run < max_tiles; ++t) plan[run++] = make_int4(cu[b], len, nt - 1 - t, 1);
        }
    }
    return;
#endif
    auto bucket_of = [](int nt) { return nt < PLAN_BUCKETS ? nt : PLAN_BUCKETS - 1; };
    for (int b = tid; b < B; b += PLAN_NT) {
        const int len = cu[b + 1] - cu[b];
        if (len > 0) atomicAdd(&hist[bucket_of((len + 127) / 128)], 1);
    }
    __syncthreads();
    // Sequences in the top bucket may differ in tile count, so that (normally empty) bucket is
    // laid out first, by one thread, sequentially.
    __shared__ int top_tiles;
    if (tid == 0) {
        int run = 0;
        if (hist[PLAN_BUCKETS - 1] > 0) {
            for (int b = 0; b < B; ++b) {
                const int len = cu[b + 1] - cu[b];
                const int nt = (len + 127) / 128;
                if (len > 0 && nt >= PLAN_BUCKETS - 1)
                    for (int t = 0; t < nt && run < max_tiles; ++t) plan[run++] = make_int4(cu[b], len, nt - 1 - t, 1);
            }
        }
        top_tiles = run;
    }
    // Exclusive prefix sum of hist[nt] * nt over the other buckets from the largest tile count
    // down.  Position p = 0 .. PLAN_BUCKETS-1 stands for bucket PLAN_BUCKETS-2-p (p beyond that: empty);
    // every thread owns four consecutive positions.
    auto weight = [&](int p) { const int nt = PLAN_BUCKETS - 2 - p; return nt >= 1 ? hist[nt] * nt : 0; };
    int w[4], local = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) { w[e] = weight(4 * tid + e); local += w[e]; }
    part[tid] = local;
    __syncthreads();
    for (int off = 1; off < PLAN_NT; off <<= 1) {          // inclusive Hillis-Steele scan of the partials
        const int add = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    int run = top_tiles + part[tid] - local;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int nt = PLAN_BUCKETS - 2 - (4 * tid + e);
        if (nt >= 1) tile_start[nt] = run;
        run += w[e];
    }
    __syncthreads();
    for (int i = tid; i < PLAN_BUCKETS - 1; i += PLAN_NT) hist[i] = 0;   // becomes the per-bucket sequence counter
    __syncthreads();
    for (int b = tid; b < B; b += PLAN_NT) {
        const int start = cu[b], len = cu[b + 1] - start;
        const int nt = (len + 127) / 128;
        if (len <= 0 || nt >= PLAN_BUCKETS - 1) continue;
        const int first = tile_start[nt] + atomicAdd(&hist[nt], 1) * nt;
        for (int t = 0; t < nt; ++t)
            if (first + t < max_tiles) plan[first + t] = make_int4(start, len, nt - 1 - t, 1);
    }
}

int launch_varlen_plan(const int* cu_seqlens, int B, void* plan, int max_tiles, void* stream)
{
    return launch_kernel(varlen_plan_kernel, dim3(1), dim3(PLAN_NT), 0, stream, cu_seqlens, B, (int4*)plan,
                         max_tiles) == hipSuccess ? 0 : -3;
}

}  // namespace attn
