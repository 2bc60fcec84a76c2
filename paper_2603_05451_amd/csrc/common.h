// Shared device-side vocabulary for the gfx950 attention kernels: vector types, the
// MFMA wrappers with their register layouts spelled out, LDS tile addressing and the
// asynchronous global->LDS tile copy.  HIP/CDNA4 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace attn {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef _Float16 f16;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

#define ATTN_LDS __attribute__((address_space(3)))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// Threshold of the conditional rescale in base-2 units (paper Sec. 3.1.4: log2(256)).
constexpr float kRescaleTau = 8.0f;

// v_mfma_f32_32x32x16_bf16, D = A(32x16) * B(16x32) + C.  Lane l = 32*h + c:
//   A: row c,  k = 8h..8h+7           B: column c, k = 8h..8h+7
//   C/D register r: row 8*(r/4) + 4h + r%4, column c.
// A permutation of k applied to A and B alike leaves the product unchanged.
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 mfma32(f16x8 a, f16x8 b, f32x16 c)      // v_mfma_f32_32x32x16_f16, same layouts
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// Row of a 32x32 accumulator register r for lane half h.
__device__ __forceinline__ constexpr int acc_row(int r, int h) { return 8 * (r >> 2) + 4 * h + (r & 3); }

// max / sum with the lane 32 apart (v_permlane32_swap exchanges the upper half of the first
// operand with the lower half of the second).
__device__ __forceinline__ float xhalf_max(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// ---------------------------------------------------------------------------------------
// LDS tiles.  A tile holds ROWS rows of D bf16 (D/8 chunks of 16 bytes per row), rows
// contiguous, chunks XOR-swizzled inside a row so that both access patterns below are
// bank-conflict free with no padding (padding is impossible: the global->LDS copy writes
// 64 consecutive 16-byte chunks per wave instruction).
//
//   row pattern : one 16-byte chunk per lane, 16 consecutive lanes = 16 consecutive rows,
//                 same logical chunk (MFMA operand contracted over the head dimension);
//   tr pattern  : ds_read_b64_tr_b16, 16 lanes fetch 4 consecutive rows x 32 bytes, a pair
//                 of such groups covers 4 rows x 64 bytes = one aligned group of 4 chunks
//                 (MFMA operand contracted over the row index).
//
// Banks repeat every 256 bytes = 16 chunks.  With 16 chunks per row (D = 128) every row
// starts at bank 0, so the XOR value must (a) take 16 distinct values over 16 consecutive
// rows and (b) move the aligned 4-chunk group to 4 distinct groups over 4 consecutive
// rows: x = ((row & 3) << 2) | ((row >> 2) & 3).  With 8 or 24 chunks per row (D = 64,
// 192) rows alternate between bank 0 and bank 32, the XOR stays inside an aligned group
// of 8 chunks, and the same two conditions give, with y = row >> 1,
// x = ((y & 1) << 2) | ((y >> 1) & 3).  With 12 chunks per row (D = 96) the rows start at chunk
// offsets 0, 12, 8, 4 (mod 16): four consecutive rows already occupy four different 4-chunk
// groups, rows four apart coincide, and an XOR inside the aligned group of 4 chunks (the widest
// that stays inside a 12-chunk row) with x = (row >> 2) & 3 separates those.
// ---------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ int swz_chunk(int row, int chunk)
{
    constexpr int CPR = D / 8;
    if constexpr (CPR % 16 == 0) {
        return chunk ^ (((row & 3) << 2) | ((row >> 2) & 3));
    } else if constexpr (CPR % 8 != 0) {
        static_assert(CPR % 4 == 0, "head dims are multiples of 32");
        return chunk ^ ((row >> 2) & 3);
    } else {
        const int y = row >> 1;
        return chunk ^ (((y & 1) << 2) | ((y >> 1) & 3));
    }
}

// Byte offset of logical 16-byte chunk `chunk` of row `row`.
template <int D>
__device__ __forceinline__ int tile_off(int row, int chunk)
{
    return (row * (D / 8) + swz_chunk<D>(row, chunk)) * 16;
}

// One wave instruction of the global->LDS DMA: every lane copies 16 bytes from its own global
// address to LDS address (lds_base + 16 * lane); lds_base must be wave-uniform (it travels in
// M0).  Issued through inline assembly on purpose: the compiler then does not know that LDS is
// being written asynchronously and inserts no vmcnt waits of its own in front of later LDS
// reads; the kernels order the copy explicitly (wait_async_copies + workgroup barrier).
// vmcnt operations the compiler cannot see only ever make its own waits stricter.
__device__ __forceinline__ void dma16(const void* gsrc, ATTN_LDS char* lds_base)
{
    const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(m0), "v"(gsrc) : "memory");
}
__device__ __forceinline__ void dma4(const void* gsrc, ATTN_LDS char* lds_base)   // 4 bytes per lane
{
    const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                 :: "s"(m0), "v"(gsrc) : "memory");
}

// Tile copy for the main loops: ROWS x D 16-bit elements from global memory (row stride given in
// elements) into an LDS tile, by all NT threads of the block, without VGPR staging: each wave
// instruction moves 64 x 16 bytes straight into LDS.  Completion is observed with
// wait_async_copies() followed by a workgroup barrier.  The per-lane byte offsets inside a tile
// and the wave's LDS slice offsets are computed once (init); a tile is then copied with N wave
// instructions that take the tile's global base address in SGPRs (advanced with scalar
// arithmetic per tile) and the lane offset in one VGPR: no vector ALU work per tile.
template <int ROWS, int D, int NT>
struct TileCopy {
    static constexpr int N = ROWS * (D / 8) / NT;   // wave instructions per thread and tile
    uint32_t goff[N];                                // byte offset of this lane's 16 bytes inside the tile
    uint32_t loff[N];                                // byte offset of the wave's 1 KiB slice in the LDS tile
    __device__ __forceinline__ void init(int64_t gstride, int tid)
    {
        constexpr int CPR = D / 8;
        const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
        for (int t = 0; t < N; ++t) {
            const int p0 = (t * (NT / 64) + wave) * 64;
            const int p = p0 + lane;
            const int row = p / CPR;
            goff[t] = (uint32_t)(row * (int)gstride + swz_chunk<D>(row, p % CPR) * 8) * 2u;
            loff[t] = __builtin_amdgcn_readfirstlane((uint32_t)(p0 * 16));
        }
    }
    // gtile must be wave-uniform (it is passed in SGPRs)
    __device__ __forceinline__ void issue(int t, const void* gtile, ATTN_LDS char* lds_tile) const
    {
        const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds_tile) + loff[t];
        const uint64_t base = (uint64_t)gtile;
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)base);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32));
        const uint64_t sbase = ((uint64_t)hi << 32) | lo;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(m0), "v"(goff[t]), "s"(sbase) : "memory");
    }
    __device__ __forceinline__ void issue_all(const void* gtile, ATTN_LDS char* lds_tile) const
    {
#pragma unroll
        for (int t = 0; t < N; ++t) issue(t, gtile, lds_tile);
    }
    // The same copy for a tile of which only the first `valid_rows` (>= 1) rows exist: every
    // later row re-reads the last valid one, so nothing outside the tensor is touched.  Per-lane
    // address arithmetic; meant for the one ragged tile at the end of a sequence.  `tid` and the
    // row stride must be those given to init.
    __device__ __forceinline__ void issue_all_guarded(const void* gtile, ATTN_LDS char* lds_tile,
                                                      int valid_rows, int64_t gstride, int tid) const
    {
        constexpr int CPR = D / 8;
        const int wave = tid >> 6, lane = tid & 63;
        const uint32_t row_bytes = (uint32_t)gstride * 2u;
#pragma unroll
        for (int t = 0; t < N; ++t) {
            const int row = ((t * (NT / 64) + wave) * 64 + lane) / CPR;
            const int over = row - (valid_rows - 1);
            const uint32_t off = goff[t] - (over > 0 ? (uint32_t)over * row_bytes : 0u);
            const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds_tile) + loff[t];
            const uint64_t base = (uint64_t)gtile;
            const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)base);
            const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32));
            const uint64_t sbase = ((uint64_t)hi << 32) | lo;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(m0), "v"(off), "s"(sbase) : "memory");
        }
    }
};

// Compile-time loop: f(std::integral_constant<int, I>) for I = 0 .. N-1.
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

__device__ __forceinline__ void wait_async_copies() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Make the compiler treat a register value as produced here: any wait for the load that fed
// it is placed before this point (used to keep vmcnt waits for one-off global loads out of
// loops that have DMA copies in flight).
template <typename T>
__device__ __forceinline__ void pin_ready(T& x) { asm volatile("" : "+v"(x)); }

// Scheduling fence: memory and MFMA instructions stay on their side, plain VALU/SALU/
// transcendental work may move across (so softmax arithmetic can fill MFMA shadows).
__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0x2 | 0x4 | 0x400); }

// ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives element (i % 4) of the
// 8-byte rows fetched by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4 of the group.
__device__ __forceinline__ s16x4 lds_read_tr_bits(const ATTN_LDS char* p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((ATTN_LDS s16x4*)p);
}

}  // namespace attn
