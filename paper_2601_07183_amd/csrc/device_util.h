// Small device helpers shared by the kernel files.
#pragma once
#include "rairs_common.h"

#define WG 256

static __host__ __device__ __forceinline__ int next_pow2(int x)
{
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

// Ascending bitonic sort of n (power of two) 64-bit keys in LDS by the whole workgroup.
// Callers synchronise before; the array is consistent for all threads on return.
static __device__ void bitonic_sort_lds(uint64_t *a, int n)
{
    for (int k = 2; k <= n; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < n; i += WG) {
                int p = i ^ j;
                if (p > i) {
                    bool up = (i & k) == 0;
                    uint64_t x = a[i], y = a[p];
                    if ((x > y) == up) { a[i] = y; a[p] = x; }
                }
            }
            __syncthreads();
        }
}

// Ordering point for a wave that exchanges data between its lanes through its own LDS region (no
// other wave touches it): LDS operations of one wave complete in issue order, so only the
// compiler has to be kept from moving accesses across.
static __device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Ascending bitonic sort of n (power of two) 64-bit keys in a wave's own LDS region, by that wave.
static __device__ __forceinline__ void wave_bitonic_sort_lds(uint64_t *a, int n, int lane)
{
    for (int k = 2; k <= n; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = lane; i < n; i += 64) {
                const int p = i ^ j;
                if (p > i) {
                    const bool up = (i & k) == 0;
                    const uint64_t x = a[i], y = a[p];
                    if ((x > y) == up) { a[i] = y; a[p] = x; }
                }
            }
            wave_lds_sync();
        }
}

// The value of lane (l ^ s) of a wave, s = 8, 4, 2, 1, by data-parallel register moves instead of a
// trip through the LDS crossbar: within a row of 16 lanes a rotation by 8 is l ^ 8; l ^ 4 takes a
// shift left into lanes 0-3 and 8-11 and a shift right into the others; l ^ 2 and l ^ 1 are
// permutations of four lanes.
static __device__ __forceinline__ float lane_xor8(float c)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, c), 0x128, 0xf, 0xf, false));   // row_ror:8
}
static __device__ __forceinline__ float lane_xor4(float c)
{
    const int x = __builtin_bit_cast(int, c);
    int t = __builtin_amdgcn_update_dpp(x, x, 0x104, 0xf, 0x5, false);      // row_shl:4 into lanes 0-3, 8-11 of a row
    t = __builtin_amdgcn_update_dpp(t, x, 0x114, 0xf, 0xa, false);          // row_shr:4 into lanes 4-7, 12-15
    return __builtin_bit_cast(float, t);
}
static __device__ __forceinline__ float lane_xor2(float c)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, c), 0x4e, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
}
static __device__ __forceinline__ float lane_xor1(float c)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, c), 0xb1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
}

// Smallest of the 64 lanes' 64-bit keys, in every lane: a butterfly over strides 32 .. 1 whose
// exchanges are register moves.  After swapping the upper half of one copy of a register with the
// lower half of another copy, every lane holds its own value in one and its partner's in the
// other, so the step is just the minimum of the two (likewise at stride 16 with 16-lane rows).
static __device__ __forceinline__ uint64_t wave_min_u64(uint64_t x)
{
    uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
    {
        uint32_t lo2 = lo, hi2 = hi;
        asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_permlane32_swap_b32 %2, %3\n\ts_nop 1"
            : "+v"(lo), "+v"(lo2), "+v"(hi), "+v"(hi2));
        const uint64_t a = ((uint64_t)hi << 32) | lo, b = ((uint64_t)hi2 << 32) | lo2;
        const uint64_t m = a < b ? a : b;
        lo = (uint32_t)m; hi = (uint32_t)(m >> 32);
    }
    {
        uint32_t lo2 = lo, hi2 = hi;
        asm("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\tv_permlane16_swap_b32 %2, %3\n\ts_nop 1"
            : "+v"(lo), "+v"(lo2), "+v"(hi), "+v"(hi2));
        const uint64_t a = ((uint64_t)hi << 32) | lo, b = ((uint64_t)hi2 << 32) | lo2;
        const uint64_t m = a < b ? a : b;
        lo = (uint32_t)m; hi = (uint32_t)(m >> 32);
    }
#define RAIRS_MIN_STEP(XOR_)                                                                      \
    {                                                                                             \
        const uint32_t plo = __builtin_bit_cast(uint32_t, XOR_(__builtin_bit_cast(float, lo)));   \
        const uint32_t phi = __builtin_bit_cast(uint32_t, XOR_(__builtin_bit_cast(float, hi)));   \
        const uint64_t a = ((uint64_t)hi << 32) | lo, b = ((uint64_t)phi << 32) | plo;            \
        const uint64_t m = a < b ? a : b;                                                         \
        lo = (uint32_t)m; hi = (uint32_t)(m >> 32);                                               \
    }
    RAIRS_MIN_STEP(lane_xor8)
    RAIRS_MIN_STEP(lane_xor4)
    RAIRS_MIN_STEP(lane_xor2)
    RAIRS_MIN_STEP(lane_xor1)
#undef RAIRS_MIN_STEP
    return ((uint64_t)hi << 32) | lo;
}

// The k <= 64 smallest of n distinct 64-bit keys in a wave's own LDS region (all-ones entries are
// empty), ascending: k rounds of "take the minimum and strike it out"; lane r returns the r-th
// smallest (all ones beyond the entries there are).  For the few results that refine keeps (k of
// bigK) this is well under half of a full sort's instructions.  The keys are overwritten.
static __device__ __forceinline__ uint64_t wave_take_smallest(uint64_t *keys, int n, int k, int lane)
{
    uint64_t res = ~0ull;
    for (int r = 0; r < k; r++) {
        uint64_t mine = ~0ull;
        for (int i = lane; i < n; i += 64) {
            const uint64_t x = keys[i];
            mine = x < mine ? x : mine;
        }
        const uint64_t best = wave_min_u64(mine);
        if (best != ~0ull)
            for (int i = lane; i < n; i += 64)
                if (keys[i] == best) keys[i] = ~0ull;     // keys are distinct: one lane, one slot
        if (lane == r) res = best;
        wave_lds_sync();
    }
    return res;
}

// Totals of four rows of 64 per-lane partial sums, each folded across the lanes at strides
// 32, 16, 8, 4, 2, 1 with own + partner at every stride -- the butterfly whose result is the same
// in every lane -- with 7 lane exchanges instead of 24: after stride 32 lanes 0..31 go on with
// rows 0 and 1 and lanes 32..63 with rows 2 and 3, after stride 16 each group of 16 lanes has one
// row.  Returns, in every lane of group u = lane >> 4, the total of row u, bit-identical to the
// separate butterflies (a + b = b + a).  All exchanges are register moves: swapping the upper half
// of row 0's register with the lower half of row 2's leaves, in every lane, the two values that
// the stride-32 step adds (likewise rows 1 and 3, and at stride 16 the odd 16-lane rows of one
// register against the even ones of the other); measured on 10,000-query batches the refine
// kernel and the coarse re-score were bound by these exchanges when they went through LDS.
static __device__ __forceinline__ float fold_four_rows(float p0, float p1, float p2, float p3, int lane)
{
    (void)lane;
    // (the swaps are written as instructions: through the compiler's builtin, which returns both
    // registers as a pair, this kernel family was compiled to add one register to itself)
    // (and keep the idle issue slots that the compiler puts around its own: two between a vector
    // write of an operand and the swap, two before the swapped registers are read)
    asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_permlane32_swap_b32 %2, %3\n\ts_nop 1"
        : "+v"(p0), "+v"(p2), "+v"(p1), "+v"(p3));
    float a = p0 + p2, b = p1 + p3;
    asm("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
    float c = a + b;
    c = c + lane_xor8(c);
    c = c + lane_xor4(c);
    c = c + lane_xor2(c);
    c = c + lane_xor1(c);
    return c;
}

