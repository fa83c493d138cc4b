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

#define SURV_CAP_MAX 4096   // survivor buffer entries per query (the workgroup-wide select sorts them in LDS)
#define SELW_CAP_MAX 1024   // most entries per query that the wave-wide select takes
// the wave-wide select's room per query: four times bigK, within [256, SELW_CAP_MAX]
static inline int rairs_select_wave_cap(int refine_k)
{
    const int cap = next_pow2(4 * refine_k);
    return cap < 256 ? 256 : (cap > SELW_CAP_MAX ? SELW_CAP_MAX : cap);
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

// Sum of the 64 lanes' values, in every lane (register moves only, as in wave_min_u64).
static __device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x)
{
    {
        uint32_t x2 = x;
        asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(x), "+v"(x2));
        x += x2;
    }
    {
        uint32_t x2 = x;
        asm("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(x), "+v"(x2));
        x += x2;
    }
#define RAIRS_SUM_STEP(XOR_) x += __builtin_bit_cast(uint32_t, XOR_(__builtin_bit_cast(float, x)));
    RAIRS_SUM_STEP(lane_xor8)
    RAIRS_SUM_STEP(lane_xor4)
    RAIRS_SUM_STEP(lane_xor2)
    RAIRS_SUM_STEP(lane_xor1)
#undef RAIRS_SUM_STEP
    return x;
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

// The same selection for n <= 128 keys and few results, by rank instead of k rounds of a wave-wide
// minimum: every lane takes its (up to) two keys into registers; the k-th smallest upper word is
// found bit by bit (the largest t with fewer than k upper words below it); the m >= k entries up to
// it (more than k only when upper words tie there) are packed into keys[0..m) and lane r < m counts
// how many of them are below its own: that is its key's place in the order.  Returns false, with the
// keys untouched, when more than 64 entries tie (the caller takes another route); else lane r < m
// holds a key and its rank, and every rank 0 .. m - 1 is held by exactly one lane.
static __device__ __forceinline__ bool wave_rank_smallest(uint64_t *keys, int n, int k, int lane,
                                                          uint64_t *key_out, int *rank_out, int *m_out)
{
    const uint64_t k0 = lane < n ? keys[lane] : ~0ull, k1 = lane + 64 < n ? keys[lane + 64] : ~0ull;
    const uint32_t h0 = (uint32_t)(k0 >> 32), h1 = (uint32_t)(k1 >> 32);
    uint32_t cut = 0;
    for (int bit = 31; bit >= 0; bit--) {
        const uint32_t cand = cut | (1u << bit);
        const uint32_t below = (uint32_t)__popcll(__ballot(h0 < cand)) + (uint32_t)__popcll(__ballot(h1 < cand));
        if (below < (uint32_t)k) cut = cand;
    }
    const bool in0 = k0 != ~0ull && h0 <= cut, in1 = k1 != ~0ull && h1 <= cut;
    const unsigned long long b0 = __ballot(in0), b1 = __ballot(in1);
    const int m0 = __popcll(b0), m = m0 + __popcll(b1);
    if (m > 64) return false;
    const unsigned long long lt = (1ull << lane) - 1ull;
    wave_lds_sync();                                    // every lane has read its keys
    if (in0) keys[__popcll(b0 & lt)] = k0;
    if (in1) keys[m0 + __popcll(b1 & lt)] = k1;
    wave_lds_sync();
    const uint64_t mine = lane < m ? keys[lane] : ~0ull;
    int rank = 0;
    for (int j = 0; j < m; j++) {                       // one address for the wave: a broadcast
        const uint64_t other = keys[j];
        rank += other < mine || (other == mine && j < lane) ? 1 : 0;    // (equal keys: in the order held)
    }
    *key_out = mine;
    *rank_out = rank;
    *m_out = m;
    return true;
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

