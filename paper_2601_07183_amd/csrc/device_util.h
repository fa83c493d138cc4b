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

// Totals of four rows of 64 per-lane partial sums, each folded across the lanes at strides
// 32, 16, 8, 4, 2, 1 with own + partner at every stride -- the butterfly whose result is the same
// in every lane -- with 7 lane exchanges instead of 24: after stride 32 lanes 0..31 go on with
// rows 0 and 1 and lanes 32..63 with rows 2 and 3, after stride 16 each group of 16 lanes has one
// row.  Returns, in every lane of group u = lane >> 4, the total of row u, bit-identical to the
// separate butterflies (a + b = b + a).
static __device__ __forceinline__ float fold_four_rows(float p0, float p1, float p2, float p3, int lane)
{
    const bool h32 = (lane & 32) != 0;
    float a = h32 ? p2 : p0, b = h32 ? p3 : p1;                  // rows this half keeps
    const float sa = h32 ? p0 : p2, sb = h32 ? p1 : p3;          // rows the other half keeps
    a = a + __shfl_xor(sa, 32);
    b = b + __shfl_xor(sb, 32);
    const bool h16 = (lane & 16) != 0;
    float c = h16 ? b : a;
    const float sc = h16 ? a : b;
    c = c + __shfl_xor(sc, 16);
    c = c + __shfl_xor(c, 8);
    c = c + __shfl_xor(c, 4);
    c = c + __shfl_xor(c, 2);
    c = c + __shfl_xor(c, 1);
    return c;
}

