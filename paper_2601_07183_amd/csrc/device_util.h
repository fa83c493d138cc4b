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
