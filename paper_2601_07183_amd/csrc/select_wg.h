// Workgroup-wide select of a query's survivors, for the queries that select_wave_kernel leaves on
// its list (more survivors than a wave holds): resolve the survivors and keep the bigK smallest
// (score, id).  A two-pass radix select on the 16-bit score finds the score of the bigK-th
// survivor; only entries up to that score are sorted.  (Overflowed buffers are not on this list:
// the wave kernel puts them on the list of the exact redo.)
#pragma once
#include "device_util.h"

struct SelectShared {
    uint64_t keys[SURV_CAP_MAX];
    uint32_t hist[256];
    uint32_t prefix, need, kept;
};

// All threads of the workgroup call this together; the shared state may be reused on return.
static __device__ __forceinline__ void select_query_wg(const IndexView &v, const MfmaScanArgs &a, int wave_cap,
                                                        int64_t q, SelectShared &sh)
{
    uint64_t *keys = sh.keys;
    uint32_t *hist = sh.hist;
    const int tid = threadIdx.x;
    const uint32_t n = a.surv_cnt[q];
    if (n <= (uint32_t)wave_cap || n > (uint32_t)a.surv_cap || *a.log_overflow != 0u) return;   // (uniform; not on the list)
    if (tid == 0) a.flags[q] = 0;
    for (int i = tid; i < (int)n; i += WG) {
        uint64_t key = ~0ull;
        const uint64_t e = a.surv_buf[(size_t)q * a.surv_cap + i];
        const uint32_t slot = (uint32_t)e, score = (uint32_t)(e >> 48), L = (uint32_t)v.blk_list[slot >> 5];
        const uint2 it = v.idtag[slot];
        const uint32_t id = it.x;
        const int o = (int)it.y;
        bool keep = id != RAIRS_EMPTY_ID;
        if (keep && o >= 0 && (uint32_t)o < L) {
            // RemoveVectorIfVisited: the item was already taken from list o
            const uint32_t wbits = a.bitmap[(size_t)q * a.bmwords + (o >> 5)];
            if ((wbits >> (o & 31)) & 1u) keep = false;
        }
        if (keep) key = ((uint64_t)score << 32) | id;
        keys[i] = key;
    }
    // score of the bigK-th smallest kept key: radix select, high byte then low byte
    uint32_t prefix = 0, need = (uint32_t)a.refine_k;
    bool all = false;                       // fewer than bigK kept: everything is sorted
    for (int pass = 0; pass < 2 && !all; pass++) {
        const int shift = pass == 0 ? 8 : 0;
        hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < (int)n; i += WG) {
            const uint64_t key = keys[i];
            if (key != ~0ull) {
                const uint32_t sc = (uint32_t)(key >> 32);
                if (pass == 0 || (sc >> 8) == prefix) atomicAdd(&hist[(sc >> shift) & 255u], 1u);
            }
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t cum = 0;
            sh.need = 0xFFFFFFFFu;
            for (int b = 0; b < 256; b++) {
                if (cum + hist[b] >= need) { sh.prefix = (uint32_t)b; sh.need = need - cum; break; }
                cum += hist[b];
            }
        }
        __syncthreads();
        if (sh.need == 0xFFFFFFFFu) all = true;
        else { prefix = pass == 0 ? sh.prefix : ((prefix << 8) | sh.prefix); need = sh.need; }
        __syncthreads();
    }
    const uint32_t cut = all ? 0xFFFFu : prefix;          // keep scores <= cut
    // compact the kept keys with score <= cut to the front (order is irrelevant before the sort)
    if (tid == 0) sh.kept = 0;
    __syncthreads();
    uint64_t mine[SURV_CAP_MAX / WG];
    int nm = 0;
    for (int i = tid; i < (int)n; i += WG) {
        const uint64_t key = keys[i];
        if (key != ~0ull && (uint32_t)(key >> 32) <= cut) mine[nm++] = key;
    }
    __syncthreads();
    uint32_t at = nm ? atomicAdd(&sh.kept, (uint32_t)nm) : 0u;
    for (int i = 0; i < nm; i++) keys[at + i] = mine[i];
    __syncthreads();
    const int kept = (int)sh.kept;
    const int n2 = next_pow2(kept < 2 ? 2 : kept);
    for (int i = kept + tid; i < n2; i += WG) keys[i] = ~0ull;
    __syncthreads();
    bitonic_sort_lds(keys, n2);
    for (int i = tid; i < a.refine_k; i += WG) {
        const uint64_t key = i < n2 ? keys[i] : ~0ull;
        const bool ok = key != ~0ull;
        a.cand_ids[(size_t)q * a.refine_k + i] = ok ? (int64_t)(uint32_t)key : -1;
        if (a.cand_score) a.cand_score[(size_t)q * a.refine_k + i] = ok ? (int32_t)(key >> 32) : -1;
    }
    __syncthreads();                        // the keys are the next query's
}
