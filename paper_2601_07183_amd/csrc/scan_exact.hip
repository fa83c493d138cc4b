// Exact SEIL scan with a bounded top-bigK queue, one workgroup per query (SeilSearch, Alg. 5,
// with rqueue).  Used as the whole scan for table shapes the MFMA kernel is not built for and as
// the fallback for queries whose survivor buffer overflowed.  A helper of the MFMA scan lives
// here too: the bound from a sample of each query's first list.
//
// listVisited is replaced by the order-free equivalent over the query's probe bitmap P:
//   reference entry (owner i) of list j is scanned  iff  i not in P;
//   own shared blocks are always scanned;
//   a miscellaneous item of list L tagged with other list o is dropped  iff  o in P and o < L.
// (Alg. 5 visits lists in ascending id and owners have the smaller id, hence "visited" == "in P
// and smaller".)  Every (query, list) pair is then independent of all others.
//
// rqueue: survivors with key (score << 32 | id) below the current bound are appended to an LDS
// buffer; when it fills, the buffer is sorted, cut to bigK entries and the bound tightened.
#include "device_util.h"
#include "select_wg.h"

#define SCAN_CAP 2048
#define SCAN_ROUND 16     // blocks per workgroup between buffer checks (4 per wave)

struct ScanShared {
    uint64_t buf[SCAN_CAP];
    uint32_t bm[RAIRS_MAX_NLIST / 32];
    uint8_t lut[RAIRS_MAX_M * 16];
    uint64_t tau;
    uint32_t cnt;
    unsigned long long dco;
};

static __device__ __forceinline__ void scan_prune(ScanShared &sh, int refine_k)
{
    // all threads arrive here together
    __syncthreads();
    int n = (int)sh.cnt;
    int n2 = next_pow2(n < 2 ? 2 : n);
    for (int i = n + threadIdx.x; i < n2; i += WG) sh.buf[i] = ~0ull;
    __syncthreads();
    bitonic_sort_lds(sh.buf, n2);
    if (threadIdx.x == 0) {
        int keep = n < refine_k ? n : refine_k;
        sh.cnt = (uint32_t)keep;
        sh.tau = keep == refine_k ? sh.buf[refine_k - 1] : ~0ull;
    }
    __syncthreads();
}

static __device__ __forceinline__ uint32_t scan_block_acc(const IndexView &v, const ScanShared &sh,
                                                          int64_t blk, int lane)
{
    const int g = lane >> 5;
    const uint32_t *cp = v.codes + (size_t)blk * v.nd * 64 + lane;
    uint32_t part = 0;
    for (int w = 0; w < v.nd; w++) {
        uint32_t c = cp[(size_t)w * 64];
        const int tmax = v.T - 8 * w < 8 ? v.T - 8 * w : 8;
        for (int n = 0; n < tmax; n++) {
            int m = 2 * (8 * w + n) + g;
            part += sh.lut[m * 16 + ((c >> (4 * n)) & 15u)];
        }
    }
    return part + (uint32_t)__shfl_xor((int)part, 32);
}

static __device__ __forceinline__ void scan_exact_query(const IndexView &v, const ExactScanArgs &a, ScanShared &sh,
                                                        const int64_t qi)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nprobe = a.nprobe, refine_k = a.refine_k;
    for (int i = tid; i < v.M * 16; i += WG) sh.lut[i] = a.lut[(size_t)qi * v.M * 16 + i];
    for (int i = tid; i < a.bmwords; i += WG) sh.bm[i] = a.bitmap[(size_t)qi * a.bmwords + i];
    if (tid == 0) { sh.tau = ~0ull; sh.cnt = 0; sh.dco = 0; }
    __syncthreads();

    unsigned long long my_dco = 0;
    for (int p = 0; p < nprobe; p++) {
        const int L = a.probe_ids[(size_t)qi * nprobe + p];
        if (L < 0 || L >= v.nlist) continue;              // caller-supplied ids: never index with them unchecked
        const ListEntry le = v.lists[L];
        // segment -1: the list's own blocks; segments 0..ref_cnt-1: its reference entries
        for (int seg = -1; seg < le.ref_cnt; seg++) {
            int64_t begin;
            int cnt, misc_from;
            if (seg < 0) {
                begin = le.blk_begin;
                cnt = le.shared_cnt + le.misc_cnt;
                misc_from = le.shared_cnt;
            } else {
                const RefEntry re = v.refs[le.ref_begin + seg];
                if ((sh.bm[re.owner >> 5] >> (re.owner & 31)) & 1u) continue;   // scanned via owner
                begin = re.blk_begin;
                cnt = re.nblocks;
                misc_from = cnt;
            }
            for (int base = 0; base < cnt; base += SCAN_ROUND) {
                for (int j = 0; j < SCAN_ROUND / 4; j++) {
                    int b = base + j * 4 + wave;
                    if (b < cnt) {
                        int64_t blk = begin + b;
                        uint32_t acc = scan_block_acc(v, sh, blk, lane);
                        bool push = false;
                        uint32_t id = RAIRS_EMPTY_ID;
                        if (lane < 32) {
                            id = v.ids[(size_t)blk * 32 + lane];
                            push = id != RAIRS_EMPTY_ID;
                        }
                        my_dco += (unsigned long long)__popcll(__ballot(push));
                        if (push && b >= misc_from) {
                            int o = v.other[(size_t)blk * 32 + lane];
                            if (o >= 0 && o < L && ((sh.bm[o >> 5] >> (o & 31)) & 1u)) push = false;
                        }
                        if (push) {
                            uint64_t key = ((uint64_t)acc << 32) | id;
                            if (key < sh.tau) {
                                uint32_t pos = atomicAdd(&sh.cnt, 1u);
                                sh.buf[pos] = key;
                            }
                        }
                    }
                }
                // snapshot the fill level between two barriers so that every thread takes the
                // same branch (other waves resume pushing right after the second barrier)
                __syncthreads();
                const uint32_t fill = sh.cnt;
                __syncthreads();
                if (fill > SCAN_CAP - SCAN_ROUND * 32) scan_prune(sh, refine_k);
            }
        }
    }
    scan_prune(sh, refine_k);
    const int n = (int)sh.cnt;
    for (int i = tid; i < refine_k; i += WG) {
        uint64_t key = sh.buf[i];
        bool ok = i < n;
        a.cand_ids[(size_t)qi * refine_k + i] = ok ? (int64_t)(uint32_t)key : -1;
        if (a.cand_score) a.cand_score[(size_t)qi * refine_k + i] = ok ? (int32_t)(key >> 32) : -1;
    }
    if (a.dco) {
        if (lane == 0 && my_dco) atomicAdd(&sh.dco, my_dco);
        __syncthreads();
        if (tid == 0) a.dco[qi] = (int64_t)sh.dco;
    }
}

__global__ __launch_bounds__(WG) void scan_exact_kernel(IndexView v, ExactScanArgs a)
{
    __shared__ ScanShared sh;
    const int64_t qi = blockIdx.x;
    if (a.only_flagged && a.only_flagged[qi] == 0) return;
    scan_exact_query(v, a, sh, qi);
}

// The two repairs behind the wave-wide select of the MFMA scan, in one launch: the workgroup-wide
// select for the queries on the first list (more survivors than a wave holds), then the exact scan
// for the queries on the second (overflowed buffers).  Both lists are normally empty, and then a
// handful of workgroups read two counters and exit, instead of one workgroup per query of the
// batch looking at its flag, twice.  No query is on both lists, and neither repair reads what the
// other writes, so the workgroups need no order between the two loops.
__global__ __launch_bounds__(WG) void scan_repair_kernel(IndexView v, MfmaScanArgs ma, int wave_cap, ExactScanArgs a)
{
    __shared__ union { SelectShared sel; ScanShared scan; } sh;
    const uint32_t nwork = ma.work[0];
    for (uint32_t i = blockIdx.x; i < nwork; i += gridDim.x)
        select_query_wg(v, ma, wave_cap, (int64_t)ma.work[1 + i], sh.sel);
    const uint32_t n = a.redo[0];
    for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
        scan_exact_query(v, a, sh.scan, (int64_t)a.redo[1 + i]);
        __syncthreads();                                // the shared state is set up again for the next query
    }
}

int rairs_launch_scan_exact(const IndexView &v, const ExactScanArgs &a, int64_t nq, hipStream_t s)
{
    hipLaunchKernelGGL(scan_exact_kernel, dim3((unsigned)nq), dim3(WG), 0, s, v, a);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

int rairs_launch_scan_repair(const IndexView &v, const MfmaScanArgs &ma, const ExactScanArgs &a, hipStream_t s)
{
    if (!a.redo || !ma.work) {
        rairs_set_error("scan repair without its two query lists");
        return RAIRS_EINVAL;
    }
    hipLaunchKernelGGL(scan_repair_kernel, dim3((unsigned)(ma.nq < 1024 ? ma.nq : 1024)), dim3(WG), 0, s, v, ma,
                       rairs_select_wave_cap(ma.refine_k), a);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

// ---- bound from a sample ------------------------------------------------------------------------
//
// bound[q] = bigK-th smallest score among the items of the first `sample_blocks` own blocks of the
// query's first probed list (0xFFFF when they hold fewer than bigK items); tau[q] = the range of
// the query's score histogram (the same value when it exists).  Every item there is
// either an entry of the query's candidate queue or, when the duplicate rule drops it, the twin of
// an entry with the same code that is queued from its other list (SEIL keeps the remainder of a
// cell in the miscellaneous areas of both lists, Section 5.1); so at least bigK entries of the
// queue score <= tau.  One wave per query; the sample's scores sit in LDS and the rank is found by
// bisection on the 16 score bits.
// Scores of one block for this lane: `part` sums the table entries of the lane's half of the
// sub-quantizer pairs; ND code dwords with 8 four-bit codes each.  No branch per lookup, so the
// LDS reads of a block are all in flight together.
template <int ND>
static __device__ __forceinline__ uint32_t sample_block_part(const uint8_t *lq, const uint32_t (&c)[ND], int g)
{
    uint32_t part = 0;
#pragma unroll
    for (int w = 0; w < ND; w++)
#pragma unroll
        for (int n = 0; n < 8; n++) part += lq[(2 * (8 * w + n) + g) * 16 + ((c[w] >> (4 * n)) & 15u)];
    return part;
}

// ND > 0: exactly ND code dwords per block and lane (T = 8 ND), blocks taken 4 or 2 at a time with
// all their dwords fetched before the first lookup.  ND == 0: any T, dwords in groups of four.
template <int ND>
__global__ __launch_bounds__(WG) void sample_bound_kernel(IndexView v, const uint8_t *__restrict__ lut,
                                                          const int32_t *__restrict__ probe_ids,
                                                          int nprobe, int refine_k, int sample_blocks,
                                                          int64_t nq, int32_t *__restrict__ tau,
                                                          int32_t *__restrict__ bound)
{
    extern __shared__ __align__(16) uint8_t sample_lds[];  // per wave: M*16 table bytes, then sample_blocks*32 scores
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
    const int64_t qi0 = (int64_t)blockIdx.x * (WG / 64) + wave;
    const int64_t qi = qi0 < nq ? qi0 : nq - 1;          // surplus waves redo the last query
    const size_t per_wave = (size_t)v.M * 16 + (size_t)sample_blocks * 64;
    uint8_t *lq = sample_lds + wave * per_wave;
    uint16_t *sc = (uint16_t *)(lq + (size_t)v.M * 16);
    {
        const uint4 *src = (const uint4 *)(lut + (size_t)qi * v.M * 16);
        uint4 *dst = (uint4 *)lq;
        for (int i = lane; i < v.M; i += 64) dst[i] = src[i];
    }
    __syncthreads();
    const int L = probe_ids[(size_t)qi * nprobe];
    int cnt = 0;
    int64_t begin = 0;
    if (L >= 0 && L < v.nlist) {
        const ListEntry le = v.lists[L];
        begin = le.blk_begin;
        cnt = le.shared_cnt + le.misc_cnt;
        cnt = cnt < sample_blocks ? cnt : sample_blocks;
    }
    uint32_t nvalid = 0;
    // slots without an item (the tail of the list's last block, invalidated items) do not count
#define SAMPLE_STORE(blk_, part_)                                                              \
    do {                                                                                       \
        const uint32_t acc_ = (part_) + (uint32_t)__shfl_xor((int)(part_), 32);                \
        const bool valid_ = lane < 32 && (blk_) < cnt && ((v.vmask[begin + (blk_)] >> lane) & 1u); \
        if (lane < 32 && (blk_) < cnt) sc[(blk_) * 32 + lane] = valid_ ? (uint16_t)acc_ : (uint16_t)0xFFFFu; \
        nvalid += (uint32_t)__popcll(__ballot(valid_));                                        \
    } while (0)
    if (ND > 0) {
        constexpr int NDS = ND > 0 ? ND : 1, U = NDS <= 4 ? 4 : 2;
        for (int b0 = 0; b0 < cnt; b0 += U) {
            uint32_t c[U][NDS];
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int64_t blk = begin + (b0 + u < cnt ? b0 + u : cnt - 1);
                const uint32_t *cp = v.codes + (size_t)blk * NDS * 64 + lane;
#pragma unroll
                for (int w = 0; w < NDS; w++) c[u][w] = cp[w * 64];
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                const uint32_t part = sample_block_part<NDS>(lq, c[u], g);
                SAMPLE_STORE(b0 + u, part);
            }
        }
    } else {
        for (int b = 0; b < cnt; b++) {
            const uint32_t *cp = v.codes + (size_t)(begin + b) * v.nd * 64 + lane;
            uint32_t part = 0;
            for (int w0 = 0; w0 < v.nd; w0 += 4) {
                uint32_t c[4];
#pragma unroll
                for (int w = 0; w < 4; w++) c[w] = cp[(size_t)(w0 + w < v.nd ? w0 + w : v.nd - 1) * 64];
#pragma unroll
                for (int w = 0; w < 4; w++) {
                    const int t0 = 8 * (w0 + w);            // first code pair of this dword
                    if (t0 + 8 <= v.T) {                    // uniform: a full dword
#pragma unroll
                        for (int n = 0; n < 8; n++)
                            part += lq[(2 * (t0 + n) + g) * 16 + ((c[w] >> (4 * n)) & 15u)];
                    } else {
                        for (int n = 0; t0 + n < v.T; n++)
                            part += lq[(2 * (t0 + n) + g) * 16 + ((c[w] >> (4 * n)) & 15u)];
                    }
                }
            }
            SAMPLE_STORE(b, part);
        }
    }
#undef SAMPLE_STORE
    __syncthreads();
    uint32_t t = 0xFFFFu;
    if (nvalid >= (uint32_t)refine_k) {
        // largest t with fewer than bigK scores below it == the bigK-th smallest score
        // (empty slots hold 0xFFFF, which no candidate t exceeds)
        // The first 512 scores stay in registers; counting is a ballot and a scalar population
        // count per 64 scores, so no lane waits for another.
        const int n = cnt * 32;
        uint32_t mine[8];
#pragma unroll
        for (int u = 0; u < 8; u++) mine[u] = lane + 64 * u < n ? (uint32_t)sc[lane + 64 * u] : 0xFFFFu;
        t = 0;
        for (int bit = 15; bit >= 0; bit--) {
            const uint32_t cand = t | (1u << bit);
            uint32_t below = 0;                          // wave-uniform
#pragma unroll
            for (int u = 0; u < 8; u++) below += (uint32_t)__popcll(__ballot(mine[u] < cand));
            for (int e0 = 512; e0 < n; e0 += 64)
                below += (uint32_t)__popcll(__ballot(e0 + lane < n && sc[e0 + lane] < cand));
            if (below < (uint32_t)refine_k) t = cand;
        }
    }
    // Range of the query's score histogram: tau when there is one; else (the sample held fewer than
    // bigK items, so there is no bound yet) twice the largest sampled score -- a guess that only
    // sets the width of the bins, scores beyond it share the last bin, which never yields a bound.
    uint32_t range = t;
    if (t == 0xFFFFu) {
        uint32_t smax = 0;
        for (int e = lane; e < cnt * 32; e += 64) {
            const uint32_t x = sc[e];
            if (x != 0xFFFFu && x > smax) smax = x;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)smax, off);
            smax = o > smax ? o : smax;
        }
        const uint32_t full = 255u * (uint32_t)v.M;
        range = nvalid > 0 && 2u * smax + 64u < full ? 2u * smax + 64u : full;
    }
    if (lane == 0 && qi0 < nq) {
        tau[qi] = (int32_t)range;
        if (bound) bound[qi] = (int32_t)t;
    }
}

// Bound of every query from the scores the matrix-core sample kernel wrote, pre[q][sample_blocks *
// 32] (0xFFFF: no item): the bigK-th smallest of them; same outputs as sample_bound_kernel.  One
// wave per query holds the query's scores in registers (WPL words of two scores per lane) and
// finds the value bit by bit: t becomes the largest value with fewer than bigK scores below it.
// With fewer than bigK scores no candidate ever has bigK below it and t ends as 0xFFFF.  (A radix
// select with a histogram in LDS was two and a half times slower: the scores of a query crowd into
// a few bins, and LDS atomics on one address are served one at a time.)
template <int WPL>
__global__ __launch_bounds__(WG) void sample_rank_kernel(IndexView v, const int32_t *__restrict__ probe_ids,
                                                         int nprobe, int refine_k, int sample_blocks,
                                                         int64_t nq, const uint16_t *__restrict__ pre,
                                                         int32_t *__restrict__ tau,
                                                         int32_t *__restrict__ bound,
                                                         const int32_t *__restrict__ check_ids, int check_n)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t qi = (int64_t)blockIdx.x * (WG / 64) + wave;
    if (qi >= nq) return;
    int L = probe_ids[(size_t)qi * nprobe];
    if (check_ids) {
        // the sample was taken from a list chosen before the probe lists existed: its scores bound
        // the query's candidates only if that list is one of them (else: no bound for this query)
        bool found = false;
        for (int i = lane; i < check_n; i += 64) found |= check_ids[(size_t)qi * check_n + i] == L;
        if (__ballot(found) == 0ull) L = -1;
    }
    int cnt = 0;
    if (L >= 0 && L < v.nlist) {
        const ListEntry le = v.lists[L];
        cnt = le.shared_cnt + le.misc_cnt;
        cnt = cnt < sample_blocks ? cnt : sample_blocks;
    }
    const int nw = cnt * 16;                             // score pairs
    const uint32_t *row = (const uint32_t *)(pre + (size_t)qi * sample_blocks * 32);
    // Scores are below 0x7FFF (255 M with M <= 64, checked at launch); an empty slot counts as
    // 0x7FFF, above all of them.  With both values below 2^15, (a - c) mod 2^16 = a - c + 2^16 [a < c],
    // so the number of scores below c is (sum of the 16-bit differences - sum of the scores + N c)
    // / 2^16: one packed subtraction and one two-way dot product per pair of scores, and one sum
    // over the wave per candidate.
    typedef unsigned short us2 __attribute__((ext_vector_type(2)));
    us2 x[WPL];
    uint32_t sum_a = 0;
    const us2 one2 = {1, 1};
#pragma unroll
    for (int u = 0; u < WPL; u++) {
        const int e = 64 * u + lane;
        const uint32_t w = e < nw ? row[e] : 0xFFFFFFFFu;
        const uint32_t a = w & 0xFFFFu, b = w >> 16;
        x[u] = (us2){(unsigned short)(a < 0x7FFFu ? a : 0x7FFFu), (unsigned short)(b < 0x7FFFu ? b : 0x7FFFu)};
        sum_a = __builtin_amdgcn_udot2(x[u], one2, sum_a, false);
    }
    sum_a = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_sum_u32(sum_a));
    const uint32_t n_all = 2u * 64u * WPL;
    uint32_t t = 0;
    for (int bit = 14; bit >= 0; bit--) {
        const uint32_t cand = t | (1u << bit);
        const us2 c2 = {(unsigned short)cand, (unsigned short)cand};
        uint32_t sum_d = 0;
#pragma unroll
        for (int u = 0; u < WPL; u++) sum_d = __builtin_amdgcn_udot2(x[u] - c2, one2, sum_d, false);
        sum_d = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_sum_u32(sum_d));
        const uint32_t below = (sum_d - sum_a + n_all * cand) >> 16;
        if (below < (uint32_t)refine_k) t = cand;
    }
    if (t == 0x7FFFu) t = 0xFFFFu;                       // fewer than bigK scores
    // range of the score histogram, as in sample_bound_kernel
    uint32_t range = t;
    if (t == 0xFFFFu) {                                  // uniform
        uint32_t nvalid = 0, smax = 0;
#pragma unroll
        for (int u = 0; u < WPL; u++) {
            const uint32_t a = x[u].x, b = x[u].y;
            if (a != 0x7FFFu) { nvalid++; smax = a > smax ? a : smax; }
            if (b != 0x7FFFu) { nvalid++; smax = b > smax ? b : smax; }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            nvalid += (uint32_t)__shfl_xor((int)nvalid, off);
            const uint32_t o = (uint32_t)__shfl_xor((int)smax, off);
            smax = o > smax ? o : smax;
        }
        const uint32_t full = 255u * (uint32_t)v.M;
        range = nvalid > 0 && 2u * smax + 64u < full ? 2u * smax + 64u : full;
    }
    if (lane == 0) {
        tau[qi] = (int32_t)range;
        if (bound) bound[qi] = (int32_t)t;
    }
}

int rairs_launch_sample_rank(const IndexView &v, const int32_t *probe_ids, int nprobe, int refine_k,
                             int sample_blocks, int64_t nq, const uint16_t *pre, int32_t *tau,
                             int32_t *bound, hipStream_t s, const int32_t *check_ids, int check_n)
{
    if (sample_blocks < 1 || sample_blocks > RAIRS_SAMPLE_MAX_BLOCKS || 255 * v.M >= 0x7FFF) {
        rairs_set_error("sample of %d blocks with M = %d: the rank kernel takes 1..%d blocks and scores below 32767",
                        sample_blocks, v.M, RAIRS_SAMPLE_MAX_BLOCKS);
        return RAIRS_EINVAL;
    }
    static_assert(RAIRS_SAMPLE_MAX_BLOCKS * 16 <= 32 * 64, "a lane holds at most 32 score pairs");
    const dim3 grid((unsigned)((nq + WG / 64 - 1) / (WG / 64)));
    const int wpl = (sample_blocks * 16 + 63) / 64;      // score pairs per lane
#define RANK_LAUNCH(W_)                                                                           \
    hipLaunchKernelGGL(sample_rank_kernel<W_>, grid, dim3(WG), 0, s, v, probe_ids, nprobe, refine_k, \
                       sample_blocks, nq, pre, tau, bound, check_ids, check_n)
    if (wpl <= 4) RANK_LAUNCH(4);
    else if (wpl <= 8) RANK_LAUNCH(8);
    else if (wpl <= 12) RANK_LAUNCH(12);
    else if (wpl <= 16) RANK_LAUNCH(16);
    else if (wpl <= 24) RANK_LAUNCH(24);
    else RANK_LAUNCH(32);
#undef RANK_LAUNCH
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

int rairs_launch_sample_bound(const IndexView &v, const uint8_t *lut, const int32_t *probe_ids,
                              int nprobe, int refine_k, int sample_blocks, int64_t nq, int32_t *tau,
                              int32_t *bound, hipStream_t s)
{
    if (sample_blocks > RAIRS_SAMPLE_MAX_BLOCKS) sample_blocks = RAIRS_SAMPLE_MAX_BLOCKS;
    if (sample_blocks < 1) sample_blocks = 1;
    const size_t lds = (size_t)(WG / 64) * ((size_t)v.M * 16 + (size_t)sample_blocks * 64);
    const dim3 grid((unsigned)((nq + WG / 64 - 1) / (WG / 64)));
#define SAMPLE_LAUNCH(ND_)                                                                        \
    hipLaunchKernelGGL(sample_bound_kernel<ND_>, grid, dim3(WG), lds, s, v, lut, probe_ids, nprobe, \
                       refine_k, sample_blocks, nq, tau, bound)
    const int nd = v.T % 8 == 0 ? v.nd : 0;
    switch (nd) {
    case 1: SAMPLE_LAUNCH(1); break;
    case 2: SAMPLE_LAUNCH(2); break;
    case 3: SAMPLE_LAUNCH(3); break;
    case 4: SAMPLE_LAUNCH(4); break;
    case 6: SAMPLE_LAUNCH(6); break;
    case 8: SAMPLE_LAUNCH(8); break;
    default: SAMPLE_LAUNCH(0); break;
    }
#undef SAMPLE_LAUNCH
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}
