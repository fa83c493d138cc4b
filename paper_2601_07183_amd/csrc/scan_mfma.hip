// List-major SEIL scan on the matrix cores (SeilSearch of Alg. 5 for the whole query batch, with
// the list-grouped task order of the "cache optimisation for query batch" paragraph of
// Section 5.2 taken to its conclusion: a block is fetched once for 32 queries).
//
// score(query, item) = sum_m lut[query][m][code[item][m]] is a contraction of the lookup tables
// with the one-hot expansion of the codes:  sum_m sum_c lut[q][m][c] * [code[item][m] == c].
// One v_mfma_i32_32x32x32_i8 covers 32 items x 32 queries x 2 subspaces (K = 2 x 16 codewords):
//   A (rows = items):   lane (item, g) holds the 16-byte one-hot of the item's code in subspace
//                       2t+g, built in registers from the packed nibble;
//   B (cols = queries): lane (query, g) holds the 16 table bytes lut[q][2t+g][0..15] as signed
//                       bytes (value - 128; 128 * M is added back after the sum), kept in
//                       registers for the whole tile.
// Integer arithmetic throughout, so the scores equal the plain 16-bit sums bit for bit.
//
// Work is cut into tasks (list L, tile of <= 32 queries probing L, segment of <= 16 blocks);
// waves of a persistent grid draw runs of consecutive tasks from a counter.  The dedup rules are
// the order-free ones of scan_exact.hip.  A score passes when it is <= the query's bound tau;
// survivors go to the query's buffer and are cut to bigK afterwards by select_kernel.
//
// The bound.  tau0 = bigK-th smallest score in the query's first list (exact kernel).  Every
// survivor is also counted in a per-query histogram of RAIRS_HIST_BINS equal score bins over
// [0, tau0] (over [0, 255*M] when the first list had fewer than bigK items).  Survivors are
// distinct members of the query's probed lists, so once bins 0..b hold >= bigK of them, no item
// scoring above the top edge of bin b can be among the bigK best: that edge is a valid, tighter
// bound.  Waves re-derive it whenever they load a tile; a stale view is only looser, never wrong.
#include <limits.h>

#include "device_util.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define GRAB 8              // consecutive tasks drawn at once (keeps a tile's tables in registers)
#define SURV_CAP_MAX 2048   // survivor buffer entries per query (select_kernel sorts them in LDS)

// ---- grouping queries by list ----------------------------------------------------------------

__global__ void lm_zero_kernel(int32_t *lcount, int nlist, uint32_t *next_task)
{
    int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < nlist) lcount[gid] = 0;
    if (gid == 0) *next_task = 0;
}

__global__ void lm_count_kernel(const int32_t *__restrict__ probe_ids, int64_t nq, int nprobe,
                                int p_first, int nlist, int32_t *lcount)
{
    const int np = nprobe - p_first;
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= nq * np) return;
    int64_t q = gid / np;
    int p = p_first + (int)(gid % np);
    int L = probe_ids[q * nprobe + p];
    if (L >= 0 && L < nlist) atomicAdd(&lcount[L], 1);
}

// exclusive prefixes over lists: queries (loff) and tasks (toff); one workgroup of 1024
__global__ __launch_bounds__(1024) void lm_prefix_kernel(IndexView v,
                                                         const int32_t *__restrict__ lcount,
                                                         int32_t *loff, int32_t *lcursor,
                                                         int32_t *toff)
{
    __shared__ int sc[1024], st[1024];
    const int tid = threadIdx.x;
    const int per = (v.nlist + 1023) / 1024;
    const int lo = tid * per < v.nlist ? tid * per : v.nlist;
    const int hi = lo + per < v.nlist ? lo + per : v.nlist;
    int c = 0, t = 0;
    for (int L = lo; L < hi; L++) {
        int n = lcount[L];
        c += n;
        t += ((n + 31) >> 5) * v.lists[L].seg_cnt;
    }
    sc[tid] = c;
    st[tid] = t;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        int x = tid >= off ? sc[tid - off] : 0;
        int y = tid >= off ? st[tid - off] : 0;
        __syncthreads();
        sc[tid] += x;
        st[tid] += y;
        __syncthreads();
    }
    int cb = sc[tid] - c, tb = st[tid] - t;
    for (int L = lo; L < hi; L++) {
        int n = lcount[L];
        loff[L] = cb;
        toff[L] = tb;
        lcursor[L] = 0;
        cb += n;
        tb += ((n + 31) >> 5) * v.lists[L].seg_cnt;
    }
    if (tid == 1023) {
        loff[v.nlist] = sc[1023];
        toff[v.nlist] = st[1023];
    }
}

__global__ void lm_fill_kernel(const int32_t *__restrict__ probe_ids, int64_t nq, int nprobe,
                               int p_first, int nlist, const int32_t *__restrict__ loff,
                               int32_t *lcursor, int32_t *qlist)
{
    const int np = nprobe - p_first;
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= nq * np) return;
    int64_t q = gid / np;
    int p = p_first + (int)(gid % np);
    int L = probe_ids[q * nprobe + p];
    if (L >= 0 && L < nlist) {
        int pos = atomicAdd(&lcursor[L], 1);
        qlist[loff[L] + pos] = (int32_t)q;
    }
}

// ---- the scan ----------------------------------------------------------------------------------

static __device__ __forceinline__ v4i onehot16(uint32_t nib)
{
    // 16-byte one-hot: byte `nib` = 1
    uint32_t sh = 1u << ((nib & 3u) << 3);
    uint32_t w = nib >> 2;
    v4i r;
    r.x = w == 0 ? (int)sh : 0;
    r.y = w == 1 ? (int)sh : 0;
    r.z = w == 2 ? (int)sh : 0;
    r.w = w == 3 ? (int)sh : 0;
    return r;
}

// Bound of one query from its first-list bound tau0 and its survivor histogram.  Lanes (j, 0)
// and (j, 1) hold the same query and split the bins.  Called by all lanes of the wave.
static __device__ __forceinline__ int current_bound(const MfmaScanArgs &a, int qid, uint32_t tau0,
                                                    uint32_t range, int g, int bias)
{
    uint32_t part = 0, cum_here[RAIRS_HIST_BINS / 2];
    if (qid >= 0) {
        const uint4 *hq = (const uint4 *)(a.hist + (size_t)qid * RAIRS_HIST_BINS + g * (RAIRS_HIST_BINS / 2));
#pragma unroll
        for (int i = 0; i < RAIRS_HIST_BINS / 8; i++) {
            uint4 h4 = hq[i];
            part += h4.x; cum_here[4 * i] = part;
            part += h4.y; cum_here[4 * i + 1] = part;
            part += h4.z; cum_here[4 * i + 2] = part;
            part += h4.w; cum_here[4 * i + 3] = part;
        }
    }
    const uint32_t other = (uint32_t)__shfl_xor((int)part, 32);
    const uint32_t before = g ? other : 0u;
    int bfound = RAIRS_HIST_BINS;
    if (qid >= 0) {
#pragma unroll
        for (int i = RAIRS_HIST_BINS / 2 - 1; i >= 0; i--)
            if (before + cum_here[i] >= (uint32_t)a.refine_k) bfound = g * (RAIRS_HIST_BINS / 2) + i;
    }
    const int bo = __shfl_xor(bfound, 32);
    const int b = bfound < bo ? bfound : bo;
    if (qid < 0) return INT_MIN;
    uint32_t tau = tau0;
    if (b < RAIRS_HIST_BINS) {
        // every item counted in bins <= b has score <= this
        uint32_t tb = ((uint32_t)(b + 1) * (range + 1u) - 1u) / RAIRS_HIST_BINS;
        tau = tb < tau ? tb : tau;
    }
    return (int)tau - bias;
}

// A passing (item, query) pair waits in a per-wave LDS queue until 64 or more have gathered;
// then every lane finishes one: id load, duplicate rule, slot in the query's survivor buffer.
// This keeps the global-memory round trips out of the per-block path.
#define STAGE_CAP 192
struct StageQueue {
    uint32_t slot[STAGE_CAP];      // block * 32 + item
    uint32_t score[STAGE_CAP];
    int32_t qid[STAGE_CAP];
    uint32_t lrange[STAGE_CAP];    // score range of the query's histogram
    int32_t list[STAGE_CAP];       // probed list, bit 31 set for items of miscellaneous blocks
};

static __device__ __forceinline__ void stage_flush(const IndexView &v, const MfmaScanArgs &a,
                                                   StageQueue &sq, int n, int lane)
{
    for (int i = lane; i < n; i += 64) {
        const uint32_t slot = sq.slot[i];
        const int qid = sq.qid[i];
        const uint32_t id = v.ids[slot];
        bool push = id != RAIRS_EMPTY_ID;
        const int lm = sq.list[i];
        if (push && lm < 0) {
            const int L = lm & 0x7FFFFFFF;
            const int o = v.other[slot];
            if (o >= 0 && o < L) {
                uint32_t wbits = a.bitmap[(size_t)qid * a.bmwords + (o >> 5)];
                if ((wbits >> (o & 31)) & 1u) push = false;
            }
        }
        if (push) {
            const uint32_t score = sq.score[i];
            uint32_t pos = atomicAdd(&a.surv_cnt[qid], 1u);
            if (pos < (uint32_t)a.surv_cap)
                a.surv_buf[(size_t)qid * a.surv_cap + pos] = ((uint64_t)score << 32) | id;
            atomicAdd(&a.hist[(size_t)qid * RAIRS_HIST_BINS + (score * RAIRS_HIST_BINS) / (sq.lrange[i] + 1u)], 1u);
        }
    }
}

template <int T>
__global__ __launch_bounds__(WG) void scan_mfma_kernel(IndexView v, MfmaScanArgs a)
{
    constexpr int ND = (T + 7) / 8;
    constexpr int M = 2 * T;
    __shared__ StageQueue stage[WG / 64];
    const int lane = threadIdx.x & 63, g = lane >> 5, j = lane & 31;
    StageQueue &sq = stage[threadIdx.x >> 6];
    const uint32_t ntasks = (uint32_t)a.toff[v.nlist];
    const int bias = 128 * M;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;

    v4i B[T];
#pragma unroll
    for (int t = 0; t < T; t++) B[t] = (v4i){0, 0, 0, 0};
    int cur_L = -1, cur_tile = -1, qid = -1;
    uint32_t range = 0, tau0 = 0;
    int nstaged = 0;                                   // wave-uniform fill of the stage queue

    for (;;) {
        uint32_t t0 = 0;
        if (lane == 0) t0 = atomicAdd(a.next_task, (uint32_t)GRAB);
        t0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)t0);
        if (t0 >= ntasks) break;                      // every wave gets here: the counter only grows
        const uint32_t t1 = t0 + GRAB < ntasks ? t0 + GRAB : ntasks;
        // list of task t0: the last L with toff[L] <= t0 (lists without tasks are skipped over)
        int lo = 0, hi = v.nlist;
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if ((uint32_t)a.toff[mid] <= t0) lo = mid; else hi = mid;
        }
        int L = __builtin_amdgcn_readfirstlane(lo);
        uint32_t lend = (uint32_t)__builtin_amdgcn_readfirstlane(a.toff[L + 1]);
        ListEntry le = v.lists[L];
        int rem = (int)(t0 - (uint32_t)a.toff[L]);
        int tile = __builtin_amdgcn_readfirstlane(rem / le.seg_cnt);
        int seg = __builtin_amdgcn_readfirstlane(rem % le.seg_cnt);

        for (uint32_t tt = t0; tt < t1; tt++) {
            if (tt >= lend) {
                do {
                    L++;
                    lend = (uint32_t)__builtin_amdgcn_readfirstlane(a.toff[L + 1]);
                } while (tt >= lend);                 // ends: tt < ntasks = toff[nlist]
                le = v.lists[L];
                tile = 0;
                seg = 0;
            }
            if (L != cur_L || tile != cur_tile) {
                // new tile: query of this lane's column and its tables
                const int base = a.loff[L], n = a.loff[L + 1] - base;
                const int qi = tile * 32 + j;
                qid = qi < n ? a.qlist[base + qi] : -1;
                tau0 = qid >= 0 ? (uint32_t)a.tau[qid] : 0u;
                range = tau0 == 0xFFFFu ? 255u * (uint32_t)M : tau0;
                const uint8_t *lq = a.lut + (size_t)(qid >= 0 ? qid : 0) * (M * 16) + g * 16;
#pragma unroll
                for (int t = 0; t < T; t++) {
                    v4i x = *(const v4i *)(lq + t * 32);
                    x ^= (v4i){(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
                    B[t] = qid >= 0 ? x : (v4i){0, 0, 0, 0};
                }
                cur_L = L;
                cur_tile = tile;
            }
            const SegEntry se = v.segs[le.seg_begin + seg];
            int th = current_bound(a, qid, tau0, range, g, bias);
            if (se.owner >= 0 && qid >= 0) {
                // cell (owner, L) is scored through list `owner` for queries that probe it
                uint32_t wbits = a.bitmap[(size_t)qid * a.bmwords + (se.owner >> 5)];
                if ((wbits >> (se.owner & 31)) & 1u) th = INT_MIN;
            }
            if (__ballot(th != INT_MIN) != 0ull) {
                const uint32_t *cp = v.codes + (size_t)se.blk_begin * ND * 64 + lane;
                uint32_t cn[ND];
#pragma unroll
                for (int w = 0; w < ND; w++) cn[w] = cp[w * 64];
                for (int b = 0; b < se.nblk; b++) {
                    uint32_t c[ND];
#pragma unroll
                    for (int w = 0; w < ND; w++) c[w] = cn[w];
                    if (b + 1 < se.nblk) {             // fetch the next block while this one is scored
#pragma unroll
                        for (int w = 0; w < ND; w++) cn[w] = cp[(size_t)(b + 1) * ND * 64 + w * 64];
                    }
                    v16i acc;
#pragma unroll
                    for (int r = 0; r < 16; r++) acc[r] = 0;
#pragma unroll
                    for (int t = 0; t < T; t++) {
                        uint32_t nib = (c[t >> 3] >> (4 * (t & 7))) & 15u;
                        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(onehot16(nib), B[t], acc, 0, 0, 0);
                    }
                    // acc[r]: item row 8*(r/4) + 4*g + (r%4), query column j
                    int m = acc[0];
#pragma unroll
                    for (int r = 1; r < 16; r++) m = acc[r] < m ? acc[r] : m;
                    if (__ballot(m <= th) != 0ull) {
                        const uint32_t slot0 = (uint32_t)(se.blk_begin + b) * 32u + 4u * g;
                        const int lm = b >= se.misc_from ? (L | (int)0x80000000) : L;
#pragma unroll
                        for (int r = 0; r < 16; r++) {
                            const bool pass = acc[r] <= th;
                            const unsigned long long mask = __ballot(pass);
                            if (mask != 0ull) {
                                if (pass) {
                                    const int pos = nstaged + __popcll(mask & lt_mask);
                                    sq.slot[pos] = slot0 + 8u * (r >> 2) + (r & 3);
                                    sq.score[pos] = (uint32_t)(acc[r] + bias);
                                    sq.qid[pos] = qid;
                                    sq.lrange[pos] = range;
                                    sq.list[pos] = lm;
                                }
                                nstaged += __popcll(mask);
                                if (nstaged > STAGE_CAP - 64) {
                                    stage_flush(v, a, sq, nstaged, lane);
                                    nstaged = 0;
                                }
                            }
                        }
                    }
                }
            }
            seg++;
            if (seg == le.seg_cnt) { seg = 0; tile++; }
        }
        // do not sit on survivors for long: their histogram counts tighten everyone's bound
        if (nstaged >= 64) {
            stage_flush(v, a, sq, nstaged, lane);
            nstaged = 0;
        }
    }
    if (nstaged > 0) stage_flush(v, a, sq, nstaged, lane);
}

// per query: sort the survivors and keep the bigK smallest (score, id); flag overflowed buffers
__global__ __launch_bounds__(WG) void select_kernel(MfmaScanArgs a)
{
    __shared__ uint64_t keys[SURV_CAP_MAX];
    const int tid = threadIdx.x;
    const int64_t q = blockIdx.x;
    const uint32_t n = a.surv_cnt[q];
    if (n > (uint32_t)a.surv_cap) {
        if (tid == 0) a.flags[q] = 1;       // the exact kernel redoes this query
        return;
    }
    if (tid == 0) a.flags[q] = 0;
    const int n2 = next_pow2(n < 2 ? 2 : (int)n);
    for (int i = tid; i < n2; i += WG) keys[i] = i < (int)n ? a.surv_buf[(size_t)q * a.surv_cap + i] : ~0ull;
    __syncthreads();
    bitonic_sort_lds(keys, n2);
    for (int i = tid; i < a.refine_k; i += WG) {
        bool ok = i < (int)n;
        uint64_t key = ok ? keys[i] : 0;
        a.cand_ids[(size_t)q * a.refine_k + i] = ok ? (int64_t)(uint32_t)key : -1;
        if (a.cand_score) a.cand_score[(size_t)q * a.refine_k + i] = ok ? (int32_t)(key >> 32) : -1;
    }
}

bool rairs_mfma_supported(const IndexView &v)
{
    return v.T == 8 || v.T == 24 || v.T == 32;
}

int rairs_launch_scan_mfma(const IndexView &v, const MfmaScanArgs &a, hipStream_t s)
{
    const int np = a.nprobe - a.p_first;
    if (np <= 0) return RAIRS_OK;
    if (a.surv_cap > SURV_CAP_MAX) {
        rairs_set_error("survivor capacity %d above %d", a.surv_cap, SURV_CAP_MAX);
        return RAIRS_EINVAL;
    }
    const int64_t pairs = a.nq * np;
    hipLaunchKernelGGL(lm_zero_kernel, dim3((unsigned)((v.nlist + 255) / 256)), dim3(256), 0, s,
                       a.lcount, v.nlist, a.next_task);
    hipLaunchKernelGGL(lm_count_kernel, dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, s,
                       a.probe_ids, a.nq, a.nprobe, a.p_first, v.nlist, a.lcount);
    hipLaunchKernelGGL(lm_prefix_kernel, dim3(1), dim3(1024), 0, s, v, a.lcount, a.loff, a.lcursor,
                       a.toff);
    hipLaunchKernelGGL(lm_fill_kernel, dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, s,
                       a.probe_ids, a.nq, a.nprobe, a.p_first, v.nlist, a.loff, a.lcursor, a.qlist);
    // persistent grid: 256 compute units x 2 workgroups of 4 waves
    const dim3 grid(512);
    switch (v.T) {
    case 8: hipLaunchKernelGGL(scan_mfma_kernel<8>, grid, dim3(WG), 0, s, v, a); break;
    case 24: hipLaunchKernelGGL(scan_mfma_kernel<24>, grid, dim3(WG), 0, s, v, a); break;
    case 32: hipLaunchKernelGGL(scan_mfma_kernel<32>, grid, dim3(WG), 0, s, v, a); break;
    default:
        rairs_set_error("MFMA scan not built for M=%d", v.M);
        return RAIRS_EUNSUPPORTED;
    }
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

int rairs_launch_select(const MfmaScanArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL(select_kernel, dim3((unsigned)a.nq), dim3(WG), 0, s, a);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}
