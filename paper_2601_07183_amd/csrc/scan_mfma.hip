// List-major SEIL scan on the matrix cores (SeilSearch of Alg. 5 for the whole query batch, with
// the list-grouped task order of the "cache optimisation for query batch" paragraph of
// Section 5.2 taken to its conclusion: a block is fetched once for 32 queries).
//
// score(query, item) = sum_m lut[query][m][code[item][m]] is a contraction of the lookup tables
// with the one-hot expansion of the codes:  sum_m sum_c lut[q][m][c] * [code[item][m] == c].
// A one-hot row of 16 has one non-zero, so the expansion is 2:4 sparse and the register-table
// kernel uses the sparse matrix instruction: one v_smfmac_i32_32x32x64_i8 covers 32 items x 32
// queries x 4 sub-quantizers (K = 4 x 16 codewords):
//   A (rows = items):   lane (item, h) passes, compressed, positions [16h, 16h+16) and
//                       [32+16h, 48+16h) of the 64 -- sub-quantizers 4t+h and 4t+2+h, the two
//                       nibbles of one code byte: 16 kept values and 16 two-bit positions, looked
//                       up per nibble in a 16-entry LDS table;
//   B (cols = queries): lane (query, g) holds the 32 table bytes lut[q][4t+2g .. 4t+2g+1][0..15]
//                       as signed bytes (value - 128; 128 * M is added back after the sum), kept
//                       in registers for the whole tile.
// The LDS-table kernel (any M) uses the dense v_mfma_i32_32x32x32_i8, two sub-quantizers per
// instruction with both operands from LDS.
// Integer arithmetic throughout, so the scores equal the plain 16-bit sums bit for bit.
//
// Work is cut into units (list L, tile of <= 32 queries probing L, run of parts of the list; a part
// is a run of segments of about 32 blocks); waves of a persistent grid draw units from a counter.
// The dedup rules are the order-free ones of scan_exact.hip.  A score passes when it is <= the
// query's bound; passing pairs are staged per wave, logged in bulk and cut to bigK afterwards by
// collect_kernel and the select kernels.
//
// The bound.  tau0 = bigK-th smallest score in a sample, the head of the query's first list (scored
// by the bound kernel of scan_exact.hip, or, for large batches, by sample_group_kernel and
// sample_mfma_kernel below with the same matrix instruction, queries grouped by first list).  Every
// survivor that the duplicate rule can never drop (an item of a shared block, or a miscellaneous
// item whose other list has the larger id; the index keeps one bit per slot for this) is counted in
// a per-query histogram of RAIRS_HIST_BINS equal score bins over [0, tau0] (over a guessed range
// when the sample had fewer than bigK items; scores beyond it share the last bin, which proves
// nothing).  Each counted slot is an entry of the query's candidate
// queue, so once bins 0..b hold >= bigK of them, no item scoring above the top edge of bin b can be
// among the bigK best: that edge is a valid, tighter bound.  Lanes that file survivors re-derive
// the query's bound now and then and lower it with an atomic minimum; scanning waves re-read it
// for every block.  A stale view is only looser.
#include <limits.h>

#include "device_util.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v8i __attribute__((ext_vector_type(8)));


// ---- grouping queries by list ----------------------------------------------------------------

// Chunks of the survivor log that the scanning waves start with: `starters` waves (with the tables
// in registers) or workgroups (tables in LDS, `waves_each` waves) begin on the units numbered by
// their own index; each wave of those that get a unit owns the chunk of its index and, reserved,
// the one at index + active waves.  The cursor for later chunks starts behind both.  (Handing out
// the first chunks by a counter instead makes 2,048 waves hit one address as the kernel starts:
// 20 us on a 0.56 ms kernel.)
static __device__ __forceinline__ uint32_t log_active_waves(uint32_t nunits, uint32_t starters, uint32_t waves_each)
{
    return (nunits < starters ? nunits : starters) * waves_each;
}
static __device__ __forceinline__ uint32_t log_first_free(uint32_t nunits, uint32_t starters, uint32_t waves_each)
{
    return 2u * log_active_waves(nunits, starters, waves_each);
}

// The scanning waves start on the units numbered by their own index (a second one each at index +
// nwaves with the tables in registers), so the unit counter starts behind those.
__global__ void lm_zero_kernel(int32_t *lcount, int32_t *lcursor, int nlist, uint32_t *next_task, uint32_t *surv_cnt,
                               int64_t nq, uint32_t *chunk_fill, int log_chunks, uint32_t *log_cursor,
                               uint32_t *log_overflow, uint32_t first_task, unsigned long long *dco,
                               uint32_t *work)
{
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < nlist) { lcount[gid] = 0; lcursor[gid] = 0; }
    if (gid < nq) { surv_cnt[gid] = 0; if (dco) dco[gid] = 0ull; }
    if (gid < log_chunks) chunk_fill[gid] = 0;
    if (gid == 0) { *next_task = first_task; *log_cursor = 0u; *log_overflow = 0; }   // (the cursor: set again with the unit count)
    if (gid == 0) { work[0] = 0u; work[1 + nq] = 0u; }   // the two lists of queries for the kernels behind the scan
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

// A unit of work is (list, tile of <= 32 of the queries probing it, run of unit_parts consecutive
// parts of the list; a part is about 32 blocks, unit_parts is 1..4, smaller when there is little
// work).  Exclusive prefixes over lists of queries (loff) and units
// (toff), and the list of every unit; one workgroup of 1024.
// Parts per unit of list L: the lists from `tail_from` on are cut into single parts.  Waves take
// units in order, so the last ones taken are small and the waves finish closer together (the
// kernel ends with its slowest wave, and a two-part unit is 0.08 ms of work on the 1M x 128 workload).
static __device__ __forceinline__ int list_unit_parts(int L, int unit_parts, int tail_from)
{
    return L >= tail_from ? 1 : unit_parts;
}

static __device__ __forceinline__ int units_of(int nqueries, int part_cnt, int unit_parts)
{
    return ((nqueries + 31) >> 5) * ((part_cnt + unit_parts - 1) / unit_parts);
}

// Everything a scanning wave needs to start on unit `u` of list L in one look-up, so that it does
// not walk unit -> list -> directory entry -> parts at the head of every unit: the list, the tile,
// the unit's segments [seg0, seg1) as absolute segment numbers, and where the list's queries are.
#define UNIT_REC_WORDS 8
static __device__ __forceinline__ void write_unit_rec(const IndexView &v, int32_t *unit_rec, int u, int L,
                                                      int first_unit_of_list, int qbase, int qn, int unit_parts)
{
    const ListEntry le = v.lists[L];
    const int rem = u - first_unit_of_list;
    const int runs = (le.part_cnt + unit_parts - 1) / unit_parts;
    const int tile = rem / runs;
    const int p0 = (rem % runs) * unit_parts;
    const int p1 = p0 + unit_parts < le.part_cnt ? p0 + unit_parts : le.part_cnt;
    int4 lo = make_int4(L, tile, v.parts[le.part_begin + p0], v.parts[le.part_begin + p1]);
    int4 hi = make_int4(qbase, qn, 0, 0);
    *(int4 *)(unit_rec + (size_t)u * UNIT_REC_WORDS) = lo;
    *(int4 *)(unit_rec + (size_t)u * UNIT_REC_WORDS + 4) = hi;
}

__global__ __launch_bounds__(1024) void lm_prefix_kernel(IndexView v,
                                                         const int32_t *__restrict__ lcount,
                                                         int32_t *loff, int32_t *lcursor,
                                                         int32_t *toff, int32_t *unit_list,
                                                         int unit_parts, int tail_from, int32_t *unit_rec,
                                                         uint32_t *log_cursor, uint32_t starters, uint32_t waves_each)
{
    __shared__ int sc[1024], st[1024];
    // one workgroup on the critical path of the grouping, usually next to a kernel that fills the
    // chip: let its waves issue first on the compute unit they share
    __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x;
    const int per = (v.nlist + 1023) / 1024;
    const int lo = tid * per < v.nlist ? tid * per : v.nlist;
    const int hi = lo + per < v.nlist ? lo + per : v.nlist;
    int c = 0, t = 0;
    for (int L = lo; L < hi; L++) {
        int n = lcount[L];
        c += n;
        t += units_of(n, v.lists[L].part_cnt, list_unit_parts(L, unit_parts, tail_from));
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
        tb += units_of(n, v.lists[L].part_cnt, list_unit_parts(L, unit_parts, tail_from));
    }
    if (tid == 1023) {
        loff[v.nlist] = sc[1023];
        toff[v.nlist] = st[1023];
        *log_cursor = log_first_free((uint32_t)st[1023], starters, waves_each);
    }
}

// The unit table of the large-directory route, one thread per list (inside the single workgroup of
// the prefix kernel these writes took 1.5 ms for 16,384 lists and 100,000 units).
__global__ __launch_bounds__(256) void lm_units_kernel(IndexView v, const int32_t *__restrict__ lcount,
                                                       const int32_t *__restrict__ loff,
                                                       const int32_t *__restrict__ toff,
                                                       int32_t *unit_list, int unit_parts, int tail_from,
                                                       int32_t *unit_rec)
{
    const int L = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (L >= v.nlist) return;
    const int n = lcount[L], tb = toff[L], cb = loff[L];
    const int up = list_unit_parts(L, unit_parts, tail_from);
    const int nu = units_of(n, v.lists[L].part_cnt, up);
    for (int u = 0; u < nu; u++) {
        unit_list[tb + u] = L;
        write_unit_rec(v, unit_rec, tb + u, L, tb, cb, n, up);
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

// The same two steps for directories of up to LM_LDS_NLIST lists: a workgroup first groups its
// LM_PAIRS (query, probe) pairs by list in LDS and then touches each list's global counter once,
// instead of once per pair (a list is probed by hundreds of queries of a batch).
#define LM_PAIRS 4096
#define LM_LDS_NLIST 16384
#define LM_UNIT_WGS 8        // workgroups of the fill kernel that build the unit table
__global__ __launch_bounds__(256) void lm_count_lds_kernel(const int32_t *__restrict__ probe_ids,
                                                           int64_t nq, int nprobe, int p_first,
                                                           int nlist, int32_t *lcount, int qb)
{
    extern __shared__ int32_t lm_hist[];
    const int tid = threadIdx.x;
    for (int i = tid; i < nlist; i += 256) lm_hist[i] = 0;
    __syncthreads();
    const int np = nprobe - p_first;
    const int64_t q0 = (int64_t)blockIdx.x * qb;
    const int pairs = qb * np;
    for (int i = tid; i < pairs; i += 256) {
        const int64_t q = q0 + i / np;
        if (q >= nq) continue;
        const int L = probe_ids[q * nprobe + p_first + i % np];
        if (L >= 0 && L < nlist) atomicAdd(&lm_hist[L], 1);
    }
    __syncthreads();
    for (int i = tid; i < nlist; i += 256) {
        const int c = lm_hist[i];
        if (c) atomicAdd(&lcount[i], c);
    }
}

// Exclusive prefix sums, by a workgroup of 256 threads, of x[0 .. n): thread t owns the contiguous
// run [t per, (t+1) per); `mine` is the sum over its run.  Returns the sum over the runs before
// this thread's and leaves the total in *total (LDS).  wsum: LDS, 4 words.
static __device__ __forceinline__ int wg256_exclusive(int mine, int32_t *wsum, int32_t *total)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int x = __shfl_up(incl, off);
        if (lane >= off) incl += x;
    }
    __syncthreads();                                   // wsum may still be read from an earlier call
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 4; w++) {
        const int x = wsum[w];
        if (w < wave) before += x;
        all += x;
    }
    if (tid == 0) *total = all;
    return before + incl - mine;
}

// Second step for directories of up to LM_LDS_NLIST lists.  No separate prefix kernel sits between
// counting and filling: every workgroup derives the list offsets from the counts itself (a few KB,
// from L2), and LM_UNIT_WGS extra workgroups (the last ones) write them out for the scan together
// with the unit table (toff, unit_list).
__global__ __launch_bounds__(256) void lm_fill_lds_kernel(IndexView v, const int32_t *__restrict__ probe_ids,
                                                          int64_t nq, int nprobe, int p_first,
                                                          const int32_t *__restrict__ lcount,
                                                          int32_t *loff, int32_t *lcursor, int32_t *qlist,
                                                          int qb, int32_t *toff, int32_t *unit_list,
                                                          int unit_parts, int tail_from, int32_t *unit_rec,
                                                          uint32_t *log_cursor, uint32_t starters, uint32_t waves_each)
{
    extern __shared__ int32_t lm_lds[];                // [nlist] ranks / run starts, [nlist + 1] offsets
    __shared__ int32_t wsum[4], total;
    const int nlist = v.nlist;
    int32_t *lm_hist = lm_lds, *loff_s = lm_lds + nlist;
    const int tid = threadIdx.x;
    const int per = (nlist + 255) / 256;
    const int lo = tid * per < nlist ? tid * per : nlist;
    const int hi = lo + per < nlist ? lo + per : nlist;
    {
        int mine = 0;
        for (int L = lo; L < hi; L++) mine += lcount[L];
        int run = wg256_exclusive(mine, wsum, &total);
        for (int L = lo; L < hi; L++) {
            loff_s[L] = run;
            run += lcount[L];
        }
    }
    __syncthreads();
    const int nfill = (int)gridDim.x - LM_UNIT_WGS;
    if ((int)blockIdx.x >= nfill) {
        // The unit table: every one of these workgroups derives the unit offsets of all lists
        // (into LDS), the first writes the offsets out, and each fills its share of unit_list,
        // finding a unit's list by bisection on the offsets.
        const int ub = (int)blockIdx.x - nfill;
        int32_t *toff_s = lm_hist;                     // [nlist]
        if (ub == 0) {
            if (tid == 0) loff[nlist] = total;
            for (int L = lo; L < hi; L++) loff[L] = loff_s[L];
        }
        int mine = 0;
        for (int L = lo; L < hi; L++) mine += units_of(lcount[L], v.lists[L].part_cnt, list_unit_parts(L, unit_parts, tail_from));
        int run = wg256_exclusive(mine, wsum, &total);
        for (int L = lo; L < hi; L++) {
            toff_s[L] = run;
            if (ub == 0) toff[L] = run;
            run += units_of(lcount[L], v.lists[L].part_cnt, list_unit_parts(L, unit_parts, tail_from));
        }
        __syncthreads();
        const int nunits = total;
        if (ub == 0 && tid == 0) {
            toff[nlist] = nunits;
            *log_cursor = log_first_free((uint32_t)nunits, starters, waves_each);
        }
        const int share = (nunits + LM_UNIT_WGS - 1) / LM_UNIT_WGS;
        const int e1 = (ub + 1) * share < nunits ? (ub + 1) * share : nunits;
        for (int e = ub * share + tid; e < e1; e += 256) {
            // the last list whose first unit is <= e (lists without units share their successor's offset)
            int a0 = 0, b0 = nlist - 1;
            while (a0 < b0) {
                const int mid = (a0 + b0 + 1) >> 1;
                if (toff_s[mid] <= e) a0 = mid; else b0 = mid - 1;
            }
            unit_list[e] = a0;
            write_unit_rec(v, unit_rec, e, a0, toff_s[a0], loff_s[a0], lcount[a0], list_unit_parts(a0, unit_parts, tail_from));
        }
        return;
    }
    for (int i = tid; i < nlist; i += 256) lm_hist[i] = 0;
    __syncthreads();
    const int np = nprobe - p_first;
    const int64_t q0 = (int64_t)blockIdx.x * qb;
    const int pairs = qb * np;                         // <= LM_PAIRS
    int myL[LM_PAIRS / 256], myr[LM_PAIRS / 256];
#pragma unroll
    for (int k = 0; k < LM_PAIRS / 256; k++) {
        const int i = tid + 256 * k;
        myL[k] = -1;
        myr[k] = 0;
        if (i < pairs) {
            const int64_t q = q0 + i / np;
            if (q < nq) {
                const int L = probe_ids[q * nprobe + p_first + i % np];
                if (L >= 0 && L < nlist) {
                    myL[k] = L;
                    myr[k] = atomicAdd(&lm_hist[L], 1);        // rank within this workgroup
                }
            }
        }
    }
    __syncthreads();
    for (int i = tid; i < nlist; i += 256) {
        const int c = lm_hist[i];
        if (c) lm_hist[i] = loff_s[i] + atomicAdd(&lcursor[i], c);   // where this workgroup's run starts
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < LM_PAIRS / 256; k++)
        if (myL[k] >= 0) qlist[lm_hist[myL[k]] + myr[k]] = (int32_t)(q0 + (tid + 256 * k) / np);
}

// ---- the scan ----------------------------------------------------------------------------------

// Bin of a score: floor(score * mul / 2^32) with mul = floor(BINS 2^32 / (range + 1)), range >=
// BINS, so that scores 0..range fall into bins 0..BINS-1 without a division on the hot path
// (larger scores are put into the last bin by the caller).
static __device__ __forceinline__ uint32_t hist_mul(uint32_t range)
{
    const uint32_t r = range < (uint32_t)RAIRS_HIST_BINS ? (uint32_t)RAIRS_HIST_BINS : range;
    return (uint32_t)(((unsigned long long)RAIRS_HIST_BINS << 32) / (uint64_t)(r + 1u));
}

// Tightest bound the histogram of query `qid` proves: the histogram counts queue entries, so once
// bins 0..b hold >= bigK of them nothing scoring above the top edge of bin b can be among the
// bigK best.
static __device__ __forceinline__ uint32_t histogram_bound(const MfmaScanArgs &a, int qid,
                                                           uint32_t mul)
{
    const uint4 *hq = (const uint4 *)(a.hist + (size_t)qid * RAIRS_HIST_BINS);
    const uint32_t need = (uint32_t)a.refine_k;
    uint32_t cum = 0;
    int b = RAIRS_HIST_BINS;
    // (16 bins in flight at a time: all 64 at once take 64 registers, which the scan loop around
    // this call then pays for with spills)
    constexpr int HB = 4;
    for (int i0 = 0; i0 < RAIRS_HIST_BINS / 4; i0 += HB) {
        uint4 h[HB];
#pragma unroll
        for (int i = 0; i < HB; i++) h[i] = hq[i0 + i];
#pragma unroll
        for (int i = 0; i < HB; i++) {
            cum += h[i].x; b = (cum >= need && b == RAIRS_HIST_BINS) ? 4 * (i0 + i) : b;
            cum += h[i].y; b = (cum >= need && b == RAIRS_HIST_BINS) ? 4 * (i0 + i) + 1 : b;
            cum += h[i].z; b = (cum >= need && b == RAIRS_HIST_BINS) ? 4 * (i0 + i) + 2 : b;
            cum += h[i].w; b = (cum >= need && b == RAIRS_HIST_BINS) ? 4 * (i0 + i) + 3 : b;
        }
    }
    if (b >= RAIRS_HIST_BINS - 1) return 0xFFFFu;      // the last bin also holds scores beyond the range
    // largest score whose bin is <= b
    const uint64_t edge = ((((uint64_t)(b + 1)) << 32) - 1ull) / (uint64_t)mul;
    return edge < 0xFFFFull ? (uint32_t)edge : 0xFFFFu;
}

// A passing (item, query) pair waits in a per-wave LDS queue until enough have gathered; then the
// wave appends them to its current chunk of a global survivor log with plain stores, counts them
// in the queries' histograms and, for some, lowers the query's bound.  Nothing on this path
// waits for a returning atomic: the wave owns its chunk, and the next chunk's number is requested
// long before it is needed (only waves with work own chunks, so the log of a small batch is
// small).  Chunks of 2,048 entries: with 256 the scan kernel of the 1M x 128 workload took
// 0.610 ms instead of 0.558 (1,024 and more: the same) and the collect step, whose atomics go by
// chunk and query, 49 us instead of 35.  Ids, tags and the duplicate rule are resolved afterwards,
// in bulk, by collect_kernel and the select kernels.
#define STAGE_CAP 128              // a multiple of 64 (a flush takes the queue in rows of 64); 192 and 256 measured slower
static_assert(STAGE_CAP % 64 == 0 && STAGE_CAP >= 128, "stage queue rows");
#define LOG_CHUNK RAIRS_LOG_CHUNK
#define LOG_COUNTED 0x80000000u    // bit 31 of a staged slot: the entry counts in the histogram
struct StageQueue {
    uint2 ent[STAGE_CAP];          // the log entry: {block * 32 + item (| LOG_COUNTED), score << 16 | query of the pass}
    uint32_t hmul[STAGE_CAP];      // hist_mul of the query's score range
};

struct LogCursor {
    uint32_t chunk, used;               // wave-uniform
    uint32_t next_v;                    // lane 0: the chunk reserved for later (left in a vector
                                        // register so that nobody waits for the atomic's answer
                                        // before the chunk is needed)
};

// When a wave refreshes bounds: every `gap`-th flush.  The gap starts at 4, doubles (up to 16)
// each time a refresh lowers no bound -- late in the scan the bounds have settled and reading
// histograms is wasted time -- and returns to 4 when one does.  (With the bound that the sample
// gives, a start of 2 is 1 % slower on the 1M x 128 workload and 3 % on the 960-dimension one,
// a start of 8 is slower again.)
// (measured on the 1M x 128 workload: all or half of the lanes refreshing, at any pacing, is slower
// than a quarter -- a refresh costs memory traffic per lane, not only latency)
#define REFRESH_LANES_MASK 3
#define REFRESH_GAP_MIN 4u
#define REFRESH_GAP_MAX 16u
struct RefreshPace {
    uint32_t gap, since, turn;          // wave-uniform
};

static __device__ __forceinline__ void stage_flush(const MfmaScanArgs &a, StageQueue &sq, int n,
                                                   int lane, LogCursor &lc, RefreshPace &rp)
{
    if (lc.used + (uint32_t)n > LOG_CHUNK) {
        // close the chunk, move to the one reserved earlier, reserve another
        if (lane == 0 && lc.chunk < (uint32_t)a.log_chunks) a.chunk_fill[lc.chunk] = lc.used;
        lc.chunk = (uint32_t)__builtin_amdgcn_readfirstlane((int)lc.next_v);
        lc.used = 0;
        uint32_t nx = 0;
        if (lane == 0) nx = atomicAdd(a.log_cursor, 1u);
        lc.next_v = nx;
    }
    const bool room = lc.chunk < (uint32_t)a.log_chunks;
    if (!room && lane == 0) *a.log_overflow = 1u;      // every query is then redone exactly
#pragma unroll
    for (int u = 0; u < STAGE_CAP / 64; u++) {
        const int i = lane + 64 * u;
        if (i < n) {
            const uint2 e = sq.ent[i];
            const uint32_t qid = e.y & 0xFFFFu;
            if (room) a.log[(size_t)lc.chunk * LOG_CHUNK + lc.used + i] = make_uint2(e.x & ~LOG_COUNTED, e.y);
            if (e.x & LOG_COUNTED) {
                // scores beyond the histogram's range share the last bin
                const uint32_t bin = __umulhi(e.y >> 16, sq.hmul[i]);
                atomicAdd(&a.hist[(size_t)qid * RAIRS_HIST_BINS + (bin < RAIRS_HIST_BINS - 1 ? bin : RAIRS_HIST_BINS - 1)], 1u);
            }
        }
    }
    if (++rp.since >= rp.gap) {
        // a quarter of the first row's entries, a different quarter each time, refresh their
        // query's bound.  A stale histogram only gives a looser bound; the bound itself only
        // ever shrinks.
        rp.since = 0;
        bool lowered = false;
        if (lane < n && ((lane + rp.turn) & (REFRESH_LANES_MASK)) == 0) {
            const int qid = (int)(sq.ent[lane].y & 0xFFFFu);
            const int32_t cur = __hip_atomic_load(&a.bound[qid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t nb = histogram_bound(a, qid, sq.hmul[lane]);
            if (nb < 0xFFFFu && (int32_t)nb < cur) {
                atomicMin(&a.bound[qid], (int32_t)nb);
                lowered = true;
            }
        }
        rp.turn++;
        rp.gap = __ballot(lowered) != 0ull ? REFRESH_GAP_MIN : (rp.gap < REFRESH_GAP_MAX ? rp.gap * 2u : REFRESH_GAP_MAX);
    }
    lc.used += (uint32_t)n;
}

// The accumulators of a block start at -(th + 1), th the lane's threshold in the matrix core's
// signed units, so a row passes (score <= th) exactly when its accumulator ends up negative, and
// the mask of passing rows is the 16 sign bits: one funnel shift per row, no compare, no select.
// Lanes that must not pass anything start at a large positive value instead.
#define ACC_NEVER 0x3FFFFFFF
static __device__ __forceinline__ uint32_t negative_rows(const v16i &acc)
{
    uint32_t pm = 0;
#pragma unroll
    for (int r = 15; r >= 0; r--) pm = __builtin_amdgcn_alignbit(pm, (uint32_t)acc[r], 31);   // pm << 1 | sign
    return pm;
}

// Kept values and positions of the compressed one-hot operand, by code: entry c of the first 16
// is the 8 kept values (a one in the first slot of group c >> 2), entry 16 + c the 8 two-bit
// positions (c & 3 in that slot) once as the low and once as the high half of the position word.
static __device__ __forceinline__ void fill_sparse_tab(uint2 *tab)
{
    if (threadIdx.x < 16) {
        const int c = threadIdx.x;
        const unsigned long long val = 1ull << (16 * (c >> 2));
        const uint32_t pos = (uint32_t)(c & 3) << (4 * (c >> 2));
        tab[c] = make_uint2((uint32_t)val, (uint32_t)(val >> 32));
        tab[16 + c] = make_uint2(pos, pos << 16);
    }
}

// Number of set bits of `mask` below this lane.
static __device__ __forceinline__ int lanes_below(unsigned long long mask)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// acc[r] for a row index that differs from lane to lane: four levels of bitwise selection on the
// bits of r, in registers (an indexed array would go through memory).
static __device__ __forceinline__ int select_row(const v16i &acc, int r)
{
    const int m0 = -(r & 1), m1 = -((r >> 1) & 1), m2 = -((r >> 2) & 1), m3 = -((r >> 3) & 1);
    int s8[8], s4[4];
#pragma unroll
    for (int k = 0; k < 8; k++) s8[k] = (acc[2 * k + 1] & m0) | (acc[2 * k] & ~m0);
#pragma unroll
    for (int k = 0; k < 4; k++) s4[k] = (s8[2 * k + 1] & m1) | (s8[2 * k] & ~m1);
    const int s2a = (s4[1] & m2) | (s4[0] & ~m2), s2b = (s4[3] & m2) | (s4[2] & ~m2);
    return (s2b & m3) | (s2a & ~m3);
}

template <int T>
__global__ __launch_bounds__(WG, 2) void scan_mfma_kernel(IndexView v, MfmaScanArgs a)
{
    constexpr int ND = (T + 7) / 8;
    constexpr int M = 2 * T;
    constexpr int TS = T / 2;                          // sparse matrix instructions per block
    static_assert(T % 2 == 0, "a sparse instruction takes four sub-quantizers");
    __shared__ StageQueue stage[WG / 64];
    // A code byte holds the codes (c1, c2) of two sub-quantizers of one instruction; their one-hot
    // rows of 16 + 16 zeros and ones are 2:4 sparse, so the matrix core takes them compressed:
    // per group of four positions two kept values and their 2-bit positions, looked up by code.
    __shared__ uint2 sparse_tab[32];
    fill_sparse_tab(sparse_tab);
    __syncthreads();
    const int lane = threadIdx.x & 63, g = lane >> 5, j = lane & 31;
    StageQueue &sq = stage[threadIdx.x >> 6];
    const int bias = 128 * M;

    v8i B[TS];
#pragma unroll
    for (int t = 0; t < TS; t++) B[t] = (v8i){0, 0, 0, 0, 0, 0, 0, 0};
    int nstaged = 0;                                   // wave-uniform fill of the stage queue
    const uint32_t nunits = (uint32_t)a.toff[v.nlist];
    if (nunits == 0u) return;                          // nothing was written: all chunk fills stay 0
    // first unit and first two log chunks by wave index; the counters start behind them
    const uint32_t gwave = blockIdx.x * (WG / 64) + (threadIdx.x >> 6), nwaves = gridDim.x * (WG / 64);
    LogCursor lc;
    lc.chunk = gwave;                                  // (a wave without a unit never writes)
    lc.next_v = gwave + log_active_waves(nunits, nwaves, 1u);
    lc.used = 0;
    RefreshPace pace = {REFRESH_GAP_MIN, REFRESH_GAP_MIN - 1u, 0u};
#define FLUSH_STAGE()                                                   \
    do {                                                                \
        stage_flush(a, sq, nstaged, lane, lc, pace);     \
        nstaged = 0;                                                    \
    } while (0)

    // A wave works on unit u, already knows the one after it (u_next) and asks the counter for
    // the one after that: so the record of the next unit can be fetched a whole unit ahead and a
    // unit starts with its list, tile and segments in registers instead of a chain of look-ups.
    uint32_t u = gwave, u_next = gwave + nwaves;       // the counter starts behind both
    int rec = u < nunits ? a.unit_rec[(size_t)u * UNIT_REC_WORDS + (lane & 7)] : 0;
    while (u < nunits) {                               // every wave leaves: the counter only grows
        uint32_t u_next2 = 0;
        if (lane == 0) u_next2 = atomicAdd(a.next_task, 1u);
        const int tile = __builtin_amdgcn_readlane(rec, 1);
        const int seg0 = __builtin_amdgcn_readlane(rec, 2), seg1 = __builtin_amdgcn_readlane(rec, 3);
        const int qbase = __builtin_amdgcn_readlane(rec, 4), qn = __builtin_amdgcn_readlane(rec, 5);
        rec = a.unit_rec[(size_t)(u_next < nunits ? u_next : u) * UNIT_REC_WORDS + (lane & 7)];
        int qid;
        uint32_t hmul;
        {
            // the tile: query of this lane's column and its tables
            const int qi = tile * 32 + j;
            qid = qi < qn ? a.qlist[qbase + qi] : -1;
            hmul = hist_mul(qid >= 0 ? (uint32_t)a.tau[qid] : 0u);
            // instruction t takes sub-quantizers 4t .. 4t+3; this lane's half of its 64 positions
            // is the 16 + 16 table entries of sub-quantizers 4t + 2g and 4t + 2g + 1
            const uint8_t *lq = a.lut + (size_t)(qid >= 0 ? qid : 0) * (M * 16) + g * 32;
            // every lane loads (an absent column reads query 0's rows and masks them to zero): a
            // conditional load would be waited for one by one
            const int keep = qid >= 0 ? -1 : 0;
            const v4i flip = {(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
            const v4i keep4 = {keep, keep, keep, keep};
#pragma unroll
            for (int t = 0; t < TS; t++) {
                const v4i x = (*(const v4i *)(lq + t * 64) ^ flip) & keep4;
                const v4i y = (*(const v4i *)(lq + t * 64 + 16) ^ flip) & keep4;
                B[t] = (v8i){x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
            }
        }
        // the query's bound: other waves keep lowering it, so it is looked up again during the
        // run, ahead of the block that uses it (a stale bound is only looser)
        // per-lane addresses stay 32-bit offsets from uniform bases (a 64-bit pointer per lane
        // costs two of the registers this kernel is short of)
        const uint32_t q0 = (uint32_t)(qid >= 0 ? qid : 0);
        const uint32_t bm0 = q0 * (uint32_t)a.bmwords;   // < 2^27: a pass has at most 65,536 queries of at most 2,048 words
        int bound_next = __hip_atomic_load(a.bound + q0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        // segment entries run two ahead and the owner's bitmap word one ahead, so that neither
        // is waited for at the head of a segment
        SegEntry se = v.segs[seg0];
        SegEntry sen = v.segs[seg0 + 1 < seg1 ? seg0 + 1 : seg0];
        uint32_t owner_bits = a.bitmap[bm0 + (uint32_t)(se.owner >= 0 ? se.owner >> 5 : 0)];
        const uint32_t *cp = v.codes + (size_t)se.blk_begin * ND * 64;      // wave-uniform
        uint32_t cn[ND];
#pragma unroll
        for (int w = 0; w < ND; w++) cn[w] = cp[w * 64 + lane];
        // {countable slots, slots in use} of the block, fetched with its codes
        uint2 cmn = v.bmask[se.blk_begin];
        uint32_t scored = 0;                           // items this lane's query was scored against in this unit
        for (int seg = seg0; seg < seg1; seg++) {
            const bool has_next = seg + 1 < seg1;
            const SegEntry sen2 = v.segs[seg + 2 < seg1 ? seg + 2 : seg1 - 1];
            const uint32_t ob_next = a.bitmap[bm0 + (uint32_t)(sen.owner >= 0 ? sen.owner >> 5 : 0)];
            const uint32_t *cpn = v.codes + (size_t)sen.blk_begin * ND * 64;   // wave-uniform
            // cell (owner, L) is scored through list `owner` for queries that probe it
            const bool live = qid >= 0 && !(se.owner >= 0 && ((owner_bits >> (se.owner & 31)) & 1u));
            if (__ballot(live) == 0ull) {
                // nobody needs this run; keep the prefetch chain going
                if (has_next) {
#pragma unroll
                    for (int w = 0; w < ND; w++) cn[w] = cpn[w * 64 + lane];
                    cmn = v.bmask[sen.blk_begin];
                }
            } else {
                uint32_t seg_items = 0;                // wave-uniform: slots in use of the blocks contracted
                for (int b = 0; b < se.nblk; b++) {
                    uint32_t c[ND];
#pragma unroll
                    for (int w = 0; w < ND; w++) c[w] = cn[w];
                    const uint32_t cmask = cmn.x;
                    seg_items += (uint32_t)__popc(cmn.y);
                    // the accumulators start at -(threshold + 1): a row passes iff it ends up negative
                    const int negth = live ? -(bound_next - bias + 1) : ACC_NEVER;
                    // (every fourth block is often enough: the bound moves rarely)
                    if ((b & 3) == 3) bound_next = __hip_atomic_load(a.bound + q0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    if (b + 1 < se.nblk) {             // fetch the next block while this one is scored
#pragma unroll
                        for (int w = 0; w < ND; w++) cn[w] = cp[(size_t)(b + 1) * ND * 64 + w * 64 + lane];
                        cmn = v.bmask[se.blk_begin + b + 1];
                    } else if (has_next) {             // ... or the first block of the next run
#pragma unroll
                        for (int w = 0; w < ND; w++) cn[w] = cpn[w * 64 + lane];
                        cmn = v.bmask[sen.blk_begin];
                    }
                    // (a copy the compiler cannot see through: the accumulators' start value must
                    // not stay tied to the register that the survivor path reads later, or the
                    // whole 16-register tuple is built elsewhere and moved)
                    int acc0 = negth;
                    asm volatile("" : "+v"(acc0));
                    v16i acc;
#pragma unroll
                    for (int r = 0; r < 16; r++) acc[r] = acc0;
                    // The table reads of an instruction (values, positions) go out two
                    // instructions ahead of it, so that an LDS round trip hides behind matrix
                    // work; the scheduling fences keep the compiler from moving them either way
                    // (all at the front costs 80 registers, none ahead stalls every instruction).
#define CODE_LO(t_) ((c[(t_) >> 2] >> (8 * ((t_) & 3))) & 15u)
#define CODE_HI(t_) ((c[(t_) >> 2] >> (8 * ((t_) & 3) + 4)) & 15u)
#define LOAD_A(t_)                                                                        \
    do {                                                                                  \
        const uint2 *e1_ = &sparse_tab[CODE_LO(t_)], *e2_ = &sparse_tab[CODE_HI(t_)];      \
        v1[t_] = e1_[0]; v2[t_] = e2_[0];                                                 \
        p1[t_] = e1_[16].x; p2[t_] = e2_[16].y;                                           \
    } while (0)
                    // raw table words; they are put together where they are used, not where
                    // they are loaded, so that nothing waits for a load in its own stage
                    uint2 v1[TS], v2[TS];
                    uint32_t p1[TS], p2[TS];
                    LOAD_A(0);
                    if (TS > 1) LOAD_A(1);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int t = 0; t < TS; t++) {
                        const v4i av = {(int)v1[t].x, (int)v1[t].y, (int)v2[t].x, (int)v2[t].y};
                        acc = __builtin_amdgcn_smfmac_i32_32x32x64_i8(av, B[t], acc, (int)(p1[t] | p2[t]), 0, 0);
                        if (t + 2 < TS) LOAD_A(t + 2);
                        __builtin_amdgcn_sched_barrier(0);
                    }
#undef LOAD_A
#undef CODE_LO
#undef CODE_HI
                    // acc[r]: item row 8*(r/4) + 4*g + (r%4), query column j
                    uint32_t pm = negative_rows(acc);     // rows of this lane that pass
                    if (__ballot(pm != 0u) != 0ull) {
                        const uint32_t slot0 = (uint32_t)(se.blk_begin + b) * 32u + 4u * g;
                        if (b == se.nblk - 1 && se.tail_valid < 32) {
                            // the list's last block: drop rows whose slot holds no item
#pragma unroll
                            for (int r = 0; r < 16; r++)
                                if (8 * (r >> 2) + 4 * g + (r & 3) >= se.tail_valid) pm &= ~(1u << r);
                        }
                        for (;;) {
                            const bool has = pm != 0u;
                            const unsigned long long mask = __ballot(has);
                            if (mask == 0ull) break;
                            // every lane selects (lanes without a row select row 0 and drop it)
                            const int r = has ? __builtin_ctz(pm) : 0;
                            pm &= pm - 1u;
                            const int sc = select_row(acc, r) - negth;    // the row's sum, in the matrix core's units
                            if (has) {
                                const int pos = nstaged + lanes_below(mask);
                                const uint32_t item = 8u * (uint32_t)(r >> 2) + (uint32_t)(r & 3);   // + 4 g
                                sq.ent[pos] = make_uint2((slot0 + item) | (((cmask >> (item + 4u * g)) & 1u) << 31),
                                                         ((uint32_t)(sc + bias) << 16) | (uint32_t)qid);
                                sq.hmul[pos] = hmul;
                            }
                            nstaged += __popcll(mask);
                            if (nstaged > STAGE_CAP - 64) {
                                FLUSH_STAGE();
                            }
                        }
                    }
                }
                // the distance computations of this run (Section 6.1's DCO): every slot in use of
                // every block that was contracted, for each query the run was live for
                scored += live ? seg_items : 0u;
            }
            se = sen;
            sen = sen2;
            owner_bits = ob_next;
            cp = cpn;
        }
        // do not sit on survivors for long: their histogram counts tighten everyone's bound
        if (nstaged >= 32) FLUSH_STAGE();
        if (a.dco && g == 0 && scored) atomicAdd(&a.dco[qid], (unsigned long long)scored);
        u = u_next;
        u_next = (uint32_t)__builtin_amdgcn_readfirstlane((int)u_next2);
    }
    if (nstaged > 0) FLUSH_STAGE();
    // (a wave that never had a unit wrote nothing, and the chunk of its index may be another wave's)
    if (lane == 0 && lc.used > 0 && lc.chunk < (uint32_t)a.log_chunks) a.chunk_fill[lc.chunk] = lc.used;
}

// Distribute the survivor log to the per-query buffers (a workgroup takes one chunk at a time).  A chunk holds
// entries of a few dozen queries; they are grouped in LDS first so that each query's counter is
// bumped once per chunk, not once per entry.
#define COLLECT_WG 1024
#define COLLECT_EPT (LOG_CHUNK / COLLECT_WG)            // entries of a chunk per thread
#define COLLECT_SLOTS 512
static_assert(LOG_CHUNK % COLLECT_WG == 0, "a chunk is a whole number of entries per thread");
static_assert(COLLECT_WG >= COLLECT_SLOTS, "a thread per slot clears and publishes the tables");
__global__ __launch_bounds__(COLLECT_WG) void collect_kernel(MfmaScanArgs a)
{
    __shared__ int32_t key[COLLECT_SLOTS];
    __shared__ uint32_t cnt[COLLECT_SLOTS], base[COLLECT_SLOTS];
    const int tid = threadIdx.x;
    uint32_t lim = *a.log_cursor;                       // chunks handed out
    lim = lim < (uint32_t)a.log_chunks ? lim : (uint32_t)a.log_chunks;
    for (uint32_t c = blockIdx.x; c < lim; c += gridDim.x) {
    const uint32_t n = a.chunk_fill[c];
    if (n == 0) continue;                               // uniform
    if (tid < COLLECT_SLOTS) { key[tid] = -1; cnt[tid] = 0; }
    __syncthreads();
    uint2 e[COLLECT_EPT];                               // {slot, score << 16 | query}
    int slot[COLLECT_EPT];
    uint32_t rank[COLLECT_EPT];
    // an entry logged under an earlier, looser bound is dropped when its score is above the
    // query's final bound: it cannot be among the bigK best
    bool live[COLLECT_EPT];
#pragma unroll
    for (int k = 0; k < COLLECT_EPT; k++) {
        const int i = tid + COLLECT_WG * k;
        e[k] = make_uint2(0, 0);
        if (i < (int)n) e[k] = a.log[(size_t)c * LOG_CHUNK + i];
    }
#pragma unroll
    for (int k = 0; k < COLLECT_EPT; k++) {
        const int i = tid + COLLECT_WG * k;
        live[k] = i < (int)n && (int32_t)(e[k].y >> 16) <= a.bound[e[k].y & 0xFFFFu];
        slot[k] = -1;
        rank[k] = 0;
    }
#pragma unroll
    for (int k = 0; k < COLLECT_EPT; k++) {
        if (live[k]) {
            const int qid = (int)(e[k].y & 0xFFFFu);
            // open addressing on the query id; a full table falls back to a direct atomic below
            int h = (int)(((uint32_t)qid * 2654435761u) >> 23);          // 9 bits
            for (int probe = 0; probe < COLLECT_SLOTS; probe++) {
                const int prev = atomicCAS(&key[h], -1, qid);
                if (prev == -1 || prev == qid) { slot[k] = h; break; }
                h = (h + 1) & (COLLECT_SLOTS - 1);
            }
            if (slot[k] >= 0) rank[k] = atomicAdd(&cnt[slot[k]], 1u);
        }
    }
    __syncthreads();
    if (tid < COLLECT_SLOTS && cnt[tid] > 0) base[tid] = atomicAdd(&a.surv_cnt[key[tid]], cnt[tid]);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < COLLECT_EPT; k++) {
        if (live[k]) {
            const uint32_t qid = e[k].y & 0xFFFFu;
            const uint32_t pos = slot[k] >= 0 ? base[slot[k]] + rank[k] : atomicAdd(&a.surv_cnt[qid], 1u);
            if (pos < (uint32_t)a.surv_cap)
                a.surv_buf[(size_t)qid * a.surv_cap + pos] = ((uint64_t)(e[k].y >> 16) << 48) | e[k].x;
        }
    }
    __syncthreads();                                    // the tables are reused for the next chunk
    }
}

// Per query with at most `cap` survivors (the usual case): one wave resolves them (id,
// duplicate rule of the miscellaneous area), sorts them by (score, id) in its own LDS region and
// writes the bigK smallest.  No workgroup barrier is used: a wave only touches its own region, and
// LDS operations of one wave complete in issue order.
#define SELW_STRIKE_MAX 8           // ties beyond bigK that are struck out one by one; more: a full sort
template <int NU>
static __device__ __forceinline__ uint32_t selw_cut(const uint64_t (&mine)[SELW_CAP_MAX / 64], uint32_t k)
{
    uint32_t cut = 0;
    for (int bit = 15; bit >= 0; bit--) {
        const uint32_t cand = cut | (1u << bit);
        uint32_t below = 0;
#pragma unroll
        for (int u = 0; u < NU; u++) below += (uint32_t)__popcll(__ballot((uint32_t)(mine[u] >> 32) < cand));
        if (below < k) cut = cand;
    }
    return cut;
}

__global__ __launch_bounds__(WG) void select_wave_kernel(IndexView v, MfmaScanArgs a, int cap)
{
    extern __shared__ __align__(16) uint64_t selw_keys[];      // [WG / 64][cap]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t q = (int64_t)blockIdx.x * (WG / 64) + wave;
    if (q >= a.nq) return;
    // the first 256 slots of the query's buffer (it has at least 1024) are requested together
    // with the count; slots beyond the count hold stale bits and are replaced below
    const uint64_t *sb = a.surv_buf + (size_t)q * a.surv_cap;
    uint64_t e_first[4];
#pragma unroll
    for (int u = 0; u < 4; u++) e_first[u] = sb[64 * u + lane];
    const uint32_t n = a.surv_cnt[q];
    // (queries that this kernel leaves to the two kernels behind it go on a list each, so that those
    // kernels, which normally have nothing to do, are a few workgroups looking at a count)
    if (n > (uint32_t)a.surv_cap || *a.log_overflow != 0u) {
        if (lane == 0) {
            a.flags[q] = 1;                 // redone by the exact kernel
            uint32_t *redo = a.work + 1 + a.nq;
            redo[1 + atomicAdd(&redo[0], 1u)] = (uint32_t)q;
        }
        return;
    }
    if (n > (uint32_t)cap) {                // the workgroup-wide select's case
        if (lane == 0) a.work[1 + atomicAdd(&a.work[0], 1u)] = (uint32_t)q;
        return;
    }
    if (lane == 0) a.flags[q] = 0;
    uint64_t *keys = selw_keys + (size_t)wave * cap;
    const uint32_t *bm = a.bitmap + (size_t)q * a.bmwords;
    for (uint32_t i0 = 0; i0 < n; i0 += 256) {
        uint64_t e[4];
        uint32_t id[4], Lb[4];
        int o[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const uint32_t i = i0 + 64 * u + lane;
            if (i0 == 0) e[u] = i < n ? e_first[u] : 0ull;      // slot 0 of block 0: read and discarded
            else e[u] = sb[i < n ? i : n - 1];
        }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const uint2 it = v.idtag[(uint32_t)e[u]];
            Lb[u] = (uint32_t)v.blk_list[(uint32_t)e[u] >> 5];      // the list that stores the block
            id[u] = it.x;
            o[u] = (int)it.y;
        }
        uint32_t bw[4];                     // the tags' probe-bitmap words, all fetched together
#pragma unroll
        for (int u = 0; u < 4; u++) bw[u] = bm[o[u] >= 0 ? o[u] >> 5 : 0];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const uint32_t i = i0 + 64 * u + lane;
            // a tagged item sits in a miscellaneous block, which is only ever scanned through the
            // list that stores it
            const uint32_t score = (uint32_t)(e[u] >> 48), L = Lb[u];
            bool keep = id[u] != RAIRS_EMPTY_ID;
            // RemoveVectorIfVisited: the item was already taken from list o
            if (keep && o[u] >= 0 && (uint32_t)o[u] < L && ((bw[u] >> (o[u] & 31)) & 1u)) keep = false;
            if (i < n) keys[i] = keep ? (((uint64_t)score << 32) | id[u]) : ~0ull;
        }
    }
    wave_lds_sync();
    // Only entries up to the score of the bigK-th best need sorting: take the kept keys back into
    // registers, find that score by bisection on its 16 bits, and pack the entries up to it.
    uint64_t mine[SELW_CAP_MAX / 64];
#pragma unroll
    for (int u = 0; u < SELW_CAP_MAX / 64; u++) {
        mine[u] = ~0ull;
        if (64 * u < (int)n) {                          // uniform
            const uint32_t i = 64 * u + lane;
            if (i < n) mine[u] = keys[i];
        }
    }
    // largest t with fewer than bigK scores below it (over the rows of 64 that hold entries)
    const uint32_t cut = n <= 128   ? selw_cut<2>(mine, (uint32_t)a.refine_k)
                         : n <= 256 ? selw_cut<4>(mine, (uint32_t)a.refine_k)
                         : n <= 512 ? selw_cut<8>(mine, (uint32_t)a.refine_k)
                                    : selw_cut<SELW_CAP_MAX / 64>(mine, (uint32_t)a.refine_k);
    // (dropped entries carry score 0xFFFFFFFF and are never below a candidate; with fewer than bigK
    // kept entries cut ends at 0xFFFF and everything kept is packed)
    wave_lds_sync();                                    // every lane has its keys in registers
    uint32_t m = 0;
#pragma unroll
    for (int u = 0; u < SELW_CAP_MAX / 64; u++) {
        if (64 * u < (int)n) {
            const bool in = (uint32_t)(mine[u] >> 32) <= cut;
            const unsigned long long bal = __ballot(in);
            if (in) keys[m + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull))] = mine[u];
            m += (uint32_t)__popcll(bal);
        }
    }
    // The whole search does not need the candidates in order (refine orders by exact distance):
    // of the m entries up to the cut all but m - bigK are results, and those few -- entries that
    // tie on the cut's score -- are struck out largest (score, id) first.
    if (a.any_order && (int)m - a.refine_k <= SELW_STRIKE_MAX) {
        wave_lds_sync();
        for (int extra = (int)m - a.refine_k; extra > 0; extra--) {
            uint64_t mine_max = 0ull;
            for (int i = lane; i < (int)m; i += 64) {
                const uint64_t x = keys[i];
                if (x != ~0ull && x > mine_max) mine_max = x;
            }
            const uint64_t largest = ~wave_min_u64(~mine_max);
            for (int i = lane; i < (int)m; i += 64)
                if (keys[i] == largest) keys[i] = ~0ull;     // keys are distinct: one lane, one slot
            wave_lds_sync();
        }
        uint32_t out = 0;
        for (int i0 = 0; i0 < (int)m; i0 += 64) {
            const int i = i0 + lane;
            const uint64_t key = i < (int)m ? keys[i] : ~0ull;
            const bool ok = key != ~0ull;
            const unsigned long long bal = __ballot(ok);
            if (ok) {
                const uint32_t pos = out + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
                a.cand_ids[(size_t)q * a.refine_k + pos] = (int64_t)(uint32_t)key;
                if (a.cand_score) a.cand_score[(size_t)q * a.refine_k + pos] = (int32_t)(key >> 32);
            }
            out += (uint32_t)__popcll(bal);
        }
        for (int i = (int)out + lane; i < a.refine_k; i += 64) {   // fewer than bigK entries exist
            a.cand_ids[(size_t)q * a.refine_k + i] = -1;
            if (a.cand_score) a.cand_score[(size_t)q * a.refine_k + i] = -1;
        }
        return;
    }
    const int n2 = next_pow2(m < 2 ? 2 : (int)m);
    for (int i = (int)m + lane; i < n2; i += 64) keys[i] = ~0ull;
    wave_lds_sync();
    wave_bitonic_sort_lds(keys, n2, lane);
    for (int i = lane; i < a.refine_k; i += 64) {
        const uint64_t key = i < n2 ? keys[i] : ~0ull;
        const bool ok = key != ~0ull;
        a.cand_ids[(size_t)q * a.refine_k + i] = ok ? (int64_t)(uint32_t)key : -1;
        if (a.cand_score) a.cand_score[(size_t)q * a.refine_k + i] = ok ? (int32_t)(key >> 32) : -1;
    }
}

// (Queries with more survivors than a wave holds are left on a list for the workgroup-wide select,
// select_wg.h, which runs in the launch behind this one together with the exact redo.)

// ---- the same scan with the tile's tables in LDS (any M up to 256) ----------------------------
//
// For tables too large for registers (M = 240: 30 KB per query pair of lanes) the waves of a
// workgroup (as many as LDS leaves room for, up to 16) share one tile: its tables sit in LDS as [K-step][lane] 16-byte operands, zero beyond
// the last subspace, and the waves take the unit's blocks round robin.  Each MFMA then reads both
// operands from LDS (one-hot row and table row), which holds it to about half the matrix-core
// rate; survivors, bounds and the log work exactly as in scan_mfma_kernel.
#define LDSK_MAX_ND 16      // code dwords per lane and block: M <= 256
#define LDSK_MAX_SEGS 32    // segments per unit: up to 4 parts of RAIRS_PART_SEGS segments
__global__ __launch_bounds__(1024, 1) void scan_mfma_lds_kernel(IndexView v, MfmaScanArgs a)
{
    extern __shared__ __align__(16) unsigned char dyn_lds[];
    __shared__ v4i onehot[16];
    __shared__ SegEntry segs_s[LDSK_MAX_SEGS];
    __shared__ uint32_t s_unit;
    const int ND = v.nd, KS = ND * 8;                   // K-steps incl. zero padding, ND <= LDSK_MAX_ND
    const int nthreads = blockDim.x, nwave = nthreads >> 6;
    v4i *Bl = (v4i *)dyn_lds;                           // [KS][64]
    StageQueue *stage = (StageQueue *)(dyn_lds + (size_t)KS * 64 * 16);   // [nwave]
    if (threadIdx.x < 16) {
        v4i r = {0, 0, 0, 0};
        const int sh = 1 << ((threadIdx.x & 3) * 8);
        if ((threadIdx.x >> 2) == 0) r.x = sh;
        if ((threadIdx.x >> 2) == 1) r.y = sh;
        if ((threadIdx.x >> 2) == 2) r.z = sh;
        if ((threadIdx.x >> 2) == 3) r.w = sh;
        onehot[threadIdx.x] = r;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5, j = lane & 31;
    StageQueue &sq = stage[wave];
    const int M = v.M, T = v.T;
    const int bias = 128 * M;
    int nstaged = 0;
    RefreshPace pace = {REFRESH_GAP_MIN, REFRESH_GAP_MIN - 1u, 0u};
    const uint32_t nunits = (uint32_t)a.toff[v.nlist];
    if (nunits == 0u) return;                          // uniform; nothing was written
    const uint32_t gwave = blockIdx.x * nwave + wave, nwaves = gridDim.x * nwave;
    LogCursor lc;
    lc.chunk = gwave;                                  // (a workgroup without a unit never writes)
    lc.next_v = gwave + log_active_waves(nunits, gridDim.x, (uint32_t)nwave);
    lc.used = 0;
    for (bool first = true;; first = false) {
        __syncthreads();                               // everyone is done with the previous tile
        if (threadIdx.x == 0) s_unit = first ? blockIdx.x : atomicAdd(a.next_task, 1u);
        __syncthreads();
        const uint32_t u = s_unit;
        if (u >= nunits) break;                        // uniform for the workgroup; the counter only grows
        const int L = a.unit_list[u];
        const ListEntry le = v.lists[L];
        const int rem = (int)u - a.toff[L];
        const int up = list_unit_parts(L, a.unit_parts, a.unit_tail_from);
        const int runs = (le.part_cnt + up - 1) / up;
        const int tile = rem / runs;
        const int p0 = (rem % runs) * up;
        const int p1 = p0 + up < le.part_cnt ? p0 + up : le.part_cnt;
        const int seg0 = v.parts[le.part_begin + p0] - le.seg_begin;
        const int seg1 = v.parts[le.part_begin + p1] - le.seg_begin;
        const int base = a.loff[L], nql = a.loff[L + 1] - base;
        const int nseg = seg1 - seg0;                  // <= LDSK_MAX_SEGS
        if ((int)threadIdx.x < nseg) segs_s[threadIdx.x] = v.segs[le.seg_begin + seg0 + threadIdx.x];
        // tables of the tile into LDS: operand (t, lane (j, g)) = lut[q_j][2t+g][0..15] - 128
        for (int e = threadIdx.x; e < KS * 64; e += nthreads) {
            const int t = e >> 6, ln = e & 63, jj = ln & 31, gg = ln >> 5;
            const int qi = tile * 32 + jj;
            v4i x = {0, 0, 0, 0};
            if (t < T && qi < nql) {
                const int qq = a.qlist[base + qi];
                x = *(const v4i *)(a.lut + (size_t)qq * (M * 16) + (size_t)(2 * t + gg) * 16);
                x ^= (v4i){(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
            }
            Bl[e] = x;
        }
        const int qi = tile * 32 + j;
        const int qid = qi < nql ? a.qlist[base + qi] : -1;
        const uint32_t hmul = hist_mul(qid >= 0 ? (uint32_t)a.tau[qid] : 0u);
        const int32_t *bq = a.bound + (qid >= 0 ? qid : 0);
        const uint32_t *bmq = a.bitmap + (size_t)(qid >= 0 ? qid : 0) * a.bmwords;
        __syncthreads();
        // The unit's blocks, numbered through its segments, are dealt to the waves in turn; a wave
        // fetches all code dwords of its next block (and that block's segment facts) while it
        // multiplies the current one.
        struct Blk { int valid, seg, b, blk, last; bool live; };
        int fpos = wave;                               // number of this wave's next block in the unit
        int wseg = 0, wbase = 0;                       // segment that holds it, blocks before that segment
        auto locate = [&]() {
            Blk r;
            r.valid = 0; r.seg = 0; r.b = 0; r.blk = 0; r.last = 0; r.live = false;
            while (wseg < nseg && fpos >= wbase + segs_s[wseg].nblk) { wbase += segs_s[wseg].nblk; wseg++; }
            if (wseg < nseg) {
                const int owner = segs_s[wseg].owner;
                r.valid = 1; r.seg = wseg; r.b = fpos - wbase;
                r.blk = segs_s[wseg].blk_begin + r.b;
                r.last = r.b == segs_s[wseg].nblk - 1;
                // cell (owner, L) is scored through list `owner` for queries that probe it
                const uint32_t ob = bmq[owner >= 0 ? owner >> 5 : 0];
                r.live = qid >= 0 && !(owner >= 0 && ((ob >> (owner & 31)) & 1u));
            }
            return r;
        };
        uint32_t cn[LDSK_MAX_ND];
        uint2 cmn = make_uint2(0u, 0u);
        uint32_t scored = 0;                           // items this lane's query was scored against, by this wave
        int bound_next = 0;
        auto fetch = [&](const Blk &bk) {
            const uint32_t *cp = v.codes + (size_t)bk.blk * ND * 64 + lane;
#pragma unroll
            for (int w = 0; w < LDSK_MAX_ND; w++)
                if (w < ND) cn[w] = cp[(size_t)w * 64];
            cmn = v.bmask[bk.blk];
            bound_next = __hip_atomic_load(bq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        };
        Blk cur = locate();
        if (cur.valid) fetch(cur);
        while (cur.valid) {
            uint32_t c[LDSK_MAX_ND];
#pragma unroll
            for (int w = 0; w < LDSK_MAX_ND; w++) c[w] = cn[w];
            const uint32_t cmask = cmn.x;
            const uint32_t blk_items = (uint32_t)__popc(cmn.y);
            const int negth = cur.live ? -(bound_next - bias + 1) : ACC_NEVER;
            fpos += nwave;
            const Blk nxt = locate();
            if (nxt.valid) fetch(nxt);
            if (__ballot(cur.live) != 0ull) {
                scored += cur.live ? blk_items : 0u;   // the block is contracted now: its DCO
                v16i acc;
#pragma unroll
                for (int r = 0; r < 16; r++) acc[r] = negth;
#pragma unroll
                for (int w = 0; w < LDSK_MAX_ND; w++) {
                    if (w < ND) {                      // uniform
                        const v4i *Bw = Bl + (size_t)w * 8 * 64 + lane;
#pragma unroll
                        for (int n = 0; n < 8; n++) {
                            const uint32_t nib = (c[w] >> (4 * n)) & 15u;
                            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(onehot[nib], Bw[n * 64], acc, 0, 0, 0);
                        }
                    }
                }
                uint32_t pm = negative_rows(acc);
                if (__ballot(pm != 0u) != 0ull) {
                    const uint32_t slot0 = (uint32_t)cur.blk * 32u + 4u * g;
                    const int tail_valid = segs_s[cur.seg].tail_valid;
                    if (cur.last && tail_valid < 32) {
#pragma unroll
                        for (int r = 0; r < 16; r++)
                            if (8 * (r >> 2) + 4 * g + (r & 3) >= tail_valid) pm &= ~(1u << r);
                    }
                    for (;;) {
                        const bool has = pm != 0u;
                        const unsigned long long mask = __ballot(has);
                        if (mask == 0ull) break;
                        if (has) {
                            const int r = __builtin_ctz(pm);
                            pm &= pm - 1u;
                            int s8[8], s4[4];
#pragma unroll
                            for (int k = 0; k < 8; k++) s8[k] = (r & 1) ? acc[2 * k + 1] : acc[2 * k];
#pragma unroll
                            for (int k = 0; k < 4; k++) s4[k] = (r & 2) ? s8[2 * k + 1] : s8[2 * k];
                            const int s2a = (r & 4) ? s4[1] : s4[0], s2b = (r & 4) ? s4[3] : s4[2];
                            const int sc = ((r & 8) ? s2b : s2a) - negth;
                            const int pos = nstaged + lanes_below(mask);
                            const uint32_t item = 8u * (uint32_t)(r >> 2) + (uint32_t)(r & 3);   // + 4 g
                            sq.ent[pos] = make_uint2((slot0 + item) | (((cmask >> (item + 4u * g)) & 1u) << 31),
                                                     ((uint32_t)(sc + bias) << 16) | (uint32_t)qid);
                            sq.hmul[pos] = hmul;
                        }
                        nstaged += __popcll(mask);
                        if (nstaged > STAGE_CAP - 64) {
                            stage_flush(a, sq, nstaged, lane, lc, pace);
                            nstaged = 0;
                        }
                    }
                }
            }
            cur = nxt;
        }
        if (nstaged >= 32) {
            stage_flush(a, sq, nstaged, lane, lc, pace);
            nstaged = 0;
        }
        if (a.dco && g == 0 && scored) atomicAdd(&a.dco[qid], (unsigned long long)scored);
    }
    if (nstaged > 0) stage_flush(a, sq, nstaged, lane, lc, pace);
    // (a wave that never had a unit wrote nothing, and the chunk of its index may be another wave's)
    if (lane == 0 && lc.used > 0 && lc.chunk < (uint32_t)a.log_chunks) a.chunk_fill[lc.chunk] = lc.used;
}

// ---- the bound sample on the matrix cores -----------------------------------------------------
//
// The sample that seeds a query's bound is the head of its first probed list.  Queries that share
// a first list are scored together: one workgroup groups the batch by first list, then a wave
// scores the head of a list for a tile of up to 32 such queries with the scan's matrix
// instruction, and writes every (query, item) score out for the rank kernel.  About ten queries
// share a first list in a 10,000-query batch over 1,024 lists, so the tiles are a third full --
// still several times cheaper than one table lookup per code on the vector units.
#define SAMPLE_GROUP_MAX_NLIST 8192
#define SAMPLE_GROUP_MIN_QUERIES 1024
#define SG_HELD 12

// s_off: exclusive prefix over lists of the queries whose first probe is the list; s_q: those
// queries, list by list; s_toff: exclusive prefix of tiles (32 queries); s_tiles: list of every tile.
__global__ __launch_bounds__(1024) void sample_group_kernel(const int32_t *__restrict__ probe_ids,
                                                            int64_t nq, int nprobe, int nlist,
                                                            int32_t *s_off, int32_t *s_toff,
                                                            int32_t *s_q, int32_t *s_tiles)
{
    extern __shared__ int32_t sg_lds[];                // [nlist] counts, then cursors; [nlist] offsets
    __shared__ int sc[16], st[16];
    int32_t *cnt_s = sg_lds, *off_s = sg_lds + nlist;
    const int tid = threadIdx.x;
    for (int i = tid; i < nlist; i += 1024) cnt_s[i] = 0;
    __syncthreads();
    // the first SG_HELD queries of a thread stay in registers: their loads are all in flight at
    // once and the second pass does not fetch them again
    int myL[SG_HELD];
#pragma unroll
    for (int k = 0; k < SG_HELD; k++) {
        const int64_t q = tid + 1024 * k;
        int L = q < nq ? probe_ids[q * nprobe] : -1;
        myL[k] = L >= 0 && L < nlist ? L : -1;
    }
#pragma unroll
    for (int k = 0; k < SG_HELD; k++)
        if (myL[k] >= 0) atomicAdd(&cnt_s[myL[k]], 1);
    for (int64_t q = tid + 1024 * SG_HELD; q < nq; q += 1024) {
        const int L = probe_ids[q * nprobe];
        if (L >= 0 && L < nlist) atomicAdd(&cnt_s[L], 1);
    }
    __syncthreads();
    const int per = (nlist + 1023) / 1024;
    const int lo = tid * per < nlist ? tid * per : nlist;
    const int hi = lo + per < nlist ? lo + per : nlist;
    int c = 0, t = 0;
    for (int L = lo; L < hi; L++) {
        const int n = cnt_s[L];
        c += n;
        t += (n + 31) >> 5;
    }
    // exclusive prefixes of (c, t) over the 1024 threads: a scan inside each wave, then the totals
    // of the 16 waves through LDS
    const int lane = tid & 63, wave = tid >> 6;
    int ci = c, ti = t;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int x = __shfl_up(ci, off), y = __shfl_up(ti, off);
        if (lane >= off) { ci += x; ti += y; }
    }
    if (lane == 63) { sc[wave] = ci; st[wave] = ti; }
    __syncthreads();
    int cw = 0, tw = 0, call = 0, tall = 0;
#pragma unroll
    for (int w2 = 0; w2 < 16; w2++) {
        const int x = sc[w2], y = st[w2];
        if (w2 < wave) { cw += x; tw += y; }
        call += x;
        tall += y;
    }
    int cb = cw + ci - c, tb = tw + ti - t;
    for (int L = lo; L < hi; L++) {
        const int n = cnt_s[L], nt = (n + 31) >> 5;
        s_off[L] = cb;
        off_s[L] = cb;
        s_toff[L] = tb;
        for (int u = 0; u < nt; u++) s_tiles[tb + u] = L;
        cb += n;
        tb += nt;
    }
    if (tid == 0) {
        s_off[nlist] = call;
        s_toff[nlist] = tall;
    }
    __syncthreads();
    for (int i = tid; i < nlist; i += 1024) cnt_s[i] = 0;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < SG_HELD; k++)
        if (myL[k] >= 0) s_q[off_s[myL[k]] + atomicAdd(&cnt_s[myL[k]], 1)] = tid + 1024 * k;
    for (int64_t q = tid + 1024 * SG_HELD; q < nq; q += 1024) {
        const int L = probe_ids[q * nprobe];
        if (L >= 0 && L < nlist) s_q[off_s[L] + atomicAdd(&cnt_s[L], 1)] = (int32_t)q;
    }
}

// scores[q][b * 32 + i] = score of item i of block b of the first `sample_blocks` own blocks of
// q's first list (0xFFFF: the slot holds no item); blocks the list does not have are not written.
template <int T>
__global__ __launch_bounds__(WG) void sample_mfma_kernel(IndexView v, const uint8_t *__restrict__ lut,
                                                            int sample_blocks,
                                                            const int32_t *__restrict__ s_off,
                                                            const int32_t *__restrict__ s_toff,
                                                            const int32_t *__restrict__ s_q,
                                                            const int32_t *__restrict__ s_tiles,
                                                            uint16_t *__restrict__ scores)
{
    constexpr int ND = (T + 7) / 8;
    constexpr int M = 2 * T;
    constexpr int TS = T / 2;
    __shared__ uint2 sparse_tab[32];                   // as in scan_mfma_kernel
    fill_sparse_tab(sparse_tab);
    __syncthreads();
    const int lane = threadIdx.x & 63, g = lane >> 5, j = lane & 31;
    const uint32_t bias = 128u * M;
    const uint32_t ntiles = (uint32_t)s_toff[v.nlist];
    const uint32_t gwave = blockIdx.x * (WG / 64) + (threadIdx.x >> 6), nwaves = gridDim.x * (WG / 64);
    v8i B[TS];
    for (uint32_t u = gwave; u < ntiles; u += nwaves) {
        const int L = __builtin_amdgcn_readfirstlane(s_tiles[u]);
        const ListEntry le = v.lists[L];
        const int tile = (int)u - __builtin_amdgcn_readfirstlane(s_toff[L]);
        const int base = s_off[L], n = s_off[L + 1] - base;
        const int qi = tile * 32 + j;
        const int qid = qi < n ? s_q[base + qi] : -1;
        {
            const uint8_t *lq = lut + (size_t)(qid >= 0 ? qid : 0) * (M * 16) + g * 32;
            const int keep = qid >= 0 ? -1 : 0;
            const v4i flip = {(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
            const v4i keep4 = {keep, keep, keep, keep};
#pragma unroll
            for (int t = 0; t < TS; t++) {
                const v4i x = (*(const v4i *)(lq + t * 64) ^ flip) & keep4;
                const v4i y = (*(const v4i *)(lq + t * 64 + 16) ^ flip) & keep4;
                B[t] = (v8i){x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
            }
        }
        int cnt = le.shared_cnt + le.misc_cnt;
        cnt = cnt < sample_blocks ? cnt : sample_blocks;
        if (cnt <= 0) continue;                        // uniform for the wave
        const uint32_t *cp = v.codes + (size_t)le.blk_begin * ND * 64 + lane;
        uint32_t cn[ND];
#pragma unroll
        for (int w = 0; w < ND; w++) cn[w] = cp[w * 64];
        uint32_t vmn = v.vmask[le.blk_begin];
        uint16_t *row = scores + (size_t)(qid >= 0 ? qid : 0) * sample_blocks * 32;
        for (int b = 0; b < cnt; b++) {
            uint32_t c[ND];
#pragma unroll
            for (int w = 0; w < ND; w++) c[w] = cn[w];
            const uint32_t vm = vmn;
            if (b + 1 < cnt) {
#pragma unroll
                for (int w = 0; w < ND; w++) cn[w] = cp[(size_t)(b + 1) * ND * 64 + w * 64];
                vmn = v.vmask[le.blk_begin + b + 1];
            }
            // the accumulators start at the bias of the signed table entries, so they end as the
            // scores themselves (below 2^16)
            v16i acc;
#pragma unroll
            for (int r = 0; r < 16; r++) acc[r] = (int)bias;
#define CODE_LO(t_) ((c[(t_) >> 2] >> (8 * ((t_) & 3))) & 15u)
#define CODE_HI(t_) ((c[(t_) >> 2] >> (8 * ((t_) & 3) + 4)) & 15u)
#define LOAD_A(t_)                                                                        \
    do {                                                                                  \
        const uint2 *e1_ = &sparse_tab[CODE_LO(t_)], *e2_ = &sparse_tab[CODE_HI(t_)];      \
        v1[t_] = e1_[0]; v2[t_] = e2_[0];                                                 \
        p1[t_] = e1_[16].x; p2[t_] = e2_[16].y;                                           \
    } while (0)
            uint2 v1[TS], v2[TS];
            uint32_t p1[TS], p2[TS];
            LOAD_A(0);
            if (TS > 1) LOAD_A(1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < TS; t++) {
                const v4i av = {(int)v1[t].x, (int)v1[t].y, (int)v2[t].x, (int)v2[t].y};
                acc = __builtin_amdgcn_smfmac_i32_32x32x64_i8(av, B[t], acc, (int)(p1[t] | p2[t]), 0, 0);
                if (t + 2 < TS) LOAD_A(t + 2);
                __builtin_amdgcn_sched_barrier(0);
            }
#undef LOAD_A
#undef CODE_LO
#undef CODE_HI
            // acc[r]: item 8 * (r / 4) + 4 * g + r % 4, query column j: four consecutive items
            // per group of four registers, written as one 8-byte store.  A block whose 32 slots
            // all hold items (every block but a list's last, unless items were deleted) needs no
            // look at the slot mask: two scores to a word and out.
            if (qid >= 0) {
                if (vm == 0xFFFFFFFFu) {               // uniform
#pragma unroll
                    for (int k = 0; k < 4; k++)
                        *(uint2 *)(row + b * 32 + 8 * k + 4 * g) =
                            make_uint2((uint32_t)acc[4 * k] | ((uint32_t)acc[4 * k + 1] << 16),
                                       (uint32_t)acc[4 * k + 2] | ((uint32_t)acc[4 * k + 3] << 16));
                } else {
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        const int item = 8 * k + 4 * g;
                        uint32_t sc4[4];
#pragma unroll
                        for (int e = 0; e < 4; e++)
                            sc4[e] = ((vm >> (item + e)) & 1u) ? (uint32_t)acc[4 * k + e] : 0xFFFFu;
                        *(uint2 *)(row + b * 32 + item) = make_uint2(sc4[0] | (sc4[1] << 16), sc4[2] | (sc4[3] << 16));
                    }
                }
            }
        }
    }
}

bool rairs_sample_scores_supported(const IndexView &v, int64_t nq)
{
    return (v.T == 8 || v.T == 24 || v.T == 32) && v.nlist <= SAMPLE_GROUP_MAX_NLIST &&
           nq >= SAMPLE_GROUP_MIN_QUERIES;
}

int rairs_launch_sample_group(const IndexView &v, const int32_t *probe_ids, int nprobe, int64_t nq,
                              int32_t *s_off, int32_t *s_toff, int32_t *s_q, int32_t *s_tiles,
                              hipStream_t s)
{
    if (!rairs_sample_scores_supported(v, nq)) {
        rairs_set_error("matrix-core sample not available for this index or batch");
        return RAIRS_EINVAL;
    }
    const size_t lds = (size_t)2 * v.nlist * 4;
    if (lds > 32 * 1024)
        RAIRS_HIP(hipFuncSetAttribute((const void *)sample_group_kernel,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(sample_group_kernel, dim3(1), dim3(1024), lds, s, probe_ids, nq, nprobe, v.nlist,
                       s_off, s_toff, s_q, s_tiles);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

int rairs_launch_sample_scores(const IndexView &v, const uint8_t *lut, int sample_blocks, int64_t nq,
                               const int32_t *s_off, const int32_t *s_toff, const int32_t *s_q,
                               const int32_t *s_tiles, uint16_t *scores, hipStream_t s)
{
    if (!rairs_sample_scores_supported(v, nq) || sample_blocks < 1 || sample_blocks > RAIRS_SAMPLE_MAX_BLOCKS) {
        rairs_set_error("matrix-core sample not available for this index or batch");
        return RAIRS_EINVAL;
    }
    const int64_t tiles_max = nq / 32 + v.nlist;
    unsigned grid = (unsigned)((tiles_max + WG / 64 - 1) / (WG / 64));
    if (grid > 512u) grid = 512u;
#define SAMPLE_MFMA(T_)                                                                           \
    hipLaunchKernelGGL(sample_mfma_kernel<T_>, dim3(grid), dim3(WG), 0, s, v, lut, sample_blocks, s_off, \
                       s_toff, s_q, s_tiles, scores)
    switch (v.T) {
    case 8: SAMPLE_MFMA(8); break;
    case 24: SAMPLE_MFMA(24); break;
    default: SAMPLE_MFMA(32); break;
    }
#undef SAMPLE_MFMA
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

bool rairs_mfma_supported(const IndexView &v)
{
    return v.T >= 1 && v.nd * 8 * 64 * 16 <= 128 * 1024;    // tables of a tile must fit 128 KB of LDS
}

bool rairs_mfma_reg_tables(const IndexView &v) { return v.T == 8 || v.T == 24 || v.T == 32; }

// persistent grids: 256 compute units x 2 workgroups of 4 waves with the tables in registers; one
// workgroup per compute unit, with as many waves as LDS leaves room for, with the tables in LDS
static void scan_launch_shape(const IndexView &v, bool *reg_tables, unsigned *grid, int *lds_waves,
                              size_t *table_bytes)
{
    *reg_tables = rairs_mfma_reg_tables(v);
    *grid = *reg_tables ? 512u : 256u;
    *table_bytes = (size_t)v.nd * 8 * 64 * 16;
    int w = 16;
    while (w > 4 && *table_bytes + (size_t)w * sizeof(StageQueue) > 158 * 1024) w >>= 1;
    *lds_waves = w;
}

// Most waves that can own chunks of the survivor log at once when the pass has at most `units` units.
int64_t rairs_scan_log_waves(const IndexView &v, int64_t units)
{
    bool reg_tables;
    unsigned gridx;
    int lds_waves;
    size_t table_bytes;
    scan_launch_shape(v, &reg_tables, &gridx, &lds_waves, &table_bytes);
    if (reg_tables) return units < (int64_t)gridx * (WG / 64) ? units : (int64_t)gridx * (WG / 64);
    return (units < (int64_t)gridx ? units : (int64_t)gridx) * lds_waves;
}

int rairs_launch_group(const IndexView &v, const MfmaScanArgs &a, hipStream_t s)
{
    const int np = a.nprobe - a.p_first;
    if (np <= 0) return RAIRS_OK;
    bool reg_tables;
    unsigned gridx;
    int lds_waves;
    size_t table_bytes;
    scan_launch_shape(v, &reg_tables, &gridx, &lds_waves, &table_bytes);
    const uint32_t nwaves = gridx * (reg_tables ? WG / 64 : lds_waves);
    // who starts on a unit of its own index, and with how many waves (see log_active_waves)
    const uint32_t starters = reg_tables ? nwaves : gridx, waves_each = reg_tables ? 1u : (uint32_t)lds_waves;
    if (a.log_chunks < 2) {
        rairs_set_error("survivor log of %d chunks", a.log_chunks);
        return RAIRS_EINVAL;
    }
    const int64_t pairs = a.nq * np;
    int64_t nz = v.nlist > a.nq ? v.nlist : a.nq;
    nz = nz > a.log_chunks ? nz : a.log_chunks;
    hipLaunchKernelGGL(lm_zero_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, s, a.lcount,
                       a.lcursor, v.nlist, a.next_task, a.surv_cnt, a.nq, a.chunk_fill, a.log_chunks,
                       a.log_cursor, a.log_overflow, reg_tables ? 2 * nwaves : gridx, a.dco, a.work);
    const bool lds_group = v.nlist <= LM_LDS_NLIST;
    const int qb = LM_PAIRS / np > 0 ? LM_PAIRS / np : 1;
    const unsigned lgrid = (unsigned)((a.nq + qb - 1) / qb);
    if (lds_group) {
        if ((size_t)v.nlist * 4 > 48 * 1024)
            RAIRS_HIP(hipFuncSetAttribute((const void *)lm_count_lds_kernel,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, v.nlist * 4));
        hipLaunchKernelGGL(lm_count_lds_kernel, dim3(lgrid), dim3(256), (size_t)v.nlist * 4, s,
                           a.probe_ids, a.nq, a.nprobe, a.p_first, v.nlist, a.lcount, qb);
    } else
        hipLaunchKernelGGL(lm_count_kernel, dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, s,
                           a.probe_ids, a.nq, a.nprobe, a.p_first, v.nlist, a.lcount);
    if (lds_group) {
        const size_t lds = ((size_t)2 * v.nlist + 1) * 4;
        if (lds > 48 * 1024)
            RAIRS_HIP(hipFuncSetAttribute((const void *)lm_fill_lds_kernel,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(lm_fill_lds_kernel, dim3(lgrid + LM_UNIT_WGS), dim3(256), lds, s, v, a.probe_ids, a.nq,
                           a.nprobe, a.p_first, a.lcount, a.loff, a.lcursor, a.qlist, qb, a.toff,
                           a.unit_list, a.unit_parts, a.unit_tail_from, a.unit_rec, a.log_cursor, starters, waves_each);
    } else {
        hipLaunchKernelGGL(lm_prefix_kernel, dim3(1), dim3(1024), 0, s, v, a.lcount, a.loff, a.lcursor,
                           a.toff, a.unit_list, a.unit_parts, a.unit_tail_from, a.unit_rec, a.log_cursor, starters, waves_each);
        hipLaunchKernelGGL(lm_units_kernel, dim3((unsigned)((v.nlist + 255) / 256)), dim3(256), 0, s, v, a.lcount,
                           a.loff, a.toff, a.unit_list, a.unit_parts, a.unit_tail_from, a.unit_rec);
        hipLaunchKernelGGL(lm_fill_kernel, dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, s,
                           a.probe_ids, a.nq, a.nprobe, a.p_first, v.nlist, a.loff, a.lcursor, a.qlist);
    }
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

int rairs_launch_scan_mfma(const IndexView &v, const MfmaScanArgs &a, hipStream_t s, hipEvent_t *ev)
{
    if (a.nprobe - a.p_first <= 0) return RAIRS_OK;
    if (a.surv_cap > SURV_CAP_MAX) {
        rairs_set_error("survivor capacity %d above %d", a.surv_cap, SURV_CAP_MAX);
        return RAIRS_EINVAL;
    }
    if (a.nq > 65536) {                                // a log entry has 16 bits for the query of the pass
        rairs_set_error("a scan pass takes at most 65536 queries, got %lld", (long long)a.nq);
        return RAIRS_EINVAL;
    }
    bool reg_tables;
    unsigned gridx;
    int lds_waves;
    size_t table_bytes;
    scan_launch_shape(v, &reg_tables, &gridx, &lds_waves, &table_bytes);
    const dim3 grid(gridx);
    if (ev) RAIRS_HIP(hipEventRecord(ev[0], s));
    switch (v.T) {
    case 8: hipLaunchKernelGGL(scan_mfma_kernel<8>, grid, dim3(WG), 0, s, v, a); break;
    case 24: hipLaunchKernelGGL(scan_mfma_kernel<24>, grid, dim3(WG), 0, s, v, a); break;
    case 32: hipLaunchKernelGGL(scan_mfma_kernel<32>, grid, dim3(WG), 0, s, v, a); break;
    default: {
        const size_t lds = table_bytes + (size_t)lds_waves * sizeof(StageQueue);
        RAIRS_HIP(hipFuncSetAttribute((const void *)scan_mfma_lds_kernel,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(scan_mfma_lds_kernel, grid, dim3(64 * lds_waves), lds, s, v, a);
    }
    }
    if (ev) RAIRS_HIP(hipEventRecord(ev[1], s));
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

int rairs_launch_select(const IndexView &v, const MfmaScanArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL(collect_kernel, dim3((unsigned)(a.log_chunks < 4096 ? a.log_chunks : 4096)),
                       dim3(COLLECT_WG), 0, s, a);
    const int cap = rairs_select_wave_cap(a.refine_k);
    hipLaunchKernelGGL(select_wave_kernel, dim3((unsigned)((a.nq + WG / 64 - 1) / (WG / 64))), dim3(WG),
                       (size_t)cap * 8 * (WG / 64), s, v, a, cap);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}
