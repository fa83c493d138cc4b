// Exact SEIL scan with a bounded top-bigK queue, one workgroup per query (SeilSearch, Alg. 5,
// with rqueue).  Used for the first probed list of every query (which also yields the score bound
// for the MFMA scan), as the whole scan for table shapes the MFMA kernel is not built for, and as
// the fallback for queries whose survivor buffer overflowed.
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

__global__ __launch_bounds__(WG) void scan_exact_kernel(IndexView v, ExactScanArgs a)
{
    __shared__ ScanShared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t qi = blockIdx.x;
    if (a.only_flagged && a.only_flagged[qi] == 0) return;
    const int nprobe = a.nprobe, refine_k = a.refine_k;
    for (int i = tid; i < v.M * 16; i += WG) sh.lut[i] = a.lut[(size_t)qi * v.M * 16 + i];
    for (int i = tid; i < a.bmwords; i += WG) sh.bm[i] = a.bitmap[(size_t)qi * a.bmwords + i];
    if (tid == 0) { sh.tau = ~0ull; sh.cnt = 0; sh.dco = 0; }
    __syncthreads();

    // items that the probes beyond p_scan will score (they are scanned by another kernel):
    // every valid slot of the list's own blocks plus 32 per block of each unskipped reference
    unsigned long long my_dco = 0;
    for (int p = (a.sample_blocks > 0 ? 0 : a.p_scan) + tid; p < nprobe; p += WG) {
        const int L = a.probe_ids[(size_t)qi * nprobe + p];
        if (L < 0 || L >= v.nlist) continue;
        const ListEntry le = v.lists[L];
        unsigned long long c = (unsigned long long)le.valid_items;
        for (int r = 0; r < le.ref_cnt; r++) {
            const RefEntry re = v.refs[le.ref_begin + r];
            if (!((sh.bm[re.owner >> 5] >> (re.owner & 31)) & 1u)) c += 32ull * re.nblocks;
        }
        my_dco += c;
    }
    if (my_dco) atomicAdd(&sh.dco, my_dco);
    my_dco = 0;

    const bool sample = a.sample_blocks > 0;
    const int p_scan = sample ? 1 : (a.p_scan < nprobe ? a.p_scan : nprobe);
    for (int p = 0; p < p_scan; p++) {
        const int L = a.probe_ids[(size_t)qi * nprobe + p];
        if (L < 0 || L >= v.nlist) continue;              // caller-supplied ids: never index with them unchecked
        const ListEntry le = v.lists[L];
        // segment -1: the list's own blocks; segments 0..ref_cnt-1: its reference entries
        const int nseg = sample ? 0 : le.ref_cnt;
        for (int seg = -1; seg < nseg; seg++) {
            int64_t begin;
            int cnt, misc_from;
            if (seg < 0) {
                begin = le.blk_begin;
                cnt = le.shared_cnt + le.misc_cnt;
                misc_from = le.shared_cnt;
                if (sample) {
                    // any valid item of the list's own blocks is a distinct member of the probed
                    // set, duplicate rule or not: enough for a bound
                    cnt = cnt < a.sample_blocks ? cnt : a.sample_blocks;
                    misc_from = cnt;
                }
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
    if (sample) {
        if (tid == 0) {
            const int32_t t = n == refine_k ? (int32_t)(sh.buf[refine_k - 1] >> 32) : 0xFFFF;
            a.tau[qi] = t;
            if (a.bound) a.bound[qi] = t;
        }
        my_dco = 0;                                  // the sampled blocks are scored again, and counted, by the main scan
    } else if (a.surv_buf) {
        // hand the queue over to the MFMA scan: its entries seed the query's survivor buffer and
        // the bigK-th smallest score bounds what any other item needs to reach
        const uint32_t tau0 = n == refine_k ? (uint32_t)(sh.buf[refine_k - 1] >> 32) : 0xFFFFu;
        const uint32_t range = tau0 == 0xFFFFu ? 255u * (uint32_t)v.M : tau0;
        for (int i = tid; i < n; i += WG) {
            uint64_t key = sh.buf[i];
            a.surv_buf[(size_t)qi * a.surv_cap + i] = key;
            uint32_t bin = (((uint32_t)(key >> 32)) * RAIRS_HIST_BINS) / (range + 1u);
            atomicAdd(&a.hist[(size_t)qi * RAIRS_HIST_BINS + bin], 1u);
        }
        if (tid == 0) {
            a.surv_cnt[qi] = (uint32_t)n;
            a.tau[qi] = (int32_t)tau0;
        }
    } else {
        for (int i = tid; i < refine_k; i += WG) {
            uint64_t key = sh.buf[i];
            bool ok = i < n;
            a.cand_ids[(size_t)qi * refine_k + i] = ok ? (int64_t)(uint32_t)key : -1;
            if (a.cand_score) a.cand_score[(size_t)qi * refine_k + i] = ok ? (int32_t)(key >> 32) : -1;
        }
    }
    if (a.dco) {
        if (lane == 0 && my_dco) atomicAdd(&sh.dco, my_dco);
        __syncthreads();
        if (tid == 0) a.dco[qi] = (int64_t)sh.dco;
    }
}

int rairs_launch_scan_exact(const IndexView &v, const ExactScanArgs &a, int64_t nq, hipStream_t s)
{
    hipLaunchKernelGGL(scan_exact_kernel, dim3((unsigned)nq), dim3(WG), 0, s, v, a);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}
