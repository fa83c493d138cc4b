// C ABI of librairs: argument checks, index upload into the device format, workspace and the
// stage sequence of RairsSearch (Alg. 2).  No kernel code here.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "rairs_common.h"

static thread_local char g_err[512] = "";

void rairs_set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char *rairs_last_error(void) { return g_err; }

#define FAIL(code, ...)              \
    do {                             \
        rairs_set_error(__VA_ARGS__); \
        return (code);               \
    } while (0)

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int dev_alloc(rairs_index *h, void **p, size_t bytes)
{
    if (bytes == 0) bytes = 16;
    hipError_t e = hipMalloc(p, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        FAIL(RAIRS_ENOMEM, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
    }
    h->dev_alloc[h->ndev_alloc++] = *p;
    h->total_bytes += (int64_t)bytes;
    return RAIRS_OK;
}

static void destroy(rairs_index *h)
{
    if (!h) return;
    for (int i = 0; i < h->ndev_alloc; i++) (void)hipFree(h->dev_alloc[i]);
    if (h->ws) (void)hipFree(h->ws);
    if (h->ev_ready)
        for (int r = 0; r < RAIRS_EV_RING; r++)
            for (int i = 0; i < 2 * RAIRS_NSTAGES; i++) (void)hipEventDestroy(h->ev[r][i]);
    if (h->side_ready) {
        (void)hipEventDestroy(h->ev_fork); (void)hipEventDestroy(h->ev_lut);
        (void)hipEventDestroy(h->ev_probe); (void)hipEventDestroy(h->ev_group);
        (void)hipEventDestroy(h->ev_scored);
        (void)hipStreamDestroy(h->side);
    }
    delete h;
}

static int validate(const rairs_host_index_t *x)
{
    if (!x) FAIL(RAIRS_EINVAL, "host index is NULL");
    if (x->nbits != 4) FAIL(RAIRS_EINVAL, "nbits must be 4, got %d", x->nbits);
    if (x->metric != RAIRS_METRIC_L2 && x->metric != RAIRS_METRIC_IP) FAIL(RAIRS_EINVAL, "unknown metric %d", x->metric);
    if (x->blk != 32) FAIL(RAIRS_EINVAL, "blk must be 32, got %d", x->blk);
    if (x->d <= 0 || x->M <= 0 || x->d % x->M != 0 || (x->M & 1))
        FAIL(RAIRS_EINVAL, "need d > 0, M > 0 even, d %% M == 0 (d=%d M=%d)", x->d, x->M);
    if (255 * (int64_t)x->M > 65535) FAIL(RAIRS_EINVAL, "255*M exceeds 16 bits (M=%d)", x->M);
    if (x->M > RAIRS_MAX_M) FAIL(RAIRS_EUNSUPPORTED, "M=%d above the built limit %d", x->M, RAIRS_MAX_M);
    if (x->d > RAIRS_MAX_D) FAIL(RAIRS_EUNSUPPORTED, "d=%d above the built limit %d", x->d, RAIRS_MAX_D);
    if (x->nlist <= 0) FAIL(RAIRS_EINVAL, "nlist must be positive");
    if (x->nlist > RAIRS_MAX_NLIST) FAIL(RAIRS_EUNSUPPORTED, "nlist=%d above the built limit %d", x->nlist, RAIRS_MAX_NLIST);
    if (x->ntotal < 0 || x->ntotal >= 0xFFFFFFFFll) FAIL(RAIRS_EINVAL, "ntotal out of range");
    if (x->nblocks < 0 || x->nblocks > 0x7FFFFFFFll / 64) FAIL(RAIRS_EINVAL, "nblocks out of range");
    if (x->nrefs < 0 || x->nrefs > 0x7FFFFFFFll) FAIL(RAIRS_EINVAL, "nrefs out of range");
    if (!x->centroids || !x->codebook || !x->list_shared_begin || !x->list_shared_cnt ||
        !x->list_misc_begin || !x->list_misc_cnt || !x->list_ref_begin || !x->list_ref_cnt)
        FAIL(RAIRS_EINVAL, "null array in host index");
    if (x->nblocks > 0 && (!x->codes || !x->ids || !x->other)) FAIL(RAIRS_EINVAL, "null block arrays");
    if (x->nrefs > 0 && (!x->ref_owner || !x->ref_block_begin || !x->ref_nblocks))
        FAIL(RAIRS_EINVAL, "null reference arrays");
    if (x->ntotal > 0 && !x->raw) FAIL(RAIRS_EINVAL, "null raw vectors");
    for (int l = 0; l < x->nlist; l++) {
        int64_t sb = x->list_shared_begin[l], mb = x->list_misc_begin[l], rb = x->list_ref_begin[l];
        int64_t sc = x->list_shared_cnt[l], mc = x->list_misc_cnt[l], rc = x->list_ref_cnt[l];
        if (sc < 0 || mc < 0 || rc < 0 || sb < 0 || sb + sc > x->nblocks || mb != sb + sc ||
            mb + mc > x->nblocks || rb < 0 || rb + rc > x->nrefs)
            FAIL(RAIRS_EINVAL, "directory of list %d out of bounds", l);
    }
    // a block belongs to at most one list
    std::vector<int32_t> blk_owner((size_t)x->nblocks, -1);
    for (int l = 0; l < x->nlist; l++) {
        const int64_t b0 = x->list_shared_begin[l], b1 = b0 + x->list_shared_cnt[l] + x->list_misc_cnt[l];
        for (int64_t b = b0; b < b1; b++) {
            if (blk_owner[(size_t)b] >= 0)
                FAIL(RAIRS_EINVAL, "block %lld belongs to lists %d and %d", (long long)b, blk_owner[(size_t)b], l);
            blk_owner[(size_t)b] = l;
        }
    }
    // reference entries of list l: cells (owner, l) with owner < l (Section 5.1), inside the
    // owner's shared blocks
    for (int l = 0; l < x->nlist; l++)
        for (int64_t r = x->list_ref_begin[l]; r < x->list_ref_begin[l] + x->list_ref_cnt[l]; r++) {
            int32_t o = x->ref_owner[r];
            if (o < 0 || o >= l)
                FAIL(RAIRS_EINVAL, "reference %lld of list %d: owner %d is not a smaller list id", (long long)r, l, o);
            int64_t b = x->ref_block_begin[r], n = x->ref_nblocks[r];
            int64_t ob = x->list_shared_begin[o], oc = x->list_shared_cnt[o];
            if (n < 1 || b < ob || b + n > ob + oc)
                FAIL(RAIRS_EINVAL, "reference %lld does not point into its owner's shared blocks", (long long)r);
        }
    // a shared block may hold invalidated slots anywhere (deletion leaves them); the miscellaneous
    // items of a list are dense: only the tail of its last block is empty
    for (int l = 0; l < x->nlist; l++) {
        const int64_t b0 = x->list_misc_begin[l];
        const int64_t b1 = b0 + x->list_misc_cnt[l];
        bool seen_empty = false;
        for (int64_t i = b0 * 32; i < b1 * 32; i++) {
            const bool empty = x->ids[i] < 0;
            if ((empty && i < (b1 - 1) * 32) || (!empty && seen_empty))
                FAIL(RAIRS_EINVAL, "list %d: empty miscellaneous slots must be the tail of its last block", l);
            seen_empty |= empty;
        }
    }
    // Every vector is stored either once in a shared block (no tag), or once in the miscellaneous
    // area of its only list (tag = that list), or as twins in the miscellaneous areas of its two
    // lists, same code, each tagged with the other list (Section 5.1).  The scan relies on this:
    // an item that the duplicate rule drops in one list is queued from the other.
    // first[id]: -1 not seen, -2 complete, else the slot of a tagged item that waits for its twin.
    std::vector<int32_t> first((size_t)x->ntotal, -1);
    const int hb = x->M / 2;
    for (int l = 0; l < x->nlist; l++) {
        const int64_t b0 = x->list_shared_begin[l], bs = b0 + x->list_shared_cnt[l];
        const int64_t b1 = bs + x->list_misc_cnt[l];
        for (int64_t i = b0 * 32; i < b1 * 32; i++) {
            const int64_t id = x->ids[i];
            const int32_t o = x->other[i];
            if (id < -1 || id >= x->ntotal) FAIL(RAIRS_EINVAL, "id out of range in slot %lld", (long long)i);
            if (o < -1 || o >= x->nlist) FAIL(RAIRS_EINVAL, "list tag out of range in slot %lld", (long long)i);
            if (id < 0) continue;
            int32_t &f = first[(size_t)id];
            if (i < bs * 32) {
                if (o != -1) FAIL(RAIRS_EINVAL, "slot %lld of a shared block carries a list tag", (long long)i);
                if (f != -1) FAIL(RAIRS_EINVAL, "vector %lld is stored in a shared block and elsewhere", (long long)id);
                f = -2;
            } else if (o == l) {
                if (f != -1) FAIL(RAIRS_EINVAL, "vector %lld of cell (%d, %d) is stored more than once", (long long)id, l, l);
                f = -2;
            } else {
                if (o < 0) FAIL(RAIRS_EINVAL, "miscellaneous slot %lld has no list tag", (long long)i);
                if (f == -1) {
                    f = (int32_t)i;
                } else {
                    if (f < 0) FAIL(RAIRS_EINVAL, "vector %lld is stored more often than its cell allows", (long long)id);
                    const int64_t t = f;               // the twin seen earlier
                    if (blk_owner[(size_t)(t >> 5)] != o || x->other[t] != l ||
                        memcmp(x->codes + (size_t)t * hb, x->codes + (size_t)i * hb, (size_t)hb) != 0)
                        FAIL(RAIRS_EINVAL, "miscellaneous slots %lld and %lld of vector %lld are not twins "
                             "(lists, tags or codes differ)", (long long)t, (long long)i, (long long)id);
                    f = -2;
                }
            }
        }
    }
    for (int64_t id = 0; id < x->ntotal; id++)
        if (first[(size_t)id] >= 0)
            FAIL(RAIRS_EINVAL, "vector %lld in slot %d is tagged with another list but has no twin there",
                 (long long)id, first[(size_t)id]);
    // slots of blocks that no list owns are never read
    return RAIRS_OK;
}

static int upload_impl(const rairs_host_index_t *x, void *hip_stream, rairs_index_t **out, rairs_index **made)
{
    int rc = validate(x);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    rairs_index *h = new (std::nothrow) rairs_index();
    if (!h) FAIL(RAIRS_ENOMEM, "out of host memory");
    memset(h, 0, sizeof(*h));
    *made = h;                                         // released by the caller if anything below throws
    IndexView &v = h->v;
    v.d = x->d; v.M = x->M; v.T = x->M / 2; v.nd = (v.T + 7) / 8; v.nlist = x->nlist;
    v.raw_u8 = x->raw_is_u8 ? 1 : 0;
    v.metric = x->metric;
    v.ntotal = x->ntotal; v.nblocks = x->nblocks; v.nrefs = x->nrefs;

#define UP_CHECK(call)            \
    do {                          \
        int rc_ = (call);         \
        if (rc_) { *made = nullptr; destroy(h); return rc_; } \
    } while (0)
#define UP_HIP(call)                                                                  \
    do {                                                                              \
        hipError_t e_ = (call);                                                       \
        if (e_ != hipSuccess) {                                                       \
            rairs_set_error("%s failed: %s", #call, hipGetErrorString(e_));           \
            *made = nullptr;                                                          \
            destroy(h);                                                               \
            return RAIRS_EHIP;                                                        \
        }                                                                             \
    } while (0)

    float *cent = nullptr, *cent_t = nullptr, *cb = nullptr;
    uint32_t *codes = nullptr, *ids = nullptr;
    int32_t *other = nullptr;
    ListEntry *lists = nullptr;
    RefEntry *refs = nullptr;
    void *raw = nullptr;
    const size_t cent_bytes = (size_t)x->nlist * x->d * sizeof(float);
    const size_t cb_bytes = (size_t)x->M * 16 * (x->d / x->M) * sizeof(float);
    h->code_bytes = (int64_t)x->nblocks * v.nd * 64 * 4;
    // fp32 raw vectors whose components are all integers in [0, 255] (SIFT-like data) are kept
    // as bytes: the conversion back is exact, so refined distances do not change, and a
    // candidate row is a quarter of the bytes to gather
    std::vector<uint8_t> narrow;
    const void *raw_src = x->raw;
    if (!v.raw_u8 && x->ntotal > 0) {
        const float *rf = (const float *)x->raw;
        const size_t n = (size_t)x->ntotal * x->d;
        bool bytes_ok = true;
        for (size_t i = 0; i < n && bytes_ok; i++) {
            const float f = rf[i];
            bytes_ok = f >= 0.0f && f <= 255.0f && f == (float)(int)f;
        }
        if (bytes_ok) {
            narrow.resize(n);
            for (size_t i = 0; i < n; i++) narrow[i] = (uint8_t)(int)rf[i];
            raw_src = narrow.data();
            v.raw_u8 = 1;
        }
    }
    const size_t raw_bytes = (size_t)x->ntotal * x->d * (v.raw_u8 ? 1 : 4);
    float *cnorm = nullptr;
    UP_CHECK(dev_alloc(h, (void **)&cent, cent_bytes));
    UP_CHECK(dev_alloc(h, (void **)&cent_t, cent_bytes));
    UP_CHECK(dev_alloc(h, (void **)&cnorm, (size_t)x->nlist * sizeof(float)));
    UP_CHECK(dev_alloc(h, (void **)&cb, cb_bytes));
    UP_CHECK(dev_alloc(h, (void **)&codes, (size_t)h->code_bytes));
    UP_CHECK(dev_alloc(h, (void **)&ids, (size_t)x->nblocks * 32 * 4));
    UP_CHECK(dev_alloc(h, (void **)&other, (size_t)x->nblocks * 32 * 4));
    UP_CHECK(dev_alloc(h, (void **)&lists, (size_t)x->nlist * sizeof(ListEntry)));
    UP_CHECK(dev_alloc(h, (void **)&refs, (size_t)x->nrefs * sizeof(RefEntry)));
    UP_CHECK(dev_alloc(h, &raw, raw_bytes));

    // centroids: row-major for the re-scoring of shortlisted lists and transposed to [d][nlist] so
    // that lanes walking over lists read coalesced.  The GEMM form works on centred copies,
    // c' = fl(c - mean of the centroids): distances do not change, but the rounding-error margin
    // scales with |q'|^2 + |c'|^2, which centring makes as small as the data allow.
    std::vector<float> hmean((size_t)x->d), hct((size_t)x->nlist * x->d), hn((size_t)x->nlist);
    for (int i = 0; i < x->d; i++) {
        double m = 0.0;
        for (int l = 0; l < x->nlist; l++) m += (double)x->centroids[(size_t)l * x->d + i];
        // inner products are not invariant under a common shift: no centring, and no norm term
        hmean[(size_t)i] = x->metric == RAIRS_METRIC_IP ? 0.0f : (float)(m / x->nlist);
    }
    double nmax = 0.0;
    for (int l = 0; l < x->nlist; l++) {
        double n2 = 0.0;
        for (int i = 0; i < x->d; i++) {
            const float c = x->centroids[(size_t)l * x->d + i] - hmean[(size_t)i];
            hct[(size_t)i * x->nlist + l] = c;
            n2 += (double)c * (double)c;
        }
        hn[(size_t)l] = x->metric == RAIRS_METRIC_IP ? 0.0f : (float)n2;
        if (n2 > nmax) nmax = n2;
    }
    v.cmax2 = (float)nmax;
    float *cent_ct = nullptr, *cmean = nullptr;
    UP_CHECK(dev_alloc(h, (void **)&cent_ct, cent_bytes));
    UP_CHECK(dev_alloc(h, (void **)&cmean, (size_t)x->d * sizeof(float)));
    hipError_t e = hipSuccess;
    UP_HIP(hipMemcpyAsync(cent, x->centroids, cent_bytes, hipMemcpyHostToDevice, s));
    UP_HIP(hipMemcpyAsync(cent_ct, hct.data(), cent_bytes, hipMemcpyHostToDevice, s));
    UP_HIP(hipMemcpyAsync(cmean, hmean.data(), (size_t)x->d * sizeof(float), hipMemcpyHostToDevice, s));
    UP_HIP(hipMemcpyAsync(cnorm, hn.data(), hn.size() * sizeof(float), hipMemcpyHostToDevice, s));
    UP_CHECK(rairs_launch_transpose(cent, x->nlist, x->d, cent_t, s));
    UP_HIP(hipStreamSynchronize(s));
    v.centroids_ct = cent_ct; v.cmean = cmean;
    UP_HIP(hipMemcpyAsync(cb, x->codebook, cb_bytes, hipMemcpyHostToDevice, s));
    if (x->nblocks)
        UP_HIP(hipMemcpyAsync(other, x->other, (size_t)x->nblocks * 32 * 4, hipMemcpyHostToDevice, s));
    if (raw_bytes) UP_HIP(hipMemcpyAsync(raw, raw_src, raw_bytes, hipMemcpyHostToDevice, s));
    if (!narrow.empty()) {
        UP_HIP(hipStreamSynchronize(s));               // the staging copy goes away
        std::vector<uint8_t>().swap(narrow);
    }

    // directory
    std::vector<ListEntry> hl((size_t)x->nlist);
    for (int l = 0; l < x->nlist; l++) {
        ListEntry &e2 = hl[(size_t)l];
        e2.blk_begin = (int32_t)x->list_shared_begin[l];
        e2.shared_cnt = x->list_shared_cnt[l];
        e2.misc_cnt = x->list_misc_cnt[l];
        e2.ref_begin = (int32_t)x->list_ref_begin[l];
        e2.ref_cnt = x->list_ref_cnt[l];
        int64_t valid = 0;
        const int64_t b0 = x->list_shared_begin[l], b1 = b0 + x->list_shared_cnt[l] + x->list_misc_cnt[l];
        for (int64_t i = b0 * 32; i < b1 * 32; i++) valid += x->ids[i] >= 0;
        e2.valid_items = (int32_t)valid;
    }
    std::vector<int32_t> hbl((size_t)x->nblocks, -1);
    for (int l = 0; l < x->nlist; l++) {
        const int64_t b0 = x->list_shared_begin[l], b1 = b0 + x->list_shared_cnt[l] + x->list_misc_cnt[l];
        for (int64_t b = b0; b < b1; b++) hbl[(size_t)b] = l;
    }
    std::vector<uint32_t> hm((size_t)x->nblocks, 0u), hv((size_t)x->nblocks, 0u);
    for (int64_t b = 0; b < x->nblocks; b++) {
        uint32_t m = 0;
        for (int i = 0; i < 32; i++) m |= (uint32_t)(x->ids[b * 32 + i] >= 0) << i;
        hv[(size_t)b] = m;
    }
    for (int l = 0; l < x->nlist; l++) {
        const int64_t b0 = x->list_shared_begin[l], bs = b0 + x->list_shared_cnt[l];
        const int64_t b1 = bs + x->list_misc_cnt[l];
        for (int64_t b = b0; b < b1; b++) {
            uint32_t m = 0;
            for (int i = 0; i < 32; i++) {
                const int64_t at = b * 32 + i;
                if (x->ids[at] < 0) continue;
                const int32_t o = x->other[at];
                if (b < bs || o < 0 || o >= l) m |= 1u << i;
            }
            hm[(size_t)b] = m;
        }
    }
    std::vector<RefEntry> hr((size_t)x->nrefs);
    for (int64_t r = 0; r < x->nrefs; r++) {
        hr[(size_t)r].owner = x->ref_owner[r];
        hr[(size_t)r].blk_begin = (int32_t)x->ref_block_begin[r];
        hr[(size_t)r].nblocks = x->ref_nblocks[r];
        int32_t valid = 0;
        for (int64_t b = x->ref_block_begin[r]; b < x->ref_block_begin[r] + x->ref_nblocks[r]; b++)
            valid += __builtin_popcount(hv[(size_t)b]);
        hr[(size_t)r].valid = valid;
    }
    // scan segments: the list's own blocks, then each referenced cell, in runs of <= 16 blocks
    std::vector<SegEntry> hs;
    std::vector<int32_t> hp;
    for (int l = 0; l < x->nlist; l++) {
        ListEntry &e2 = hl[(size_t)l];
        e2.seg_begin = (int32_t)hs.size();
        const int own = e2.shared_cnt + e2.misc_cnt;
        for (int b = 0; b < own; b += RAIRS_SEG_BLOCKS) {
            SegEntry se;
            se.blk_begin = e2.blk_begin + b;
            se.nblk = own - b < RAIRS_SEG_BLOCKS ? own - b : RAIRS_SEG_BLOCKS;
            int mf = e2.shared_cnt - b;
            se.misc_from = mf < 0 ? 0 : (mf > se.nblk ? se.nblk : mf);
            se.owner = -1;
            // the list's very last block usually ends in empty slots: the scan drops those rows
            // early; any other empty slot (an invalidated item) is dropped when ids are read
            se.tail_valid = 32;
            if (b + se.nblk == own) {
                const uint32_t m = hv[(size_t)(e2.blk_begin + own - 1)];
                if ((m & (m + 1u)) == 0u) se.tail_valid = __builtin_popcount(m);
            }
            hs.push_back(se);
        }
        for (int r = 0; r < e2.ref_cnt; r++) {
            const RefEntry &re = hr[(size_t)e2.ref_begin + r];
            for (int b = 0; b < re.nblocks; b += RAIRS_SEG_BLOCKS) {
                SegEntry se;
                se.blk_begin = re.blk_begin + b;
                se.nblk = re.nblocks - b < RAIRS_SEG_BLOCKS ? re.nblocks - b : RAIRS_SEG_BLOCKS;
                se.misc_from = se.nblk;
                se.owner = re.owner;
                se.tail_valid = 32;
                hs.push_back(se);
            }
        }
        e2.seg_cnt = (int32_t)hs.size() - e2.seg_begin;
        // parts: consecutive segments of about RAIRS_PART_BLOCKS blocks, the scan's unit of work
        e2.part_begin = (int32_t)hp.size();
        int in_blocks = 0, in_segs = 0;
        for (int sidx = e2.seg_begin; sidx < e2.seg_begin + e2.seg_cnt; sidx++) {
            const int nb = hs[(size_t)sidx].nblk;
            if (in_segs == 0 || in_blocks + nb > RAIRS_PART_BLOCKS || in_segs == RAIRS_PART_SEGS) {
                hp.push_back(sidx);
                in_blocks = 0;
                in_segs = 0;
            }
            in_blocks += nb;
            in_segs++;
        }
        e2.part_cnt = (int32_t)hp.size() - e2.part_begin;
        hp.push_back(e2.seg_begin + e2.seg_cnt);
    }
    h->nsegs = (int64_t)hs.size();
    h->max_parts = 1;
    for (int l = 0; l < x->nlist; l++)
        if (hl[(size_t)l].part_cnt > h->max_parts) h->max_parts = hl[(size_t)l].part_cnt;
    int32_t *parts = nullptr;
    UP_CHECK(dev_alloc(h, (void **)&parts, hp.size() * sizeof(int32_t)));
    if (!hp.empty())
        UP_HIP(hipMemcpyAsync(parts, hp.data(), hp.size() * sizeof(int32_t), hipMemcpyHostToDevice, s));
    h->nparts = (int64_t)hp.size() - x->nlist;
    SegEntry *segs = nullptr;
    UP_CHECK(dev_alloc(h, (void **)&segs, hs.size() * sizeof(SegEntry)));
    if (!hs.empty())
        UP_HIP(hipMemcpyAsync(segs, hs.data(), hs.size() * sizeof(SegEntry), hipMemcpyHostToDevice, s));
    uint32_t *cmask = nullptr, *vmask = nullptr;
    uint2 *bmask = nullptr;
    int32_t *blk_list = nullptr;
    UP_CHECK(dev_alloc(h, (void **)&cmask, (size_t)x->nblocks * 4));
    UP_CHECK(dev_alloc(h, (void **)&vmask, (size_t)x->nblocks * 4));
    UP_CHECK(dev_alloc(h, (void **)&blk_list, (size_t)x->nblocks * 4));
    UP_CHECK(dev_alloc(h, (void **)&bmask, (size_t)x->nblocks * 8));
    std::vector<uint2> hbm((size_t)x->nblocks);
    for (int64_t b = 0; b < x->nblocks; b++) hbm[(size_t)b] = make_uint2(hm[(size_t)b], hv[(size_t)b]);
    if (x->nblocks) {
        UP_HIP(hipMemcpyAsync(bmask, hbm.data(), hbm.size() * 8, hipMemcpyHostToDevice, s));
        UP_HIP(hipMemcpyAsync(blk_list, hbl.data(), hbl.size() * 4, hipMemcpyHostToDevice, s));
        UP_HIP(hipMemcpyAsync(cmask, hm.data(), hm.size() * 4, hipMemcpyHostToDevice, s));
        UP_HIP(hipMemcpyAsync(vmask, hv.data(), hv.size() * 4, hipMemcpyHostToDevice, s));
    }
    UP_HIP(hipMemcpyAsync(lists, hl.data(), hl.size() * sizeof(ListEntry), hipMemcpyHostToDevice, s));
    if (x->nrefs)
        UP_HIP(hipMemcpyAsync(refs, hr.data(), hr.size() * sizeof(RefEntry), hipMemcpyHostToDevice, s));

    // blocks: staged in chunks in the canonical layout, repacked on the device
    if (x->nblocks) {
        const int64_t chunk = 1 << 16;   // blocks per staging chunk
        const size_t cbytes = (size_t)chunk * 32 * v.T;
        uint8_t *st_codes = nullptr;
        int64_t *st_ids = nullptr;
        UP_HIP(hipMalloc((void **)&st_codes, cbytes));
        e = hipMalloc((void **)&st_ids, (size_t)chunk * 32 * 8);
        if (e != hipSuccess) { (void)hipFree(st_codes); UP_HIP(e); }
        int r2 = RAIRS_OK;
        for (int64_t b0 = 0; b0 < x->nblocks && e == hipSuccess && r2 == RAIRS_OK; b0 += chunk) {
            int64_t nb = x->nblocks - b0 < chunk ? x->nblocks - b0 : chunk;
            e = hipMemcpyAsync(st_codes, x->codes + (size_t)b0 * 32 * v.T, (size_t)nb * 32 * v.T,
                               hipMemcpyHostToDevice, s);
            if (e == hipSuccess)
                e = hipMemcpyAsync(st_ids, x->ids + (size_t)b0 * 32, (size_t)nb * 32 * 8,
                                   hipMemcpyHostToDevice, s);
            if (e == hipSuccess) r2 = rairs_launch_pack(st_codes, st_ids, b0, nb, v.M, v.nd, codes, ids, s);
            if (e == hipSuccess) e = hipStreamSynchronize(s);
        }
        (void)hipFree(st_codes);
        (void)hipFree(st_ids);
        if (r2) { *made = nullptr; destroy(h); return r2; }
        UP_HIP(e);
    }
    uint2 *idtag = nullptr;
    UP_CHECK(dev_alloc(h, (void **)&idtag, (size_t)x->nblocks * 32 * 8));
    UP_CHECK(rairs_launch_pair_ids(ids, other, x->nblocks * 32, idtag, s));
    UP_HIP(hipStreamSynchronize(s));

    v.idtag = idtag;
    v.centroids = cent; v.cnorm = cnorm; v.centroids_t = cent_t; v.codebook = cb; v.codes = codes; v.ids = ids; v.other = other; v.cmask = cmask; v.vmask = vmask; v.bmask = bmask; v.blk_list = blk_list;
    v.lists = lists; v.refs = refs; v.segs = segs; v.parts = parts; v.raw = raw;
    for (int r = 0; r < RAIRS_EV_RING; r++)
        for (int i = 0; i < 2 * RAIRS_NSTAGES; i++) UP_HIP(hipEventCreate(&h->ev[r][i]));
    h->ev_ready = 1;
    // default priority, like every stream here
    UP_HIP(hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking));
    UP_HIP(hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming));
    UP_HIP(hipEventCreateWithFlags(&h->ev_lut, hipEventDisableTiming));
    UP_HIP(hipEventCreateWithFlags(&h->ev_probe, hipEventDisableTiming));
    UP_HIP(hipEventCreateWithFlags(&h->ev_group, hipEventDisableTiming));
    UP_HIP(hipEventCreateWithFlags(&h->ev_scored, hipEventDisableTiming));
    h->side_ready = 1;
    *made = nullptr;
    *out = h;
    return RAIRS_OK;
}

extern "C" int rairs_index_upload(const rairs_host_index_t *x, void *hip_stream, rairs_index_t **out)
{
    if (!out) FAIL(RAIRS_EINVAL, "out is NULL");
    *out = nullptr;
    rairs_index *made = nullptr;
    try {
        return upload_impl(x, hip_stream, out, &made);
    } catch (const std::bad_alloc &) {
        destroy(made);
        FAIL(RAIRS_ENOMEM, "out of host memory while preparing the index");
    }
}

extern "C" int rairs_free(rairs_index_t *h)
{
    destroy(h);
    return RAIRS_OK;
}

extern "C" int rairs_index_bytes(const rairs_index_t *h, int64_t *code_bytes, int64_t *total_bytes)
{
    if (!h) FAIL(RAIRS_EINVAL, "handle is NULL");
    if (code_bytes) *code_bytes = h->code_bytes;
    if (total_bytes) *total_bytes = h->total_bytes;
    return RAIRS_OK;
}

// ---- workspace ------------------------------------------------------------------------------

#define RAIRS_SAMPLE_BLOCKS 16

// Survivor buffer entries per query (entries at or below the query's final bound; more than this
// sends the query to the exact kernel) and survivor log entries per query on average (the scan logs
// about bigK ln(items / sample) entries per query; if the log runs out, every query of the pass
// is redone by the exact kernel).
static int surv_cap_for(int refine_k)
{
    int c = 1024;
    while (c < 8 * refine_k && c < 4096) c <<= 1;
    return c;
}

static int log_per_query_for(int refine_k)
{
    const int n = 16 * refine_k;
    return n < 1024 ? 1024 : (n > 8192 ? 8192 : n);
}

struct WsLayout {
    size_t dmat, cflags, probe_ids, probe_dists, bitmap, lut, cand, dco;
    size_t lcount, loff, lcursor, toff, unit_list, unit_rec, next_task, qlist, tau, bound, surv_cnt, flags, work, hist, surv_buf, log, chunk_fill, log_misc, total;
    size_t s_off, s_toff, s_q, s_tiles, s_scores, s_first;      // matrix-core sample (0 bytes when not used)
    int sample_blocks;
    int log_chunks;
    int surv_cap;
    int bmwords;
};

// Blocks of the first probed list that seed a query's bound: several times bigK items, so that the
// bigK-th smallest of them is a low quantile.  A larger sample starts the scan with a tighter bound
// (fewer survivors staged and logged) but the sample sits on the critical path.  With the bound
// kernel scoring it, ten times bigK pays up to about 1,024 items (measured: 32 blocks beat 16 and
// 48 at bigK = 100, 63 beat 96 at bigK = 400); scored on the matrix cores it is cheaper and
// fifteen times, up to about 1,536 items, is better (48 blocks beat 32 and 64 at bigK = 100).  With
// more than 64 sub-quantizers an item costs the bound kernel so much that five times is all that pays.
// The matrix-core route pays when tiles of queries sharing a first list are not too thin (at
// least four queries per list on average) and the sample is large enough to cover its two extra
// launches (bigK >= 64); measured on 10,000-query batches: 1,024 lists and bigK = 100 gain 2-3 %,
// 4,096 lists (2.4 queries per list) or bigK = 10 lose about as much.
static bool grouped_sample(const IndexView &v, int64_t nq, int refine_k)
{
    return rairs_sample_scores_supported(v, nq) && nq >= 4 * (int64_t)v.nlist && refine_k >= 64;
}

static int sample_blocks_for(const IndexView &v, int refine_k, bool grouped)
{
    const int times = grouped ? 15 : v.M <= 64 ? 10 : 5, most = grouped ? 1536 : 1024;
    int items = times * refine_k < most ? times * refine_k : most;
    if (items < 5 * refine_k) items = 5 * refine_k;
    int blocks = (items + 31) / 32;
    if (blocks < RAIRS_SAMPLE_BLOCKS) blocks = RAIRS_SAMPLE_BLOCKS;
    return blocks < RAIRS_SAMPLE_MAX_BLOCKS ? blocks : RAIRS_SAMPLE_MAX_BLOCKS;
}

// Workspace of one pass of `nq` queries out of a batch of `nq_total` (the DCO counts cover the
// batch).  Two pairs of buffers whose lifetimes never overlap on the caller's stream share their
// bytes: the coarse quantizer's score matrix (dead once the probe lists exist) with the survivor log
// (first written by the scan kernel), and the sample's scores (dead once the bounds exist) with
// the survivor buffers (first written after the scan).
static WsLayout ws_layout(const IndexView &v, int64_t nq, int64_t nq_total, int nprobe, int refine_k,
                          int max_parts = 1)
{
    WsLayout w;
    w.bmwords = (v.nlist + 31) / 32;
    size_t off = 0;
    auto take = [&off](size_t bytes) { size_t at = off; off = align_up(off + bytes, 256); return at; };
    w.cflags = take((size_t)nq * 4);
    w.probe_ids = take((size_t)nq * nprobe * 4);
    w.probe_dists = take((size_t)nq * nprobe * 4);
    w.bitmap = take((size_t)nq * w.bmwords * 4);
    w.lut = take((size_t)nq * v.M * 16);
    w.cand = take((size_t)nq * refine_k * 8);
    w.dco = take((size_t)nq_total * 8);
    w.lcount = take((size_t)v.nlist * 4);
    w.loff = take((size_t)(v.nlist + 1) * 4);
    w.lcursor = take((size_t)v.nlist * 4);
    w.toff = take((size_t)(v.nlist + 1) * 4);
    w.next_task = take(4);
    w.unit_list = take(((size_t)nq * nprobe / 32 + (size_t)v.nlist) * (size_t)max_parts * 4);   // max_parts = most parts in a list
    w.unit_rec = take(((size_t)nq * nprobe / 32 + (size_t)v.nlist) * (size_t)max_parts * 32);
    w.qlist = take((size_t)nq * nprobe * 4);
    w.tau = take((size_t)nq * 4);
    w.bound = take((size_t)nq * 4);
    w.surv_cnt = take((size_t)nq * 4);
    w.flags = take((size_t)nq * 4);
    w.hist = take((size_t)nq * RAIRS_HIST_BINS * 4);
    w.work = take((size_t)2 * (1 + nq) * 4);
    w.surv_cap = surv_cap_for(refine_k);
    {
        // Chunks of RAIRS_LOG_CHUNK entries; a wave moves on when its next flush (up to 128 entries)
        // does not fit, and every wave that gets a unit holds a current and a reserved chunk.
        const int64_t units = (nq * nprobe < nq * nprobe / 32 + v.nlist ? nq * nprobe : nq * nprobe / 32 + v.nlist) *
                              (int64_t)(max_parts > 0 ? max_parts : 1);
        const int64_t active = rairs_scan_log_waves(v, units);
        w.log_chunks = (int)((nq * log_per_query_for(refine_k) + RAIRS_LOG_CHUNK - 128) / (RAIRS_LOG_CHUNK - 127) +
                             2 * active + 16);
    }
    w.chunk_fill = take((size_t)w.log_chunks * 4);
    w.log_misc = take(64);
    const bool grouped = grouped_sample(v, nq, refine_k);
    w.sample_blocks = sample_blocks_for(v, refine_k, grouped);
    w.s_off = take(grouped ? (size_t)(v.nlist + 1) * 4 : 0);
    w.s_toff = take(grouped ? (size_t)(v.nlist + 1) * 4 : 0);
    w.s_q = take(grouped ? (size_t)nq * 4 : 0);
    w.s_first = take(grouped ? (size_t)nq * 4 : 0);
    w.s_tiles = take(grouped ? ((size_t)nq / 32 + (size_t)v.nlist + 1) * 4 : 0);
    const size_t dmat_bytes = (size_t)nq * v.nlist * 4, log_bytes = (size_t)w.log_chunks * RAIRS_LOG_CHUNK * 8;
    w.dmat = w.log = take(dmat_bytes > log_bytes ? dmat_bytes : log_bytes);
    const size_t samp_bytes = grouped ? (size_t)nq * w.sample_blocks * 64 : 0;
    const size_t surv_bytes = (size_t)nq * w.surv_cap * 8;
    w.s_scores = w.surv_buf = take(samp_bytes > surv_bytes ? samp_bytes : surv_bytes);
    w.total = off;
    return w;
}

// ---- the no-allocation entry point's scratch ------------------------------------------------
//
// rairs_search_noalloc runs in this array instead of a workspace that somebody allocated: one copy
// per GPU the library runs on, held until the process ends.  The array's name is only a host-side
// stand-in; the device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[RAIRS_NOALLOC_SCRATCH_BYTES];
#define RAIRS_MAX_DEVICES 64
static void *g_scratch_ptr[RAIRS_MAX_DEVICES];

static int scratch_pointer(void **out)
{
    int dev = -1;
    RAIRS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= RAIRS_MAX_DEVICES) FAIL(RAIRS_EUNSUPPORTED, "device ordinal %d above the built limit", dev);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        RAIRS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) FAIL(RAIRS_EHIP, "hipGetSymbolAddress returned no address for the scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return RAIRS_OK;
}

// Where a call's workspace comes from.  WS_HANDLE: the caller's buffer if one was set (too small:
// RAIRS_EWORKSPACE, nothing is allocated or synchronised), else the handle's own, grown on demand.
// WS_STATIC: the scratch array.
enum { WS_HANDLE = 0, WS_STATIC = 1, WS_GRAPH = 2 };
static int acquire_ws(rairs_index *h, int source, size_t bytes, char **ws)
{
    if (source == WS_GRAPH) {                          // the workspace of the graph being captured
        if (bytes > h->graph_ws_bytes) FAIL(RAIRS_EWORKSPACE, "graph workspace too small");
        *ws = (char *)h->graph_ws;
        h->last_ws = *ws;
        return RAIRS_OK;
    }
    if (source == WS_STATIC) {
        if (bytes > (size_t)RAIRS_NOALLOC_SCRATCH_BYTES)
            FAIL(RAIRS_EWORKSPACE, "this call needs %zu bytes of scratch memory, the static array has %zu",
                 bytes, (size_t)RAIRS_NOALLOC_SCRATCH_BYTES);
        void *p = nullptr;
        int rc = scratch_pointer(&p);
        if (rc) return rc;
        *ws = (char *)p;
        h->last_ws = *ws;
        return RAIRS_OK;
    }
    if (h->ws_user) {
        if (bytes > h->ws_user_bytes)
            FAIL(RAIRS_EWORKSPACE, "this call needs a workspace of %zu bytes, the caller's has %zu", bytes,
                 h->ws_user_bytes);
        *ws = (char *)h->ws_user;
        h->last_ws = *ws;
        return RAIRS_OK;
    }
    if (h->ws_bytes < bytes) {
        if (h->ws) { RAIRS_HIP(hipDeviceSynchronize()); (void)hipFree(h->ws); h->ws = nullptr; h->ws_bytes = 0; }
        hipError_t e = hipMalloc(&h->ws, bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            FAIL(RAIRS_ENOMEM, "workspace of %zu bytes: %s", bytes, hipGetErrorString(e));
        }
        h->ws_bytes = bytes;
    }
    *ws = (char *)h->ws;
    h->last_ws = *ws;
    return RAIRS_OK;
}

static int check_common(const rairs_index *h, int64_t nq)
{
    if (!h) FAIL(RAIRS_EINVAL, "handle is NULL");
    if (nq < 0) FAIL(RAIRS_EINVAL, "nq is negative");
    if (nq > 0x7FFFFFFFll / 4) FAIL(RAIRS_EUNSUPPORTED, "nq too large for one call");
    return RAIRS_OK;
}

static int check_nprobe(const rairs_index *h, int nprobe)
{
    if (nprobe < 1 || nprobe > h->v.nlist) FAIL(RAIRS_EINVAL, "nprobe=%d outside [1, nlist=%d]", nprobe, h->v.nlist);
    if (nprobe > RAIRS_MAX_NPROBE) FAIL(RAIRS_EUNSUPPORTED, "nprobe=%d above the built limit %d", nprobe, RAIRS_MAX_NPROBE);
    return RAIRS_OK;
}

static int check_k(int k, int refine_k)
{
    if (k < 1 || k > refine_k) FAIL(RAIRS_EINVAL, "need 1 <= k <= refine_k (k=%d refine_k=%d)", k, refine_k);
    if (refine_k > RAIRS_MAX_REFINE_K) FAIL(RAIRS_EUNSUPPORTED, "refine_k=%d above the built limit %d", refine_k, RAIRS_MAX_REFINE_K);
    return RAIRS_OK;
}

// Queries per internal pass: the pass's workspace stays within about 4 GiB, and a pass has at most
// 65,536 queries (a survivor log entry has 16 bits for the query of the pass).
static int64_t pass_size(const IndexView &v, int64_t nq, int nprobe, int refine_k)
{
    const int64_t score_row = (int64_t)v.nlist * 4, log_row = (int64_t)log_per_query_for(refine_k) * 8;
    const int64_t per_q = (score_row > log_row ? score_row : log_row) + (int64_t)surv_cap_for(refine_k) * 8 +
                          (int64_t)v.M * 16 + (int64_t)refine_k * 8 + (int64_t)nprobe * 12 +
                          (int64_t)((v.nlist + 31) / 32) * 4 + RAIRS_HIST_BINS * 4 + 64;
    int64_t cap = (4ll << 30) / per_q;
    if (cap < 256) cap = 256;
    if (cap > 65536) cap = 65536;
    return nq < cap ? nq : cap;
}

// ---- stages -----------------------------------------------------------------------------------

extern "C" int rairs_coarse(rairs_index_t *h, const float *d_queries, int64_t nq, int nprobe,
                            int32_t *d_probe_ids, float *d_probe_dists, void *hip_stream)
{
    int rc = check_common(h, nq);
    if (rc) return rc;
    if ((rc = check_nprobe(h, nprobe))) return rc;
    if (nq == 0) return RAIRS_OK;
    if (!d_queries || !d_probe_ids) FAIL(RAIRS_EINVAL, "null device pointer");
    const int64_t step = pass_size(h->v, nq, nprobe, 1);
    const WsLayout w = ws_layout(h->v, step, 0, nprobe, 1);
    char *ws = nullptr;
    if ((rc = acquire_ws(h, WS_HANDLE, w.total, &ws))) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    for (int64_t q0 = 0; q0 < nq; q0 += step) {
        int64_t n = nq - q0 < step ? nq - q0 : step;
        rc = rairs_launch_coarse(h->v, d_queries + (size_t)q0 * h->v.d, n, nprobe,
                                 (float *)(ws + w.dmat), d_probe_ids + (size_t)q0 * nprobe,
                                 d_probe_dists ? d_probe_dists + (size_t)q0 * nprobe : nullptr,
                                 (uint32_t *)(ws + w.cflags), s);
        if (rc) return rc;
    }
    return RAIRS_OK;
}

extern "C" int rairs_lut(rairs_index_t *h, const float *d_queries, int64_t nq, uint8_t *d_lut,
                         float *d_bias_sum, float *d_scale, void *hip_stream)
{
    int rc = check_common(h, nq);
    if (rc) return rc;
    if (nq == 0) return RAIRS_OK;
    if (!d_queries || !d_lut) FAIL(RAIRS_EINVAL, "null device pointer");
    return rairs_launch_lut(h->v, d_queries, nq, d_lut, d_bias_sum, d_scale, (hipStream_t)hip_stream);
}

// Slots of one search's stage events (rairs_index::ev[slot]): stage boundaries on the caller's
// stream, the table build on the side stream, the scan kernel itself.
enum { EV_START = 0, EV_PROBED = 1, EV_LUT0 = 2, EV_LUT1 = 3, EV_SCANNED = 4, EV_END = 5,
       EV_KERNEL0 = 6, EV_KERNEL1 = 7 };
static_assert(EV_KERNEL1 < 2 * RAIRS_NSTAGES, "event slots");

// SeilSearch for one pass of n queries: bitmap, then either the exact kernel alone or
// sample bound -> list-major MFMA scan -> collect / select -> exact redo of overflows.
// ev (may be null) receives two events bracketing the dominant scan kernel.
static int scan_pass(rairs_index *h, char *ws, const WsLayout &w, const uint8_t *lut, const int32_t *probe_ids,
                     int64_t n, int nprobe, int refine_k, int64_t *cand_ids, int32_t *cand_score,
                     int64_t *dco, hipStream_t s, hipEvent_t *ev, bool overlap, hipEvent_t lut_done,
                     bool any_order, hipEvent_t probed_on_side = nullptr)
{
    // overlap: the tables were built on the side stream (ev_lut marks them done) and the side
    // stream already waits for the probe lists; the grouping runs there next to the sample bound.
    // probed_on_side (may be null; implies the matrix-core sample): the probe lists are being
    // made on the side stream too, marked done by this event, and the caller's stream has only
    // the score matrix so far: the sample is taken from the list with the smallest key of the
    // query's row, and only its ranking waits for the probe lists (see search_impl).
    const IndexView &v = h->v;
    uint32_t *bitmap = (uint32_t *)(ws + w.bitmap);
    const bool mfma = rairs_mfma_supported(v) && !h->force_exact;
    // With the sample on the matrix cores nothing on the caller's stream reads the bitmaps before
    // the scan does, so they (and the zeroed histograms) are made on the side stream ahead of the
    // grouping, whose event the scan waits for anyway.
    const bool side_bitmap = overlap && mfma && grouped_sample(v, n, refine_k);
    int rc = rairs_launch_bitmap(v, probe_ids, n, nprobe, bitmap, w.bmwords, (uint32_t *)(ws + w.hist),
                                 side_bitmap ? h->side : s);
    if (rc) return rc;
    // the tables are first read by the sample (or the exact scan); with the grouped sample the
    // wait goes behind the sample's grouping kernel, which does not need them
    if (overlap && !side_bitmap) RAIRS_HIP(hipStreamWaitEvent(s, lut_done, 0));
    ExactScanArgs ea;
    memset(&ea, 0, sizeof(ea));
    ea.lut = lut; ea.probe_ids = probe_ids; ea.bitmap = bitmap; ea.bmwords = w.bmwords;
    ea.nprobe = nprobe; ea.refine_k = refine_k; ea.dco = dco;
    ea.cand_ids = cand_ids; ea.cand_score = cand_score;
    h->last_pass_n = 0;
    if (!mfma) {
        if (ev) RAIRS_HIP(hipEventRecord(ev[0], s));
        rc = rairs_launch_scan_exact(v, ea, n, s);
        if (ev) RAIRS_HIP(hipEventRecord(ev[1], s));
        return rc;
    }
    MfmaScanArgs ma;
    memset(&ma, 0, sizeof(ma));
    ma.lut = lut; ma.probe_ids = probe_ids; ma.bitmap = bitmap; ma.bmwords = w.bmwords;
    ma.nprobe = nprobe; ma.refine_k = refine_k; ma.p_first = 1; ma.nq = n;
    ma.any_order = any_order ? 1 : 0;
    ma.lcount = (int32_t *)(ws + w.lcount); ma.loff = (int32_t *)(ws + w.loff);
    ma.lcursor = (int32_t *)(ws + w.lcursor); ma.toff = (int32_t *)(ws + w.toff);
    ma.unit_list = (int32_t *)(ws + w.unit_list);
    ma.unit_rec = (int32_t *)(ws + w.unit_rec);
    {
        // parts per unit: large units save table reloads, small ones keep 2048 waves busy and the
        // tail of the kernel short
        const int64_t tiles = n * (int64_t)nprobe / 32 + v.nlist;
        const int64_t parts_total = tiles * (h->nparts / (v.nlist > 0 ? v.nlist : 1) + 1);
        int up = (int)(parts_total / (2048 * 12));
        ma.unit_parts = up >= 4 ? 4 : up >= 3 ? 3 : parts_total >= 16000 ? 2 : 1;
        // with the tables in LDS a whole workgroup shares a unit and reloads up to 128 KB of
        // tables for each: always the longest units
        if (!(v.T == 8 || v.T == 24 || v.T == 32)) ma.unit_parts = 4;
        // The last lists in single parts, so that the kernel's last units are small: as many lists
        // as hold about 1.3 units for each of the 2,048 waves, at most a third.  (1M x 128
        // workload, 8,200 two-part units, kernel: none 0.560 ms, last eighth 0.558, fifth 0.551,
        // third 0.542, half 0.546; a third of the 100M workload's 129,000 four-part units: 11.7 ms
        // against 11.1.)
        ma.unit_tail_from = v.nlist;
        if (ma.unit_parts > 1 && (v.T == 8 || v.T == 24 || v.T == 32)) {
            const double units = (double)parts_total / ma.unit_parts;
            double f = units > 0 ? 1.3 * 2048 / units : 0.0;
            f = f > 1.0 / 3 ? 1.0 / 3 : f;
            ma.unit_tail_from = v.nlist - (int)(v.nlist * f);
        }
    }
    ma.next_task = (uint32_t *)(ws + w.next_task); ma.qlist = (int32_t *)(ws + w.qlist);
    ma.tau = (int32_t *)(ws + w.tau); ma.surv_cnt = (uint32_t *)(ws + w.surv_cnt);
    ma.surv_buf = (uint64_t *)(ws + w.surv_buf); ma.surv_cap = w.surv_cap;
    ma.flags = (uint32_t *)(ws + w.flags); ma.cand_ids = cand_ids; ma.cand_score = cand_score;
    ma.work = (uint32_t *)(ws + w.work);
    ma.hist = (uint32_t *)(ws + w.hist);
    h->last_pass_n = n; h->last_flags_off = w.flags; h->last_cnt_off = w.surv_cnt;
    h->last_fill_off = w.chunk_fill; h->last_log_chunks = w.log_chunks;
    ma.log = (uint2 *)(ws + w.log); ma.chunk_fill = (uint32_t *)(ws + w.chunk_fill);
    ma.log_cursor = (uint32_t *)(ws + w.log_misc); ma.log_overflow = ma.log_cursor + 1;
    ma.log_chunks = w.log_chunks;
    // bound of every query from a sample (the head of its first list)
    ma.p_first = 0;
    ma.bound = (int32_t *)(ws + w.bound);
    ma.dco = (unsigned long long *)dco;                // counted by the scan kernel as it scores
    const int sample_blocks = w.sample_blocks;
    // The sample's scores come from the matrix cores, for queries grouped by their first list,
    // when the batch is large enough for that; else the bound kernel scores them itself, one
    // query per wave.  Side stream: the scan's grouping.
    const bool grouped = grouped_sample(v, n, refine_k);
    int32_t *s_off = (int32_t *)(ws + w.s_off), *s_toff = (int32_t *)(ws + w.s_toff);
    int32_t *s_q = (int32_t *)(ws + w.s_q), *s_tiles = (int32_t *)(ws + w.s_tiles);
    uint16_t *s_scores = (uint16_t *)(ws + w.s_scores);
    if (overlap) {
        if ((rc = rairs_launch_group(v, ma, h->side))) return rc;
        RAIRS_HIP(hipEventRecord(h->ev_group, h->side));
    }
    if (grouped && probed_on_side) {
        int32_t *s_first = (int32_t *)(ws + w.s_first);
        if ((rc = rairs_launch_coarse_first(v, (const float *)(ws + w.dmat), n, s_first, s))) return rc;
        if ((rc = rairs_launch_sample_group(v, s_first, 1, n, s_off, s_toff, s_q, s_tiles, s))) return rc;
        RAIRS_HIP(hipStreamWaitEvent(s, lut_done, 0));
        if ((rc = rairs_launch_sample_scores(v, lut, sample_blocks, n, s_off, s_toff, s_q, s_tiles, s_scores, s)))
            return rc;
        // the ranking checks that the sampled list is one of the query's probe lists (the keys
        // carry rounding, and a bound from a list that is not scanned would be no bound)
        RAIRS_HIP(hipStreamWaitEvent(s, probed_on_side, 0));
        if ((rc = rairs_launch_sample_rank(v, s_first, 1, refine_k, sample_blocks, n, s_scores,
                                           (int32_t *)(ws + w.tau), ma.bound, s, probe_ids, nprobe)))
            return rc;
    } else if (grouped) {
        if ((rc = rairs_launch_sample_group(v, probe_ids, nprobe, n, s_off, s_toff, s_q, s_tiles, s)))
            return rc;
        if (side_bitmap) RAIRS_HIP(hipStreamWaitEvent(s, lut_done, 0));
        if ((rc = rairs_launch_sample_scores(v, lut, sample_blocks, n, s_off, s_toff, s_q, s_tiles, s_scores, s)))
            return rc;
        if ((rc = rairs_launch_sample_rank(v, probe_ids, nprobe, refine_k, sample_blocks, n, s_scores,
                                           (int32_t *)(ws + w.tau), ma.bound, s)))
            return rc;
    } else if ((rc = rairs_launch_sample_bound(v, lut, probe_ids, nprobe, refine_k, sample_blocks, n,
                                               (int32_t *)(ws + w.tau), ma.bound, s)))
        return rc;
    if (overlap) RAIRS_HIP(hipStreamWaitEvent(s, h->ev_group, 0));
    else if ((rc = rairs_launch_group(v, ma, s))) return rc;
    if ((rc = rairs_launch_scan_mfma(v, ma, s, ev))) return rc;
    if ((rc = rairs_launch_select(v, ma, s))) return rc;
    // a query with more entries at or below its final bound than the buffer holds (thousands of
    // items with the same score), or every query if the log ran out of chunks, is redone by the
    // exact kernel (which counts that query's DCO again, to the same value); normally none is
    // flagged and every workgroup of that launch exits at once
    ea.only_flagged = ma.flags;
    ea.redo = ma.work + 1 + n;
    if ((rc = rairs_launch_scan_repair(v, ma, ea, s))) return rc;
    return RAIRS_OK;
}

extern "C" int rairs_scan(rairs_index_t *h, const uint8_t *d_lut, const int32_t *d_probe_ids,
                          int64_t nq, int nprobe, int refine_k, int64_t *d_cand_ids,
                          int32_t *d_cand_score, int64_t *d_dco, void *hip_stream)
{
    int rc = check_common(h, nq);
    if (rc) return rc;
    if ((rc = check_nprobe(h, nprobe))) return rc;
    if ((rc = check_k(1, refine_k))) return rc;
    if (nq == 0) return RAIRS_OK;
    if (!d_lut || !d_probe_ids || !d_cand_ids) FAIL(RAIRS_EINVAL, "null device pointer");
    if (((uintptr_t)d_lut & 15) != 0) FAIL(RAIRS_EINVAL, "d_lut must be 16-byte aligned");
    const int64_t step = pass_size(h->v, nq, nprobe, refine_k);
    WsLayout w = ws_layout(h->v, step, 0, nprobe, refine_k, h->max_parts);
    char *ws = nullptr;
    if ((rc = acquire_ws(h, WS_HANDLE, w.total, &ws))) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    for (int64_t q0 = 0; q0 < nq; q0 += step) {
        int64_t n = nq - q0 < step ? nq - q0 : step;
        rc = scan_pass(h, ws, w, d_lut + (size_t)q0 * h->v.M * 16, d_probe_ids + (size_t)q0 * nprobe, n,
                       nprobe, refine_k, d_cand_ids + (size_t)q0 * refine_k,
                       d_cand_score ? d_cand_score + (size_t)q0 * refine_k : nullptr,
                       d_dco ? d_dco + q0 : nullptr, s, nullptr, false, nullptr, false);
        if (rc) return rc;
    }
    return RAIRS_OK;
}

extern "C" int rairs_refine(rairs_index_t *h, const float *d_queries, const int64_t *d_cand_ids,
                            int64_t nq, int refine_k, int k, int64_t *d_out_ids,
                            float *d_out_dists, void *hip_stream)
{
    int rc = check_common(h, nq);
    if (rc) return rc;
    if ((rc = check_k(k, refine_k))) return rc;
    if (nq == 0) return RAIRS_OK;
    if (!d_queries || !d_cand_ids || !d_out_ids || !d_out_dists) FAIL(RAIRS_EINVAL, "null device pointer");
    return rairs_launch_refine(h->v, d_queries, d_cand_ids, nq, refine_k, k, d_out_ids, d_out_dists,
                               (hipStream_t)hip_stream);
}

// ---- RairsSearch (Alg. 2) -----------------------------------------------------------------------

static int search_impl(rairs_index *h, int ws_source, const float *d_queries, int64_t nq, int k, int nprobe,
                       int refine_k, int64_t *d_out_ids, float *d_out_dists, void *hip_stream)
{
    int rc = check_common(h, nq);
    if (rc) return rc;
    if ((rc = check_nprobe(h, nprobe))) return rc;
    if ((rc = check_k(k, refine_k))) return rc;
    if (nq == 0) return RAIRS_OK;
    if (!d_queries || !d_out_ids || !d_out_dists) FAIL(RAIRS_EINVAL, "null device pointer");
    const IndexView &v = h->v;
    const int64_t step = pass_size(v, nq, nprobe, refine_k);
    WsLayout w = ws_layout(v, step, nq, nprobe, refine_k, h->max_parts);
    char *ws = nullptr;
    if ((rc = acquire_ws(h, ws_source, w.total, &ws))) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    int64_t *dco_all = (int64_t *)(ws + w.dco);
    h->last_dco = dco_all;
    h->last_dco_n = nq;
    // stage timing is only meaningful when the batch fits one pass
    const int plevel = step == nq && ws_source != WS_GRAPH ? h->prof : 0;
    const bool prof = plevel == RAIRS_PROFILE_STAGES;  // every stage; otherwise at most the scan kernel
    const bool profk = plevel != 0;
    h->prof_valid = 0;
    hipEvent_t *ev = h->ev[h->ev_count % RAIRS_EV_RING];
    // the table build depends only on the queries and the grouping only on the probe lists, so
    // both run on the handle's side stream next to the coarse quantizer and the sample bound
    // (a captured search stays on one stream: a graph of a few queries gains nothing from the fork)
    const bool overlap = h->side_ready != 0 && ws_source != WS_GRAPH;
    hipStream_t side = overlap ? h->side : s;
    for (int64_t q0 = 0; q0 < nq; q0 += step) {
        int64_t n = nq - q0 < step ? nq - q0 : step;
        const float *q = d_queries + (size_t)q0 * v.d;
        int32_t *probe_ids = (int32_t *)(ws + w.probe_ids);
        uint8_t *lut = (uint8_t *)(ws + w.lut);
        int64_t *cand = (int64_t *)(ws + w.cand);
        // Every event recorded on a stream delays the kernel behind it by some microseconds, so a
        // stage boundary is one event: it ends a stage, starts the next and, where the side stream
        // has to wait for that point, is the event it waits on (see EV_* above).
        hipEvent_t start = prof ? ev[EV_START] : h->ev_fork;
        if (overlap || prof) RAIRS_HIP(hipEventRecord(start, s));
        if (overlap) {
            // everything earlier on the caller's stream (the previous pass reads the same
            // workspace) comes before the side stream's work
            RAIRS_HIP(hipStreamWaitEvent(side, start, 0));
            if (prof) RAIRS_HIP(hipEventRecord(ev[EV_LUT0], side));
            if ((rc = rairs_launch_lut(v, q, n, lut, nullptr, nullptr, side))) return rc;
            RAIRS_HIP(hipEventRecord(prof ? ev[EV_LUT1] : h->ev_lut, side));
        }
        // With the matrix-core sample, the caller's stream does not wait for the probe lists:
        // once the coarse GEMM has left the score matrix, the selection of the probe lists moves
        // to the side stream (behind the table build, ahead of the grouping), and the caller's
        // stream goes straight on with the bound's sample, taken from the list with the smallest
        // key of the query's row; see scan_pass.  The chain that the scan waits for -- GEMM,
        // sample, ranking -- thus stays on one stream, with no event hop in it.
        const bool early = overlap && !h->force_exact && rairs_mfma_supported(v) &&
                           grouped_sample(v, n, refine_k) && rairs_coarse_has_scores(v, nprobe, q);
        if ((rc = rairs_launch_coarse(v, q, n, nprobe, (float *)(ws + w.dmat), probe_ids,
                                      (float *)(ws + w.probe_dists), (uint32_t *)(ws + w.cflags), s,
                                      early ? h->ev_scored : nullptr, early ? side : nullptr)))
            return rc;
        hipEvent_t probed = prof ? ev[EV_PROBED] : h->ev_probe;
        if (overlap || prof) RAIRS_HIP(hipEventRecord(probed, early ? side : s));
        if (early) {
            // (the side stream made the probe lists itself)
        } else if (overlap) {
            RAIRS_HIP(hipStreamWaitEvent(side, probed, 0));
        } else {
            // one stream: the table build is timed between the coarse stage and the scan stage
            if ((rc = rairs_launch_lut(v, q, n, lut, nullptr, nullptr, s))) return rc;
            if (prof) RAIRS_HIP(hipEventRecord(ev[EV_LUT1], s));
        }
        if ((rc = scan_pass(h, ws, w, lut, probe_ids, n, nprobe, refine_k, cand, nullptr, dco_all + q0, s,
                            profk ? &ev[EV_KERNEL0] : nullptr, overlap,
                            prof ? ev[EV_LUT1] : h->ev_lut, true, early ? probed : nullptr))) return rc;
        if (prof) RAIRS_HIP(hipEventRecord(ev[EV_SCANNED], s));
        if ((rc = rairs_launch_refine(v, q, cand, n, refine_k, k, d_out_ids + (size_t)q0 * k,
                                      d_out_dists + (size_t)q0 * k, s))) return rc;
        if (prof) RAIRS_HIP(hipEventRecord(ev[EV_END], s));
    }
    if (profk) h->ev_count++;
    h->prof_valid = profk ? 1 : 0;
    return RAIRS_OK;
}

extern "C" int rairs_search(rairs_index_t *h, const float *d_queries, int64_t nq, int k, int nprobe,
                            int refine_k, int64_t *d_out_ids, float *d_out_dists, void *hip_stream)
{
    return search_impl(h, WS_HANDLE, d_queries, nq, k, nprobe, refine_k, d_out_ids, d_out_dists, hip_stream);
}

extern "C" int rairs_search_noalloc(rairs_index_t *h, const float *d_queries, int64_t nq, int k, int nprobe,
                                    int refine_k, int64_t *d_out_ids, float *d_out_dists, void *hip_stream)
{
    return search_impl(h, WS_STATIC, d_queries, nq, k, nprobe, refine_k, d_out_ids, d_out_dists, hip_stream);
}

// ---- a search captured as a HIP graph ---------------------------------------------------------------

struct rairs_graph {
    rairs_index *h;
    void *ws;
    size_t ws_bytes;
    hipGraph_t graph;
    hipGraphExec_t exec;
};

extern "C" int rairs_graph_free(rairs_graph_t *g)
{
    if (!g) return RAIRS_OK;
    if (g->exec) (void)hipGraphExecDestroy(g->exec);
    if (g->graph) (void)hipGraphDestroy(g->graph);
    if (g->ws) (void)hipFree(g->ws);
    delete g;
    return RAIRS_OK;
}

extern "C" int rairs_graph_create(rairs_index_t *h, const float *d_queries, int64_t nq, int k, int nprobe,
                                  int refine_k, int64_t *d_out_ids, float *d_out_dists, void *hip_stream,
                                  rairs_graph_t **out)
{
    if (!out) FAIL(RAIRS_EINVAL, "out is NULL");
    *out = nullptr;
    int rc = check_common(h, nq);
    if (rc) return rc;
    if ((rc = check_nprobe(h, nprobe))) return rc;
    if ((rc = check_k(k, refine_k))) return rc;
    if (nq < 1) FAIL(RAIRS_EINVAL, "a graph needs at least one query");
    if (!d_queries || !d_out_ids || !d_out_dists) FAIL(RAIRS_EINVAL, "null device pointer");
    if (!hip_stream) FAIL(RAIRS_EINVAL, "capture needs a stream of the caller's, not the default stream");
    if (pass_size(h->v, nq, nprobe, refine_k) < nq)
        FAIL(RAIRS_EUNSUPPORTED, "nq=%lld does not fit one pass", (long long)nq);
    rairs_graph *g = new (std::nothrow) rairs_graph();
    if (!g) FAIL(RAIRS_ENOMEM, "out of host memory");
    memset(g, 0, sizeof(*g));
    g->h = h;
    g->ws_bytes = ws_layout(h->v, nq, nq, nprobe, refine_k, h->max_parts).total;
    hipError_t e = hipMalloc(&g->ws, g->ws_bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        delete g;
        FAIL(RAIRS_ENOMEM, "graph workspace of %zu bytes: %s", g->ws_bytes, hipGetErrorString(e));
    }
    hipStream_t s = (hipStream_t)hip_stream;
    // one eager run first: kernels whose attributes are set at launch get that done outside the capture
    h->graph_ws = g->ws;
    h->graph_ws_bytes = g->ws_bytes;
    rc = search_impl(h, WS_GRAPH, d_queries, nq, k, nprobe, refine_k, d_out_ids, d_out_dists, hip_stream);
    if (rc == RAIRS_OK && hipStreamSynchronize(s) != hipSuccess) {
        rairs_set_error("the warm-up search failed: %s", hipGetErrorString(hipGetLastError()));
        rc = RAIRS_EHIP;
    }
    if (rc == RAIRS_OK) {
        e = hipStreamBeginCapture(s, hipStreamCaptureModeRelaxed);
        if (e != hipSuccess) {
            rairs_set_error("hipStreamBeginCapture failed: %s", hipGetErrorString(e));
            rc = RAIRS_EHIP;
        } else {
            rc = search_impl(h, WS_GRAPH, d_queries, nq, k, nprobe, refine_k, d_out_ids, d_out_dists, hip_stream);
            e = hipStreamEndCapture(s, &g->graph);     // always ends the capture, also after an error
            if (rc == RAIRS_OK && e != hipSuccess) {
                rairs_set_error("hipStreamEndCapture failed: %s", hipGetErrorString(e));
                rc = RAIRS_EHIP;
            }
        }
    }
    h->graph_ws = nullptr;
    h->graph_ws_bytes = 0;
    h->last_ws = nullptr;                              // the measurement helpers read the handle's own calls only
    h->last_pass_n = 0;
    h->last_dco = nullptr;
    h->last_dco_n = 0;
    if (rc == RAIRS_OK) {
        e = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0);
        if (e != hipSuccess) {
            rairs_set_error("hipGraphInstantiate failed: %s", hipGetErrorString(e));
            rc = RAIRS_EHIP;
        }
    }
    if (rc != RAIRS_OK) {
        (void)hipGetLastError();
        rairs_graph_free(g);
        return rc;
    }
    *out = g;
    return RAIRS_OK;
}

extern "C" int rairs_graph_launch(rairs_graph_t *g, void *hip_stream)
{
    if (!g || !g->exec) FAIL(RAIRS_EINVAL, "graph is NULL");
    RAIRS_HIP(hipGraphLaunch(g->exec, (hipStream_t)hip_stream));
    return RAIRS_OK;
}

extern "C" size_t rairs_workspace_bytes(const rairs_index_t *h, int64_t nq, int nprobe, int refine_k)
{
    if (!h || nq < 0 || nq > 0x7FFFFFFFll / 4 || nprobe < 1 || nprobe > h->v.nlist || nprobe > RAIRS_MAX_NPROBE ||
        refine_k < 1 || refine_k > RAIRS_MAX_REFINE_K) {
        rairs_set_error("rairs_workspace_bytes: arguments outside what rairs_search accepts");
        return 0;
    }
    if (nq == 0) return 0;
    const int64_t step = pass_size(h->v, nq, nprobe, refine_k);
    return ws_layout(h->v, step, nq, nprobe, refine_k, h->max_parts).total;
}

extern "C" int rairs_set_workspace(rairs_index_t *h, void *d_ws, size_t bytes)
{
    if (!h) FAIL(RAIRS_EINVAL, "handle is NULL");
    if (d_ws && ((uintptr_t)d_ws & 255) != 0) FAIL(RAIRS_EINVAL, "the workspace must be 256-byte aligned");
    h->ws_user = d_ws;
    h->ws_user_bytes = d_ws ? bytes : 0;
    h->last_ws = nullptr;
    h->last_pass_n = 0;
    h->last_dco = nullptr;
    h->last_dco_n = 0;
    return RAIRS_OK;
}

extern "C" int rairs_set_scan_mode(rairs_index_t *h, int mode)
{
    if (!h) FAIL(RAIRS_EINVAL, "handle is NULL");
    if (mode != RAIRS_SCAN_AUTO && mode != RAIRS_SCAN_EXACT) FAIL(RAIRS_EINVAL, "unknown scan mode %d", mode);
    h->force_exact = mode == RAIRS_SCAN_EXACT;
    return RAIRS_OK;
}

extern "C" const char *rairs_scan_kernel_name(const rairs_index_t *h)
{
    if (!h) return nullptr;
    if (h->force_exact || !rairs_mfma_supported(h->v)) return "scan_exact_kernel";
    return rairs_mfma_reg_tables(h->v) ? "scan_mfma_kernel" : "scan_mfma_lds_kernel";
}

extern "C" int rairs_set_profiling(rairs_index_t *h, int enabled)
{
    if (!h) FAIL(RAIRS_EINVAL, "handle is NULL");
    if (enabled != 0 && enabled != RAIRS_PROFILE_STAGES && enabled != RAIRS_PROFILE_SCAN_KERNEL)
        FAIL(RAIRS_EINVAL, "unknown profiling level %d", enabled);
    h->prof = enabled;
    h->prof_valid = 0;
    h->ev_count = 0;
    return RAIRS_OK;
}

extern "C" int rairs_get_stage_ms(rairs_index_t *h, float *ms)
{
    if (!h || !ms) FAIL(RAIRS_EINVAL, "null argument");
    if (!h->prof_valid) FAIL(RAIRS_EINVAL, "no profiled search recorded (profiling off, or the batch took several passes)");
    return rairs_get_stage_ms_mean(h, 1, ms);
}

extern "C" int rairs_get_stage_ms_mean(rairs_index_t *h, int last_n, float *ms)
{
    if (!h || !ms) FAIL(RAIRS_EINVAL, "null argument");
    if (!h->prof_valid || h->ev_count == 0)
        FAIL(RAIRS_EINVAL, "no profiled search recorded (profiling off, or the batch took several passes)");
    if (last_n < 1 || last_n > RAIRS_EV_RING) FAIL(RAIRS_EINVAL, "last_n must be in [1, %d]", RAIRS_EV_RING);
    if ((int64_t)last_n > h->ev_count) FAIL(RAIRS_EINVAL, "only %lld profiled searches recorded", (long long)h->ev_count);
    double sum[RAIRS_NSTAGES] = {0};
    for (int64_t c = h->ev_count - last_n; c < h->ev_count; c++) {
        hipEvent_t *ev = h->ev[c % RAIRS_EV_RING];
        const bool one_stream = !h->side_ready;
        const int pair[RAIRS_NSTAGES][2] = {{EV_START, EV_PROBED},
                                            {one_stream ? EV_PROBED : EV_LUT0, EV_LUT1},
                                            {one_stream ? EV_LUT1 : EV_PROBED, EV_SCANNED},
                                            {EV_SCANNED, EV_END},
                                            {EV_KERNEL0, EV_KERNEL1}};
        for (int i = 0; i < RAIRS_NSTAGES; i++) {
            if (h->prof != RAIRS_PROFILE_STAGES && i != RAIRS_STAGE_SCAN_KERNEL) { sum[i] = -(double)last_n; continue; }
            float t;
            RAIRS_HIP(hipEventSynchronize(ev[pair[i][1]]));
            RAIRS_HIP(hipEventElapsedTime(&t, ev[pair[i][0]], ev[pair[i][1]]));
            sum[i] += t;
        }
    }
    for (int i = 0; i < RAIRS_NSTAGES; i++) ms[i] = (float)(sum[i] / last_n);
    return RAIRS_OK;
}

extern "C" int rairs_get_scan_stats(rairs_index_t *h, int64_t *stats)
{
    if (!h || !stats) FAIL(RAIRS_EINVAL, "null argument");
    stats[0] = stats[1] = stats[2] = stats[4] = 0;
    stats[3] = h->last_pass_n;
    if (h->last_pass_n == 0 || !h->last_ws) return RAIRS_OK;
    std::vector<uint32_t> flags((size_t)h->last_pass_n), cnt((size_t)h->last_pass_n);
    RAIRS_HIP(hipDeviceSynchronize());
    RAIRS_HIP(hipMemcpy(flags.data(), (char *)h->last_ws + h->last_flags_off, flags.size() * 4, hipMemcpyDeviceToHost));
    RAIRS_HIP(hipMemcpy(cnt.data(), (char *)h->last_ws + h->last_cnt_off, cnt.size() * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < flags.size(); i++) {
        stats[0] += flags[i] != 0;
        stats[1] += cnt[i];
        if ((int64_t)cnt[i] > stats[2]) stats[2] = cnt[i];
    }
    std::vector<uint32_t> fill((size_t)h->last_log_chunks);
    RAIRS_HIP(hipMemcpy(fill.data(), (char *)h->last_ws + h->last_fill_off, fill.size() * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < fill.size(); i++) stats[4] += fill[i];
    return RAIRS_OK;
}

extern "C" int rairs_assign(rairs_index_t *h, const float *d_vectors, int64_t n, int n_cands,
                            double lambda, int strict, int32_t *d_pairs, void *hip_stream)
{
    int rc = check_common(h, n);
    if (rc) return rc;
    if (n_cands < 1) FAIL(RAIRS_EINVAL, "n_cands=%d: at least one candidate list", n_cands);
    const int nc = n_cands < h->v.nlist ? n_cands : h->v.nlist;
    if (nc > RAIRS_MAX_NCANDS) FAIL(RAIRS_EUNSUPPORTED, "n_cands=%d above the built limit %d", nc, RAIRS_MAX_NCANDS);
    if (!(lambda == lambda)) FAIL(RAIRS_EINVAL, "lambda is not a number");
    if (h->v.metric != RAIRS_METRIC_L2) FAIL(RAIRS_EUNSUPPORTED, "RairAssign is defined for the Euclidean metric");
    if (n == 0) return RAIRS_OK;
    if (!d_vectors || !d_pairs) FAIL(RAIRS_EINVAL, "null device pointer");
    const int64_t step = pass_size(h->v, n, nc, 1);
    const WsLayout w = ws_layout(h->v, step, 0, nc, 1);
    char *ws = nullptr;
    if ((rc = acquire_ws(h, WS_HANDLE, w.total, &ws))) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    for (int64_t q0 = 0; q0 < n; q0 += step) {
        const int64_t m = n - q0 < step ? n - q0 : step;
        const float *x = d_vectors + (size_t)q0 * h->v.d;
        int32_t *cand = (int32_t *)(ws + w.probe_ids);
        // FindNearestLists is the search path's coarse quantizer
        if ((rc = rairs_launch_coarse(h->v, x, m, nc, (float *)(ws + w.dmat), cand, nullptr,
                                      (uint32_t *)(ws + w.cflags), s))) return rc;
        if ((rc = rairs_launch_air_assign(h->v, x, m, nc, lambda, strict ? 1 : 0, cand,
                                          d_pairs + (size_t)q0 * 2, s))) return rc;
    }
    return RAIRS_OK;
}

extern "C" int rairs_pq_encode(const float *d_codebook, int d, int M, const float *d_vectors, int64_t n,
                               uint8_t *d_codes, void *hip_stream)
{
    if (d < 1 || M < 2 || M > RAIRS_MAX_M || M % 2 != 0 || d % M != 0)
        FAIL(RAIRS_EINVAL, "PQ shape d=%d M=%d: need M even, 2 <= M <= %d, d a multiple of M", d, M, RAIRS_MAX_M);
    if ((size_t)16 * d * sizeof(float) > 160 * 1024 - 1024) FAIL(RAIRS_EINVAL, "d=%d: the codebook does not fit LDS", d);
    if (n < 0) FAIL(RAIRS_EINVAL, "n is negative");
    if (n == 0) return RAIRS_OK;
    if (!d_codebook || !d_vectors || !d_codes) FAIL(RAIRS_EINVAL, "null device pointer");
    return rairs_launch_pq_encode(d_codebook, d, M, d_vectors, n, d_codes, (hipStream_t)hip_stream);
}

extern "C" int rairs_get_dco(rairs_index_t *h, int64_t *dco, int64_t nq)
{
    if (!h || !dco) FAIL(RAIRS_EINVAL, "null argument");
    if (nq < 0 || nq > h->last_dco_n || (nq > 0 && !h->last_dco))
        FAIL(RAIRS_EINVAL, "nq exceeds the last search's batch");
    if (nq == 0) return RAIRS_OK;
    RAIRS_HIP(hipMemcpy(dco, h->last_dco, (size_t)nq * 8, hipMemcpyDeviceToHost));
    return RAIRS_OK;
}
