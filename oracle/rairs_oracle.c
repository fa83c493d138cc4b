/*
 * CPU oracle for the RAIRS query path -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, scalar implementation of what the search path computes, written from the paper
 * (arxiv 2601.07183): Alg. 2 (RairsSearch) with SeilSearch of Alg. 5 over the list layout of
 * Section 5.1, IVF-PQ lookup tables of Section 2.2 and exact-distance refinement.  It shares no
 * code with the HIP library.  Only tests, the smoke check and the benchmark's CPU baseline call
 * it.
 *
 * Two routes to the candidate set are provided and must agree exactly:
 *   layout 0: Alg. 5 taken step by step on the SEIL directory (reference entries, shared
 *             blocks, miscellaneous blocks, listVisited);
 *   layout 1: the plain definition -- the set of vectors that are members of at least one probed
 *             list, each scored once -- from the per-vector assignment, no SEIL structures.
 *
 * Where the paper is silent the following readings are fixed (all stated again in the design
 * notes of this repository):
 *   - all distances are squared Euclidean distances (Section 2.1 defines the metric; Alg. 3
 *     already works on squares);
 *   - fp32 arithmetic without fused multiply-add; a squared distance over d dimensions is summed
 *     as 64 interleaved partial sums p[j] = sum_{i = j mod 64} (a_i - b_i)^2, i increasing,
 *     folded p[j] += p[j ^ 32], ^16, ^8, ^4, ^2, ^1;
 *   - the lookup table entry is T[m][c] = |q_m - codeword_{m,c}|^2 summed left to right over the
 *     sub-vector; it is quantised to 8 bits as
 *         u8[m][c] = min(255, rint((T[m][c] - b_m) * s)),  b_m = min_c T[m][c],
 *         s = 255 / max_m(max_c T[m][c] - b_m)   (s = 0 when that span is 0),
 *     and an item's score is the plain unsigned 16-bit sum of its M table entries;
 *   - probed lists: the nprobe smallest (distance, list id); candidates: the bigK smallest
 *     (score, vector id); results: the K smallest (exact distance, vector id); missing entries
 *     are id -1 / distance +inf;
 *   - Alg. 5 walks the selected lists in ascending list id, which is what makes its
 *     "no duplicate" claim for physically stored shared blocks hold (the owner of a shared cell
 *     is the smaller list id);
 *   - a distance computation (DCO) is one valid item slot scored during the list scan;
 *   - inner-product metric (the paper applies SEIL to an inner-product index in Section 6.4 and
 *     does not describe the search beyond that): every "distance" is the negated inner product,
 *     so that smaller is still better -- probed lists: the nprobe largest <q, c> (ties: smaller
 *     list id); table entry T[m][c] = -<q_m, codeword_{m,c}>, quantised as above; results: the K
 *     largest exact <q, x> (ties: smaller id), reported as inner products, missing entries -inf.
 *     An inner product over d dimensions is summed like a squared distance: 64 interleaved partial
 *     sums of the products q_i x_i, folded the same way.
 *
 * Build with -ffp-contract=off and without -ffast-math: the arithmetic above is the contract.
 *
 * Parity pins live in tests/ (brute-force kNN, layout equivalence, at-most-once, PQ identity,
 * quantisation bound, DCO identity, integer exactness).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif


#define METRIC_L2 0
#define METRIC_IP 1

typedef struct {
    int32_t d, M, nlist, raw_is_u8;
    int32_t metric, blk;               /* METRIC_*; items per block (BLK_SZ of Alg. 4) */
    int64_t ntotal, nblocks, nrefs;
    const float *centroids;            /* [nlist][d] */
    const float *codebook;             /* [M][16][d/M] */
    const uint8_t *codes;              /* [nblocks][blk][M/2] */
    const int64_t *ids;                /* [nblocks][blk] */
    const int32_t *other;              /* [nblocks][blk] */
    const int64_t *list_shared_begin;
    const int32_t *list_shared_cnt;
    const int64_t *list_misc_begin;
    const int32_t *list_misc_cnt;
    const int64_t *list_ref_begin;
    const int32_t *list_ref_cnt;
    const int32_t *ref_owner;
    const int64_t *ref_block_begin;
    const int32_t *ref_nblocks;
    const void *raw;                   /* [ntotal][d] f32 or u8 */
    const int32_t *assign;             /* [ntotal][2]; (-1, -1): the vector was deleted */
    const uint8_t *vec_codes;          /* [ntotal][M/2] */
} oracle_index;

/* ---- exact squared L2 in the fixed summation order ------------------------------------ */

static float fold64(float *p)
{
    for (int s = 32; s >= 1; s >>= 1)
        for (int j = 0; j < s; j++) {
            /* p[j] += p[j ^ s] for every j; only the lower half is needed afterwards */
            p[j] = p[j] + p[j ^ s];
        }
    return p[0];
}

float oracle_l2sqr(const float *a, const float *b, int d)
{
    float p[64];
    for (int j = 0; j < 64; j++) p[j] = 0.0f;
    for (int i = 0; i < d; i++) {
        float diff = a[i] - b[i];
        float sq = diff * diff;
        p[i & 63] = p[i & 63] + sq;
    }
    return fold64(p);
}

/* inner product in the same summation order */
float oracle_ip(const float *a, const float *b, int d)
{
    float p[64];
    for (int j = 0; j < 64; j++) p[j] = 0.0f;
    for (int i = 0; i < d; i++) {
        float prod = a[i] * b[i];
        p[i & 63] = p[i & 63] + prod;
    }
    return fold64(p);
}

float oracle_ip_u8(const float *a, const uint8_t *b, int d)
{
    float p[64];
    for (int j = 0; j < 64; j++) p[j] = 0.0f;
    for (int i = 0; i < d; i++) {
        float prod = a[i] * (float)b[i];
        p[i & 63] = p[i & 63] + prod;
    }
    return fold64(p);
}

float oracle_l2sqr_u8(const float *a, const uint8_t *b, int d)
{
    float p[64];
    for (int j = 0; j < 64; j++) p[j] = 0.0f;
    for (int i = 0; i < d; i++) {
        float diff = a[i] - (float)b[i];
        float sq = diff * diff;
        p[i & 63] = p[i & 63] + sq;
    }
    return fold64(p);
}

/* ---- FindNearestLists on the query side (Alg. 2) ---------------------------------------------- */

typedef struct { float dist; int64_t id; } dist_id;

static int cmp_dist_id(const void *pa, const void *pb)
{
    const dist_id *a = (const dist_id *)pa, *b = (const dist_id *)pb;
    if (a->dist < b->dist) return -1;
    if (a->dist > b->dist) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

void oracle_coarse(const oracle_index *ix, const float *q, int nprobe, int32_t *out_lists,
                   float *out_dists)
{
    dist_id *all = (dist_id *)malloc(sizeof(dist_id) * (size_t)ix->nlist);
    for (int l = 0; l < ix->nlist; l++) {
        const float *c = ix->centroids + (size_t)l * ix->d;
        /* inner product: order by the negated product, so that the same comparison serves */
        all[l].dist = ix->metric == METRIC_IP ? -oracle_ip(q, c, ix->d) : oracle_l2sqr(q, c, ix->d);
        all[l].id = l;
    }
    qsort(all, (size_t)ix->nlist, sizeof(dist_id), cmp_dist_id);
    for (int i = 0; i < nprobe; i++) {
        out_lists[i] = (int32_t)all[i].id;
        if (out_dists) out_dists[i] = ix->metric == METRIC_IP ? -all[i].dist : all[i].dist;
    }
    free(all);
}

/* ---- ComputeLookupTable (Alg. 2, Section 2.2) + 8-bit quantisation ----------------- */

void oracle_lut(const oracle_index *ix, const float *q, float *T, uint8_t *lut, float *bias_sum,
                float *scale)
{
    const int M = ix->M, dsub = ix->d / ix->M;
    float span = 0.0f, bsum = 0.0f;
    float *bias = (float *)malloc(sizeof(float) * (size_t)M);
    for (int m = 0; m < M; m++) {
        float lo = INFINITY, hi = -INFINITY;
        for (int c = 0; c < 16; c++) {
            const float *cw = ix->codebook + ((size_t)m * 16 + c) * dsub;
            float acc = 0.0f;
            for (int t = 0; t < dsub; t++) {
                float term;
                if (ix->metric == METRIC_IP) {
                    term = q[m * dsub + t] * cw[t];
                } else {
                    float a = q[m * dsub + t] - cw[t];
                    term = a * a;
                }
                if (t == 0) acc = term; else acc = acc + term;
            }
            if (ix->metric == METRIC_IP) acc = -acc;        /* smaller is better */
            T[m * 16 + c] = acc;
            if (acc < lo) lo = acc;
            if (acc > hi) hi = acc;
        }
        bias[m] = lo;
        float w = hi - lo;
        if (w > span) span = w;
        float nb = bsum + lo;
        bsum = nb;
    }
    float s = (span > 0.0f) ? 255.0f / span : 0.0f;
    for (int m = 0; m < M; m++)
        for (int c = 0; c < 16; c++) {
            float x = T[m * 16 + c] - bias[m];
            float y = x * s;
            float r = rintf(y);               /* round half to even in the default mode */
            if (r > 255.0f) r = 255.0f;
            lut[m * 16 + c] = (uint8_t)r;
        }
    *bias_sum = bsum;
    *scale = s;
    free(bias);
}

/* ---- scoring ------------------------------------------------------------------------------- */

static inline uint16_t score_code(const uint8_t *lut, const uint8_t *code, int M)
{
    uint16_t acc = 0;
    for (int m = 0; m < M; m++) {
        int nib = (m & 1) ? (code[m >> 1] >> 4) : (code[m >> 1] & 15);
        acc = (uint16_t)(acc + lut[m * 16 + nib]);
    }
    return acc;
}

typedef struct {
    uint64_t *keys; size_t n, cap;
} keyvec;

static void kv_push(keyvec *v, uint16_t acc, int64_t id)
{
    if (v->n == v->cap) {
        v->cap = v->cap ? v->cap * 2 : 4096;
        v->keys = (uint64_t *)realloc(v->keys, v->cap * sizeof(uint64_t));
    }
    v->keys[v->n++] = ((uint64_t)acc << 32) | (uint64_t)(uint32_t)id;
}

static int cmp_u64(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x > y) - (x < y);
}

/* optional instrumentation of one query (small inputs only) */
typedef struct {
    int32_t *push_count;    /* [ntotal]  times the id entered rqueue */
    int32_t *block_count;   /* [nblocks] times the block was scored  */
} probe_trace;

static int64_t scan_block(const oracle_index *ix, const uint8_t *lut, int64_t b,
                          const uint8_t *visited, int is_misc, keyvec *rq, probe_trace *tr)
{
    const int hb = ix->M / 2, BLK = ix->blk;
    int64_t dco = 0;
    if (tr) tr->block_count[b]++;
    for (int s = 0; s < BLK; s++) {
        int64_t id = ix->ids[b * BLK + s];
        if (id < 0) continue;                               /* empty slot of a partial block */
        uint16_t acc = score_code(lut, ix->codes + ((size_t)b * BLK + s) * hb, ix->M);
        dco++;
        if (is_misc && visited[ix->other[b * BLK + s]])     /* RemoveVectorIfVisited */
            continue;
        kv_push(rq, acc, id);
        if (tr) tr->push_count[id]++;
    }
    return dco;
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* SeilSearch (Alg. 5) for one query; returns the number of items scored */
static int64_t seil_search(const oracle_index *ix, const uint8_t *lut, const int32_t *probes,
                           int nprobe, keyvec *rq, probe_trace *tr)
{
    uint8_t *visited = (uint8_t *)calloc((size_t)ix->nlist, 1);
    int32_t *sel = (int32_t *)malloc(sizeof(int32_t) * (size_t)nprobe);
    memcpy(sel, probes, sizeof(int32_t) * (size_t)nprobe);
    qsort(sel, (size_t)nprobe, sizeof(int32_t), cmp_i32);
    int64_t dco = 0;
    for (int p = 0; p < nprobe; p++) {
        const int32_t L = sel[p];
        /* reference entries */
        for (int64_t r = ix->list_ref_begin[L]; r < ix->list_ref_begin[L] + ix->list_ref_cnt[L]; r++) {
            if (visited[ix->ref_owner[r]]) continue;
            for (int b = 0; b < ix->ref_nblocks[r]; b++)
                dco += scan_block(ix, lut, ix->ref_block_begin[r] + b, visited, 0, rq, tr);
        }
        /* shared blocks stored in this list: no duplicate check */
        for (int64_t b = ix->list_shared_begin[L]; b < ix->list_shared_begin[L] + ix->list_shared_cnt[L]; b++)
            dco += scan_block(ix, lut, b, visited, 0, rq, tr);
        /* miscellaneous area */
        for (int64_t b = ix->list_misc_begin[L]; b < ix->list_misc_begin[L] + ix->list_misc_cnt[L]; b++)
            dco += scan_block(ix, lut, b, visited, 1, rq, tr);
        visited[L] = 1;
    }
    free(sel);
    free(visited);
    return dco;
}

/* the definition: every member of a probed list, once */
static int64_t naive_search(const oracle_index *ix, const uint8_t *lut, const int32_t *probes,
                            int nprobe, keyvec *rq, probe_trace *tr)
{
    uint8_t *probed = (uint8_t *)calloc((size_t)ix->nlist, 1);
    for (int p = 0; p < nprobe; p++) probed[probes[p]] = 1;
    const int hb = ix->M / 2;
    int64_t n = 0;
    for (int64_t v = 0; v < ix->ntotal; v++) {
        if (ix->assign[2 * v] < 0) continue;                /* deleted: in no list */
        if (!probed[ix->assign[2 * v]] && !probed[ix->assign[2 * v + 1]]) continue;
        kv_push(rq, score_code(lut, ix->vec_codes + (size_t)v * hb, ix->M), v);
        if (tr) tr->push_count[v]++;
        n++;
    }
    free(probed);
    return n;
}

/*
 * RairsSearch (Alg. 2).  Per query, independent of all others:
 *   LUT -> nprobe nearest lists -> candidates (bigK = refine_k smallest (score, id)) ->
 *   Refine (K smallest (exact distance, id)).
 * Optional outputs (may be NULL): cand_ids/cand_acc [nq][refine_k], dco [nq],
 * probes_out [nq][nprobe] in (distance, id) order, lut_out [nq][M][16],
 * push_count [nq][ntotal], block_count [nq][nblocks].
 */
int oracle_search(const oracle_index *ix, const float *queries, int64_t nq, int k, int nprobe,
                  int refine_k, int layout, int nthreads, int64_t *out_ids, float *out_dists,
                  int64_t *cand_ids, int32_t *cand_acc, int64_t *dco, int32_t *probes_out,
                  uint8_t *lut_out, int32_t *push_count, int32_t *block_count)
{
    if (nprobe < 1 || nprobe > ix->nlist || k < 1 || k > refine_k) return -1;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
    const int d = ix->d, M = ix->M;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t qi = 0; qi < nq; qi++) {
        const float *q = queries + (size_t)qi * d;
        float *T = (float *)malloc(sizeof(float) * (size_t)M * 16);
        uint8_t *lut = (uint8_t *)malloc((size_t)M * 16);
        int32_t *probes = (int32_t *)malloc(sizeof(int32_t) * (size_t)nprobe);
        float bias_sum, scale;
        oracle_lut(ix, q, T, lut, &bias_sum, &scale);
        oracle_coarse(ix, q, nprobe, probes, NULL);
        if (probes_out) memcpy(probes_out + (size_t)qi * nprobe, probes, sizeof(int32_t) * (size_t)nprobe);
        if (lut_out) memcpy(lut_out + (size_t)qi * M * 16, lut, (size_t)M * 16);

        probe_trace tr, *trp = NULL;
        if (push_count && block_count) {
            tr.push_count = push_count + (size_t)qi * ix->ntotal;
            tr.block_count = block_count + (size_t)qi * ix->nblocks;
            trp = &tr;
        }
        keyvec rq = {0, 0, 0};
        int64_t n = layout == 0 ? seil_search(ix, lut, probes, nprobe, &rq, trp)
                                : naive_search(ix, lut, probes, nprobe, &rq, trp);
        if (dco) dco[qi] = n;
        qsort(rq.keys, rq.n, sizeof(uint64_t), cmp_u64);
        size_t nc = rq.n < (size_t)refine_k ? rq.n : (size_t)refine_k;
        for (int i = 0; i < refine_k; i++) {
            if (cand_ids) cand_ids[(size_t)qi * refine_k + i] = (size_t)i < nc ? (int64_t)(uint32_t)rq.keys[i] : -1;
            if (cand_acc) cand_acc[(size_t)qi * refine_k + i] = (size_t)i < nc ? (int32_t)(rq.keys[i] >> 32) : -1;
        }
        /* Refine */
        dist_id *ex = (dist_id *)malloc(sizeof(dist_id) * (nc ? nc : 1));
        for (size_t i = 0; i < nc; i++) {
            int64_t id = (int64_t)(uint32_t)rq.keys[i];
            ex[i].id = id;
            if (ix->metric == METRIC_IP)
                ex[i].dist = ix->raw_is_u8
                    ? -oracle_ip_u8(q, (const uint8_t *)ix->raw + (size_t)id * d, d)
                    : -oracle_ip(q, (const float *)ix->raw + (size_t)id * d, d);
            else
                ex[i].dist = ix->raw_is_u8
                    ? oracle_l2sqr_u8(q, (const uint8_t *)ix->raw + (size_t)id * d, d)
                    : oracle_l2sqr(q, (const float *)ix->raw + (size_t)id * d, d);
        }
        qsort(ex, nc, sizeof(dist_id), cmp_dist_id);
        const float sign = ix->metric == METRIC_IP ? -1.0f : 1.0f;   /* reported: the inner product itself */
        for (int i = 0; i < k; i++) {
            out_ids[(size_t)qi * k + i] = (size_t)i < nc ? ex[i].id : -1;
            out_dists[(size_t)qi * k + i] = (size_t)i < nc ? sign * ex[i].dist : sign * INFINITY;
        }
        free(ex); free(rq.keys); free(probes); free(lut); free(T);
    }
    return 0;
}

/* ---- PQEncoding (Alg. 1, Section 2.2): the code of a vector ------------------------------- */

/*
 * code[m] = index of the codeword of sub-quantizer m nearest to sub-vector m; the first one on a
 * tie.  The distances are the entries of the lookup table the vector would get as a query (same
 * fp32 arithmetic: sequential over the sub-vector's dimensions, no fused multiply-add), since
 * floating point decides an integer here and both sides must decide in one precision.
 * Packed like the index: byte i holds sub-quantizer 2i in the low nibble, 2i+1 in the high one.
 */
void oracle_pq_encode(const float *codebook, int d, int M, const float *x, int64_t n, uint8_t *codes)
{
    const int dsub = d / M;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; v++) {
        const float *xv = x + (size_t)v * d;
        for (int m = 0; m < M; m++) {
            int best = 0;
            float bestd = 0.0f;
            for (int c = 0; c < 16; c++) {
                const float *cw = codebook + ((size_t)m * 16 + c) * dsub;
                float acc = 0.0f;
                for (int t = 0; t < dsub; t++) {
                    float a = xv[m * dsub + t] - cw[t];
                    float sq = a * a;
                    if (t == 0) acc = sq; else acc = acc + sq;
                }
                if (c == 0 || acc < bestd) { best = c; bestd = acc; }
            }
            uint8_t *o = codes + (size_t)v * (M / 2) + m / 2;
            if (m % 2 == 0) *o = (uint8_t)best; else *o = (uint8_t)(*o | (best << 4));
        }
    }
}

/* ---- RairAssign (Alg. 3): the two lists of a vector ---------------------------------------- */

/*
 * FindNearestLists is the coarse quantizer of the search path (same fp32 distances, order by
 * (distance, list id)); the loss of candidate i, loss[i] = ||r_i||^2 + lambda <r_0, r_i> with
 * r_i = centroid_i - v, is taken in float64, both sums sequential over the dimensions, no fused
 * multiply-add (the paper does not fix a precision; the decision is an argmin, so one is fixed
 * here).  The secondary list is the first minimum of the loss over candidates 1.. (strict) or 0..
 * (not strict: it may equal the primary list, the vector is then stored once).  n_cands is
 * clamped to nlist.  out[v] = the pair ordered by list id.
 */
void oracle_rair_assign(const float *centroids, int nlist, int d, const float *x, int64_t n,
                        int n_cands, double lambda, int strict, int32_t *out)
{
    if (n_cands > nlist) n_cands = nlist;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; v++) {
        const float *xv = x + (size_t)v * d;
        dist_id *all = (dist_id *)malloc(sizeof(dist_id) * (size_t)nlist);
        for (int l = 0; l < nlist; l++) {
            all[l].dist = oracle_l2sqr(xv, centroids + (size_t)l * d, d);
            all[l].id = l;
        }
        qsort(all, (size_t)nlist, sizeof(dist_id), cmp_dist_id);
        const float *c0 = centroids + (size_t)all[0].id * d;
        int best = -1;
        double bestloss = 0.0;
        for (int i = strict ? 1 : 0; i < n_cands; i++) {
            const float *ci = centroids + (size_t)all[i].id * d;
            double l2 = 0.0, ip = 0.0;
            for (int t = 0; t < d; t++) {
                double r0 = (double)c0[t] - (double)xv[t];
                double r = (double)ci[t] - (double)xv[t];
                double rr = r * r, r0r = r0 * r;
                l2 = l2 + rr;
                ip = ip + r0r;
            }
            double scaled = lambda * ip;
            double loss = l2 + scaled;
            if (best < 0 || loss < bestloss) { best = i; bestloss = loss; }
        }
        const int32_t first = (int32_t)all[0].id, second = best < 0 ? first : (int32_t)all[best].id;
        out[2 * v] = first < second ? first : second;
        out[2 * v + 1] = first < second ? second : first;
        free(all);
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
