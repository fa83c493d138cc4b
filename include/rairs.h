/*
 * rairs.h -- C ABI of the MI355X (gfx950) RAIRS query path.
 *
 * The library implements Alg. 2 of the paper (RairsSearch) for a batch of queries on one GPU:
 *   coarse quantizer (FindNearestLists, Section 2.2)  ->  lookup tables (ComputeLookupTable,
 *   Section 2.2)  ->  SeilSearch over the SEIL list layout (Alg. 5, Section 5)  ->
 *   top-bigK candidates  ->  Refine with exact distances (Section 2.2).
 * Index construction (Alg. 1, 3, 4) happens on the host, outside this library; its output is
 * handed over in the canonical host layout below.
 *
 * Conventions
 *   - Every function returns 0 (RAIRS_OK) or a negative rairs_status; nothing throws, aborts or
 *     exits.  rairs_last_error() gives a thread-local message for the last failure.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory on the
 *     current device.  `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *   - Search calls only enqueue work on `hip_stream`; outputs are valid once the caller has
 *     synchronised that stream.  One search at a time per handle (calls share its workspace).
 *     With a caller-owned workspace (rairs_set_workspace) they never allocate or synchronise.
 *   - All distances are squared Euclidean distances in fp32.  Orders are total:
 *     lists by (distance, list id), candidates by (16-bit score, vector id), results by
 *     (distance, vector id).  Missing entries are id -1 / distance +inf / score -1.
 */
#ifndef RAIRS_H
#define RAIRS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rairs_index rairs_index_t;   /* opaque device-resident index */

typedef enum {
    RAIRS_OK = 0,
    RAIRS_EINVAL = -1,        /* bad argument (null pointer, size out of range, broken directory) */
    RAIRS_ENOMEM = -2,        /* host or device allocation failed */
    RAIRS_EHIP = -3,          /* a HIP runtime call failed */
    RAIRS_EUNSUPPORTED = -4,  /* valid request outside the built limits */
    RAIRS_EWORKSPACE = -5     /* the workspace the caller set (or the static scratch array) is too
                                 small for this call; nothing was enqueued */
} rairs_status;

/*
 * Metric of an index.  RAIRS_METRIC_L2: squared Euclidean distance (the paper's problem statement,
 * Section 2.1).  RAIRS_METRIC_IP: inner product, the metric of the index that Section 6.4 applies
 * SEIL to: the probed lists are the nprobe largest <q, centroid> (ties: smaller list id), a table
 * entry is -<q_m, codeword> (quantised as for distances), candidates are the refine_k smallest
 * (score, id) as always, and the results are the k largest exact <q, x> (ties: smaller id).
 * Wherever a call reports "distances" it then reports inner products, largest first; missing
 * entries are -inf.  Products are summed in the order that distances are.
 */
enum { RAIRS_METRIC_L2 = 0, RAIRS_METRIC_IP = 1 };

/* Built limits (rejected with RAIRS_EUNSUPPORTED beyond them). */
#define RAIRS_MAX_M        256     /* 255 * M must fit 16 bits: M <= 257 */
#define RAIRS_MAX_REFINE_K 1024
#define RAIRS_MAX_NPROBE   4096
#define RAIRS_MAX_D        2048

/*
 * Canonical host layout written by SeilInsert (Alg. 4); all arrays are host memory owned by the
 * caller and may be released as soon as rairs_index_upload returns.
 *
 * Blocks hold 32 items (BLK_SZ).  List L owns blocks [list_shared_begin[L], +list_shared_cnt[L])
 * -- the full blocks of every cell (L, j), stored once -- and [list_misc_begin[L],
 * +list_misc_cnt[L]) -- leftovers of all cells touching L; of these only the last may have empty
 * slots (id -1), at its end.  Reference entries [list_ref_begin[L], +list_ref_cnt[L]) of list L
 * each name blocks of a cell (owner, L), owner < L, stored in list `owner` (Section 5.1); after
 * several insertion batches a list may hold more than one entry to the same owner.  A slot of a
 * shared block whose item was deleted holds id -1 (Section 6.1's deletion rule) and is skipped.
 * The leftover items of a cell (i, j), i != j, sit in the miscellaneous areas of BOTH lists, with
 * the same code, tagged with the other list (Section 5.1); the scan relies on this pairing when
 * it bounds scores from a sample of a list.  Upload checks it: every vector id must occur exactly
 * once in a shared block (untagged), or once in the miscellaneous area of its only list (tagged
 * with that list), or as such a pair of twins; blocks belong to at most one list; the owner of a
 * reference entry has the smaller list id.  Anything else is RAIRS_EINVAL.
 */
typedef struct {
    int32_t d;               /* vector dimension */
    int32_t M;               /* PQ sub-quantizers, d % M == 0, M even */
    int32_t nbits;           /* must be 4 */
    int32_t nlist;
    int32_t blk;             /* must be 32 */
    int32_t raw_is_u8;       /* raw vectors given as uint8 (else fp32; fp32 data whose components
                                are all integers in [0, 255] is stored as uint8 on the device,
                                which changes no result) */
    int64_t ntotal;          /* vectors, < 2^32 - 1 */
    int64_t nblocks;
    int64_t nrefs;
    const float *centroids;          /* [nlist][d] */
    const float *codebook;           /* [M][16][d/M] */
    const uint8_t *codes;            /* [nblocks][32][M/2]; byte i: subspace 2i low nibble,
                                        2i+1 high nibble */
    const int64_t *ids;              /* [nblocks][32]; -1 = empty slot */
    const int32_t *other;            /* [nblocks][32]; misc items: the item's other list id
                                        (its own list for a vector stored once); else -1 */
    const int64_t *list_shared_begin;
    const int32_t *list_shared_cnt;
    const int64_t *list_misc_begin;
    const int32_t *list_misc_cnt;
    const int64_t *list_ref_begin;
    const int32_t *list_ref_cnt;
    const int32_t *ref_owner;        /* [nrefs] */
    const int64_t *ref_block_begin;  /* [nrefs] */
    const int32_t *ref_nblocks;      /* [nrefs], >= 1 */
    const void *raw;                 /* [ntotal][d] fp32 or uint8: the refine module's vectors */
    int32_t metric;                  /* RAIRS_METRIC_L2 (0) or RAIRS_METRIC_IP */
} rairs_host_index_t;

/*
 * Copy an index to the current device in the library's device format (Fig. 3: centroids,
 * inverted lists, vector data).  Validates sizes, every directory range and the layout rules
 * above; synchronises its own copies before returning.  The device copy belongs to the handle
 * (hipMalloc) and is released by rairs_free.  *out receives the handle.
 */
int rairs_index_upload(const rairs_host_index_t *host, void *hip_stream, rairs_index_t **out);

/*
 * RairsSearch (Alg. 2) for nq queries with bigK = refine_k.
 *   d_queries   device [nq][d] fp32
 *   d_out_ids   device [nq][k] int64, ascending (distance, id)
 *   d_out_dists device [nq][k] fp32 squared distances
 * Requires 1 <= k <= refine_k <= RAIRS_MAX_REFINE_K, 1 <= nprobe <= min(nlist,
 * RAIRS_MAX_NPROBE).  nq == 0 is a successful no-op.  Scratch memory: the workspace set with
 * rairs_set_workspace (too small: RAIRS_EWORKSPACE, nothing enqueued); if none was set, a
 * workspace of the handle's own that grows on demand (a growth synchronises the device and
 * calls hipMalloc; steady-state calls allocate nothing).
 * Everything is ordered after the earlier work of hip_stream and complete when hip_stream is;
 * inside, the table build and the grouping of queries by list run on a second stream that the
 * handle owns (default priority), forked from and joined to hip_stream with events.  Calls on one
 * handle share its workspace and that stream: they must not overlap.
 */
int rairs_search(rairs_index_t *h, const float *d_queries, int64_t nq, int k, int nprobe,
                 int refine_k, int64_t *d_out_ids, float *d_out_dists, void *hip_stream);

/* Release the device copy (and the handle's own workspace, never the caller's).  NULL is accepted. */
int rairs_free(rairs_index_t *h);

/*
 * Bytes of scratch memory that rairs_search (and each of the stage calls below) needs for nq
 * queries with these parameters: sizes grow with nq, nprobe and refine_k, so the value for the
 * largest of each covers every smaller call.  Batches of more than about 65,000 queries are cut
 * into passes that share the workspace.  0 if the arguments are outside what rairs_search accepts
 * (see rairs_last_error) or nq == 0.
 */
size_t rairs_workspace_bytes(const rairs_index_t *h, int64_t nq, int nprobe, int refine_k);

/*
 * Hand the handle a workspace: device memory of the caller (a PyTorch tensor's data_ptr()), 256-byte
 * aligned, of `bytes` bytes.  Later calls use it instead of allocating; one that needs more
 * returns RAIRS_EWORKSPACE.  The caller keeps ownership and must keep the buffer alive, and must
 * not set another, while work of this handle is in flight.  d_ws == NULL returns to the handle's
 * own workspace.  The measurement helpers (rairs_get_dco, rairs_get_scan_stats) read the last
 * call's workspace and are reset by this call.
 */
int rairs_set_workspace(rairs_index_t *h, void *d_ws, size_t bytes);

/*
 * rairs_search for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, same results, but all scratch
 * memory is a static device array of RAIRS_NOALLOC_SCRATCH_BYTES that the library's code object
 * carries, so the call allocates nothing (no hipMalloc, hipFree or allocating library routine).
 * A call whose rairs_workspace_bytes exceeds that size returns RAIRS_EWORKSPACE and enqueues
 * nothing (small batches fit: e.g. a few hundred queries at nprobe 32 over 1,024 lists).  Every
 * call on a GPU shares that GPU's array, on every handle: calls that overlap on one GPU race, the
 * caller serialises them (one stream, or events).  What must start at zero is cleared by the
 * call's own kernels.
 */
#define RAIRS_NOALLOC_SCRATCH_BYTES (128u << 20)
int rairs_search_noalloc(rairs_index_t *h, const float *d_queries, int64_t nq, int k, int nprobe,
                         int refine_k, int64_t *d_out_ids, float *d_out_dists, void *hip_stream);

/*
 * RairsSearch for one query at a time or a few (the one-query-at-a-time experiment of Section 6.2),
 * captured once as a HIP graph and replayed: a small batch is bound by its fifteen kernel launches,
 * which a graph submits as one.  rairs_graph_create runs the search once eagerly, then captures it
 * on `hip_stream` (a stream of the caller's; not NULL) with these device pointers and parameters
 * baked in, into a workspace that the graph owns (hipMalloc; released by rairs_graph_free).  A
 * replay reads whatever d_queries holds when it runs and overwrites d_out_ids / d_out_dists; the
 * caller orders its own writes and reads on the launch stream.  The captured search stays on one
 * stream, clears what must start at zero with its own kernels and records no memset node.  nq
 * must fit one internal pass (65,536 queries at most).  A graph must not run while another call
 * of the same handle does, must be freed before the handle, and replays on one stream at a time.
 */
typedef struct rairs_graph rairs_graph_t;
int rairs_graph_create(rairs_index_t *h, const float *d_queries, int64_t nq, int k, int nprobe,
                       int refine_k, int64_t *d_out_ids, float *d_out_dists, void *hip_stream,
                       rairs_graph_t **out);
int rairs_graph_launch(rairs_graph_t *g, void *hip_stream);
int rairs_graph_free(rairs_graph_t *g);       /* NULL is accepted */

/* ---- the stages of rairs_search, callable one by one (same kernels) ----------------------- */

/*
 * FindNearestLists for a query batch (Alg. 2): the nprobe nearest centroids per query.
 *   d_probe_ids   device [nq][nprobe] int32 in (distance, list id) order
 *   d_probe_dists device [nq][nprobe] fp32, may be NULL
 */
int rairs_coarse(rairs_index_t *h, const float *d_queries, int64_t nq, int nprobe,
                 int32_t *d_probe_ids, float *d_probe_dists, void *hip_stream);

/*
 * ComputeLookupTable (Alg. 2) quantised to 8 bits:
 *   T[m][c] = |q_m - codeword(m,c)|^2,  b_m = min_c T[m][c],  s = 255 / max_m(max_c T[m][c] - b_m)
 *   lut[m][c] = min(255, rint((T[m][c] - b_m) * s))      (s = 0 if the span is 0)
 *   d_lut device [nq][M][16] uint8; d_bias_sum [nq] = sum_m b_m; d_scale [nq] = s
 *   (either of the last two may be NULL).  bias_sum + score / s approximates the distance.
 */
int rairs_lut(rairs_index_t *h, const float *d_queries, int64_t nq, uint8_t *d_lut,
              float *d_bias_sum, float *d_scale, void *hip_stream);

/*
 * SeilSearch (Alg. 5) for given tables and probe lists, plus the top-bigK queue:
 * every member of a probed list is scored once (shared cells once per query, miscellaneous
 * duplicates removed) with score = sum_m lut[m][code_m] as an unsigned 16-bit integer.
 *   d_lut        device [nq][M][16] uint8
 *   d_probe_ids  device [nq][nprobe] int32, distinct valid list ids per row, any order
 *   d_cand_ids   device [nq][refine_k] int64: the refine_k smallest (score, id), padded with -1
 *   d_cand_score device [nq][refine_k] int32 (padded with -1), may be NULL
 *   d_dco        device [nq] int64 items scored (one per valid slot of every scanned block),
 *                may be NULL
 */
int rairs_scan(rairs_index_t *h, const uint8_t *d_lut, const int32_t *d_probe_ids, int64_t nq,
               int nprobe, int refine_k, int64_t *d_cand_ids, int32_t *d_cand_score,
               int64_t *d_dco, void *hip_stream);

/*
 * Refine (Alg. 2, the refine step): exact distances of the candidates, K smallest by (distance, id).
 *   d_cand_ids device [nq][refine_k] int64, entries < 0 are ignored.
 */
int rairs_refine(rairs_index_t *h, const float *d_queries, const int64_t *d_cand_ids, int64_t nq,
                 int refine_k, int k, int64_t *d_out_ids, float *d_out_dists, void *hip_stream);

/*
 * Which kernels SeilSearch uses.  RAIRS_SCAN_AUTO (default): a score bound per query from a
 * sample of its first probed list, then the list-major MFMA kernel over all probed lists (tables
 * in registers for M = 16, 48, 64, in LDS for any other M), selection of the bigK best survivors,
 * and the exact one-workgroup-per-query kernel for queries whose survivors do not fit their buffer.
 * RAIRS_SCAN_EXACT: the exact kernel for everything.  Results are identical in both modes.
 */
enum { RAIRS_SCAN_AUTO = 0, RAIRS_SCAN_EXACT = 1 };
int rairs_set_scan_mode(rairs_index_t *h, int mode);

/* ---- measurement --------------------------------------------------------------------------- */

/* SCAN is the whole SeilSearch stage (probe bitmap, sample bound, grouping, main scan kernel,
   selection, overflow redo); SCAN_KERNEL is its dominant kernel alone: the list-major MFMA scan,
   or the exact scan when that one runs instead. */
enum { RAIRS_STAGE_COARSE = 0, RAIRS_STAGE_LUT = 1, RAIRS_STAGE_SCAN = 2, RAIRS_STAGE_REFINE = 3,
       RAIRS_STAGE_SCAN_KERNEL = 4, RAIRS_NSTAGES = 5 };

/*
 * Stage timing of rairs_search with HIP events: 0 = off; RAIRS_PROFILE_STAGES = every stage is
 * bracketed; RAIRS_PROFILE_SCAN_KERNEL = only the dominant scan kernel (every event recorded
 * between two kernels delays the second by some microseconds; this level adds two).
 * Stages that were not timed read -1 in rairs_get_stage_ms.
 */
enum { RAIRS_PROFILE_STAGES = 1, RAIRS_PROFILE_SCAN_KERNEL = 2 };
int rairs_set_profiling(rairs_index_t *h, int level);

/*
 * Milliseconds per stage of the last rairs_search (host array of RAIRS_NSTAGES floats).
 * Synchronises on the recorded events.  RAIRS_EINVAL if profiling was off.
 */
int rairs_get_stage_ms(rairs_index_t *h, float *ms);

/*
 * The same, averaged over the last `last_n` profiled searches (1 <= last_n <= 64 and no more than
 * were recorded since profiling was switched on): each search records into its own slot of a ring
 * of events, so a timed loop needs no host synchronisation between its steps.
 */
int rairs_get_stage_ms_mean(rairs_index_t *h, int last_n, float *ms);

/* Items scored per query by the last rairs_search (counted by the scan kernels, block by block,
   as they score): device [nq] int64 copied to host `dco`. */
int rairs_get_dco(rairs_index_t *h, int64_t *dco, int64_t nq);

/*
 * Counters of the last rairs_search / rairs_scan pass (host array of 5): queries redone by the
 * exact kernel after their survivor buffer overflowed; sum, maximum of survivors per query (the
 * logged pairs that are within the query's final bound); number of queries in the pass; pairs the
 * scan logged in all (the ratio to the survivors says how early the bounds tightened).
 * Synchronises the device.  Zeros when the exact kernel ran alone.
 */
int rairs_get_scan_stats(rairs_index_t *h, int64_t *stats);

/*
 * Name of the dominant kernel that SeilSearch launches for this index in the current scan mode:
 * "scan_mfma_kernel" (2:4-sparse int8 matrix instruction, tables in registers),
 * "scan_mfma_lds_kernel" (dense int8 matrix instruction, tables in LDS) or "scan_exact_kernel"
 * (table lookups on the vector units).  A static string; NULL for a NULL handle.
 */
const char *rairs_scan_kernel_name(const rairs_index_t *h);

/* Bytes of device memory held by the index (codes, ids, tags, directory, raw vectors, ...). */
int rairs_index_bytes(const rairs_index_t *h, int64_t *code_bytes, int64_t *total_bytes);

/*
 * RairAssign (Alg. 3), a step of index construction: the two lists of each of n vectors.
 *   d_vectors device [n][d] fp32;  d_pairs device [n][2] int32, the smaller list id first
 * The candidates are the min(n_cands, nlist) nearest lists as rairs_coarse orders them
 * (FindNearestLists); loss[i] = ||r_i||^2 + lambda <r_0, r_i> with r_i = centroid_i - v is taken
 * in float64, both sums in dimension order, no fused multiply-add; the secondary list is the
 * first minimum over candidates 1.. (strict != 0; the primary list itself when there is no other
 * candidate) or 0.. (strict == 0: both ids may be equal, the vector is then stored once).
 * Uses the handle's centroids and workspace (calls on one handle must not overlap); needs
 * 1 <= n_cands and min(n_cands, nlist) <= RAIRS_MAX_NCANDS.  n == 0 is a successful no-op.
 * The AIR loss is a Euclidean criterion (Theorem 1): RAIRS_EUNSUPPORTED for an inner-product index.
 */
#define RAIRS_MAX_NCANDS 32
int rairs_assign(rairs_index_t *h, const float *d_vectors, int64_t n, int n_cands, double lambda,
                 int strict, int32_t *d_pairs, void *hip_stream);

/*
 * PQEncoding (Alg. 1; Section 2.2), a step of index construction: the 4-bit codes of n vectors.
 *   d_codebook device [M][16][d/M] fp32;  d_vectors device [n][d] fp32;
 *   d_codes    device [n][M/2] uint8, byte i: sub-quantizer 2i in the low nibble, 2i+1 in the high
 * code[m] is the nearest of the 16 codewords of sub-quantizer m to sub-vector m, the first one on
 * a tie, with the distances computed as the lookup-table entries of rairs_lut are (fp32, summed
 * in dimension order, no fused multiply-add).  Needs M even, 2 <= M <= RAIRS_MAX_M, d % M == 0 and
 * 64 d bytes of LDS for sub-vectors that are not 1, 2 or 4 long.  No handle, no allocation; the
 * caller owns all three buffers.  n == 0 is a successful no-op.
 */
int rairs_pq_encode(const float *d_codebook, int d, int M, const float *d_vectors, int64_t n,
                    uint8_t *d_codes, void *hip_stream);

const char *rairs_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RAIRS_H */
