// Internal declarations shared by the translation units of librairs (device format + launchers).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rairs.h"

#define RAIRS_EMPTY_ID 0xFFFFFFFFu
#define RAIRS_MAX_NLIST 65536
#define RAIRS_HIST_BINS 64
#define RAIRS_EV_RING 64

// One list of the SEIL directory (Section 5.1): its own blocks are contiguous,
// [blk_begin, blk_begin + shared_cnt) shared-cell blocks then misc_cnt miscellaneous blocks.
struct ListEntry {
    int32_t blk_begin;
    int32_t shared_cnt;
    int32_t misc_cnt;
    int32_t ref_begin;
    int32_t ref_cnt;
    int32_t valid_items;   // non-empty slots in the list's own blocks
    int32_t seg_begin;     // scan segments of the list (own blocks in chunks, then references)
    int32_t seg_cnt;
    int32_t part_begin;    // parts of the list: runs of consecutive segments of about equal work
    int32_t part_cnt;
};

// A run of at most RAIRS_SEG_BLOCKS consecutive blocks that one wave scores for one query tile.
#define RAIRS_SEG_BLOCKS 16
#ifndef RAIRS_PART_BLOCKS
#define RAIRS_PART_BLOCKS 32
#endif
#define RAIRS_PART_SEGS 8
struct SegEntry {
    int32_t blk_begin;
    int32_t nblk;
    int32_t misc_from;     // blocks [misc_from, nblk) of the run are miscellaneous blocks
    int32_t owner;         // -1: the list's own blocks; else the owning list of a referenced cell
    int32_t tail_valid;    // leading slots in use in the run's last block when the rest of it is empty
                           // (else 32: the run does not end its list, or the block has gaps)
};

// Reference entry of list j to the blocks of cell (owner, j) stored in list `owner`.
struct RefEntry {
    int32_t owner;
    int32_t blk_begin;
    int32_t nblocks;
    int32_t valid;         // slots of these blocks that hold an item (all, until items are deleted)
};

// Device view handed to kernels by value.
struct IndexView {
    int32_t d, M, T, nd, nlist, raw_u8;   // T = M / 2 nibbles per parity, nd = ceil(T / 8) dwords
    int32_t metric;                       // RAIRS_METRIC_L2 or RAIRS_METRIC_IP
    int64_t ntotal, nblocks, nrefs;
    const float *centroids;       // [nlist][d]
    const float *centroids_t;     // [d][nlist]
    const float *centroids_ct;    // [d][nlist] centred: fl(c - cmean)
    const float *cmean;           // [d] mean of the centroids
    const float *cnorm;           // [nlist] squared norms of the centred centroids
    float cmax2;                  // largest of them
    const float *codebook;        // [M][16][d/M]
    // codes: per block nd x 64 dwords; lane = parity * 32 + item; dword w of lane (g, item) packs
    // the codes of subspaces 2t+g, t = 8w .. 8w+7, nibble (t & 7) at bits 4*(t & 7)
    const uint32_t *codes;
    const uint32_t *ids;          // [nblocks][32], RAIRS_EMPTY_ID = empty slot
    const int32_t *other;         // [nblocks][32]
    const uint2 *idtag;           // [nblocks][32] {id, other} of each slot side by side
    // [nblocks] bit i: slot i holds an item that the duplicate rule can never drop (a shared
    // block's item, or a miscellaneous item whose other list has no smaller id than the list)
    const uint32_t *cmask;
    const uint32_t *vmask;        // [nblocks] bit i: slot i holds an item
    const uint2 *bmask;           // [nblocks] {cmask, vmask} side by side: one fetch per scanned block
    const int32_t *blk_list;      // [nblocks] the list that stores the block (-1: none)
    const ListEntry *lists;       // [nlist]
    const RefEntry *refs;         // [nrefs]
    const SegEntry *segs;         // [nsegs]
    // first segment (absolute) of every part, list by list, each list's run closed by the index
    // one past its last segment: part p of list L is segments [parts[L.part_begin + p],
    // parts[L.part_begin + p + 1]).  A part holds at most RAIRS_PART_SEGS segments and, unless a
    // single segment is larger, at most RAIRS_PART_BLOCKS blocks.
    const int32_t *parts;
    const void *raw;              // [ntotal][d] fp32 or u8
};

struct rairs_index {
    IndexView v;
    void *dev_alloc[24];
    int64_t nsegs, nparts;
    int max_parts;                // most parts in any list (bounds the work-unit table)
    int ndev_alloc;
    int64_t code_bytes, total_bytes;
    // workspace: the caller's (rairs_set_workspace), else the handle's own, grown on demand
    void *ws;
    size_t ws_bytes;
    void *ws_user;
    size_t ws_user_bytes;
    void *graph_ws;               // workspace of the graph being captured (rairs_graph_create only)
    size_t graph_ws_bytes;
    char *last_ws;                // workspace of the last call (for the measurement helpers)
    int64_t *last_dco;            // DCO counts of the last rairs_search, inside that workspace
    int64_t last_dco_n;
    // profiling
    int force_exact;
    int64_t last_pass_n;          // queries of the last MFMA pass (0: none)
    size_t last_flags_off, last_cnt_off, last_fill_off;
    int last_log_chunks;
    int prof, prof_valid;
    float stage_ms[RAIRS_NSTAGES];
    // stage events of the last RAIRS_EV_RING profiled searches (slot = search number mod ring)
    hipEvent_t ev[RAIRS_EV_RING][2 * RAIRS_NSTAGES];
    int ev_ready;
    int64_t ev_count;             // profiled single-pass searches recorded so far
    // a second stream for the steps that do not depend on each other (tables next to the coarse
    // quantizer, grouping next to the sample bound), forked from and joined to the caller's stream
    hipStream_t side;
    hipEvent_t ev_fork, ev_lut, ev_probe, ev_group, ev_scored;
    int side_ready;
};

void rairs_set_error(const char *fmt, ...);

#define RAIRS_HIP(call)                                                              \
    do {                                                                             \
        hipError_t e_ = (call);                                                      \
        if (e_ != hipSuccess) {                                                      \
            rairs_set_error("%s failed: %s", #call, hipGetErrorString(e_));          \
            return RAIRS_EHIP;                                                       \
        }                                                                            \
    } while (0)

// launchers (kernels.hip)
int rairs_launch_pack(const uint8_t *d_codes_host_layout, const int64_t *d_ids64, int64_t blk0,
                      int64_t nblk, int M, int nd, uint32_t *codes, uint32_t *ids,
                      hipStream_t s);
int rairs_launch_pair_ids(const uint32_t *ids, const int32_t *other, int64_t n, uint2 *out, hipStream_t s);
int rairs_launch_transpose(const float *d_in, int rows, int cols, float *d_out, hipStream_t s);
// dmat: [nq][nlist] words of scratch; flags: [nq] words of scratch (null: full route only)
// scored (may be null; only with rairs_coarse_has_scores): recorded on s once the score matrix of
// the matrix-core route is complete; the selection kernels then run on s_select behind it
int rairs_launch_coarse(const IndexView &v, const float *q, int64_t nq, int nprobe, float *dmat,
                        int32_t *probe_ids, float *probe_dists, uint32_t *flags, hipStream_t s,
                        hipEvent_t scored = nullptr, hipStream_t s_select = nullptr);
// whether rairs_launch_coarse takes the matrix-core route for these arguments (given flags), i.e.
// leaves the keys of all (query, list) pairs in dmat; and the list of each row's smallest key
bool rairs_coarse_has_scores(const IndexView &v, int nprobe, const float *q);
int rairs_launch_coarse_first(const IndexView &v, const float *dmat, int64_t nq, int32_t *first, hipStream_t s);
int rairs_launch_bitmap(const IndexView &v, const int32_t *probe_ids, int64_t nq, int nprobe,
                        uint32_t *bitmap, int bmwords, uint32_t *hist, hipStream_t s);
int rairs_launch_lut(const IndexView &v, const float *q, int64_t nq, uint8_t *lut, float *bias_sum,
                     float *scale, hipStream_t s);
// construction side (kernels.hip): PQ codes of n vectors (Section 2.1), and the two lists of every
// vector from its nc nearest centroids `cand` by the AIR loss (Section 4.2, Equation 2)
int rairs_launch_pq_encode(const float *cb, int d, int M, const float *x, int64_t n, uint8_t *codes,
                           hipStream_t s);
int rairs_launch_air_assign(const IndexView &v, const float *x, int64_t n, int nc, double lambda,
                            int strict, const int32_t *cand, int32_t *out, hipStream_t s);
// arguments of the exact scan kernel (scan_exact.hip)
struct ExactScanArgs {
    const uint8_t *lut;           // [nq][M][16]
    const int32_t *probe_ids;     // [nq][nprobe]
    const uint32_t *bitmap;       // [nq][bmwords]
    int bmwords, nprobe, refine_k;
    const uint32_t *only_flagged; // if set, queries with a zero flag are skipped
    const uint32_t *redo;         // if set: {count, query ...}, the flagged queries as a list (one pass of a small grid
                                  // over it instead of a workgroup per query of the batch)
    int64_t *cand_ids;            // [nq][refine_k]
    int32_t *cand_score;          // [nq][refine_k], may be null
    int64_t *dco;                 // [nq], may be null
};
int rairs_launch_scan_exact(const IndexView &v, const ExactScanArgs &a, int64_t nq, hipStream_t s);
#define RAIRS_SAMPLE_MAX_BLOCKS 128
#define RAIRS_LOG_CHUNK 2048        // entries of a chunk of the survivor log
// bound of every query from the head of its first probed list
int rairs_launch_sample_bound(const IndexView &v, const uint8_t *lut, const int32_t *probe_ids,
                              int nprobe, int refine_k, int sample_blocks, int64_t nq, int32_t *tau,
                              int32_t *bound, hipStream_t s);
// the same bound from scores that rairs_launch_sample_scores wrote
// (the sampled list of query q is first[q * stride]; with check_ids, a query whose sampled list is
// not among its check_n probe lists gets no bound)
int rairs_launch_sample_rank(const IndexView &v, const int32_t *first, int stride, int refine_k,
                             int sample_blocks, int64_t nq, const uint16_t *pre, int32_t *tau,
                             int32_t *bound, hipStream_t s, const int32_t *check_ids = nullptr,
                             int check_n = 0);
// Scores of the sample by the matrix cores: the queries are grouped by their first probed list, a
// wave scores the head of a list for a tile of up to 32 of them.  Workspace: s_cnt [nlist],
// s_off [nlist + 1], s_toff [nlist + 1], s_q [nq], s_tiles [nq / 32 + nlist].
bool rairs_sample_scores_supported(const IndexView &v, int64_t nq);
int rairs_launch_sample_group(const IndexView &v, const int32_t *probe_ids, int nprobe, int64_t nq,
                              int32_t *s_off, int32_t *s_toff, int32_t *s_q, int32_t *s_tiles,
                              hipStream_t s);
int rairs_launch_sample_scores(const IndexView &v, const uint8_t *lut, int sample_blocks, int64_t nq,
                               const int32_t *s_off, const int32_t *s_toff, const int32_t *s_q,
                               const int32_t *s_tiles, uint16_t *scores, hipStream_t s);

// list-major MFMA scan (scan_mfma.hip)
struct MfmaScanArgs {
    const uint8_t *lut;
    const int32_t *probe_ids;
    const uint32_t *bitmap;
    int bmwords, nprobe, refine_k;
    int p_first;                  // probes [p_first, nprobe) are scanned here
    int64_t nq;
    // workspace
    int32_t *lcount;              // [nlist]   queries probing each list
    int32_t *loff;                // [nlist+1] exclusive prefix of lcount
    int32_t *lcursor;             // [nlist]
    int32_t *qlist;               // [nq * nprobe] query ids grouped by list
    int32_t *toff;                // [nlist+1] exclusive prefix of work units per list
    int32_t *unit_list;           // [units] list of every work unit
    int32_t *unit_rec;            // [units][8] {list, tile, first segment, end segment, first query of the list in qlist, its queries, 0, 0}
    int unit_parts;               // parts per unit, 1..4
    int unit_tail_from;           // lists from this one on: single-part units (nlist: none)
    uint32_t *next_task;          // [1]
    const int32_t *tau;           // [nq] bound from the sample (0xFFFF: none); fixes the histogram range
    int32_t *bound;               // [nq] current bound, starts at tau, only decreases
    uint32_t *hist;               // [nq][RAIRS_HIST_BINS]
    uint32_t *surv_cnt;           // [nq]
    uint64_t *surv_buf;           // [nq][surv_cap]
    int surv_cap;
    uint32_t *flags;              // [nq] set when the survivor buffer overflowed
    uint32_t *work;               // [2][1 + nq] {count, query ...}: queries for the workgroup-wide select; flagged queries
    uint2 *log;                   // [log_chunks][RAIRS_LOG_CHUNK] survivor log {slot, score << 16 | query of the pass}
    uint32_t *chunk_fill;         // [log_chunks] entries written to each chunk
    uint32_t *log_cursor;         // [1] chunks handed out
    uint32_t *log_overflow;       // [1] set if the log ran out of chunks
    int log_chunks;
    unsigned long long *dco;      // [nq] items scored per query, counted as blocks are contracted; may be null
    int any_order;                // the bigK candidates may be written in any order (the whole search: refine orders them anyway)
    int64_t *cand_ids;            // [nq][refine_k]
    int32_t *cand_score;          // may be null
};
bool rairs_mfma_supported(const IndexView &v);
bool rairs_mfma_reg_tables(const IndexView &v);    // the tile's tables fit the registers (sparse instruction)
int64_t rairs_scan_log_waves(const IndexView &v, int64_t units);    // most waves that own log chunks at once, for a pass of at most `units` units
// grouping of the (query, probed list) pairs by list and the unit table, then the scan itself
int rairs_launch_group(const IndexView &v, const MfmaScanArgs &a, hipStream_t s);
int rairs_launch_scan_mfma(const IndexView &v, const MfmaScanArgs &a, hipStream_t s, hipEvent_t *ev);
int rairs_launch_select(const IndexView &v, const MfmaScanArgs &a, hipStream_t s);
// behind it: the workgroup-wide select and the exact redo for the queries on the two lists in a.work
int rairs_launch_scan_repair(const IndexView &v, const MfmaScanArgs &ma, const ExactScanArgs &a, hipStream_t s);
int rairs_launch_refine(const IndexView &v, const float *q, const int64_t *cand_ids, int64_t nq,
                        int refine_k, int k, int64_t *out_ids, float *out_dists, hipStream_t s);
