// HIP kernels (gfx950, wave64) of the RAIRS query path: coarse quantizer, lookup tables,
// refinement (the scans are in scan_mfma.hip and scan_exact.hip), and of two steps of index
// construction: PQ encoding and the AIR loss of RairAssign.  Built with -ffp-contract=off: the
// floating-point operation order below is part of the results' definition.
#include "device_util.h"

// ---------------------------------------------------------------------------------------------
// upload helpers
// ---------------------------------------------------------------------------------------------

// canonical [blk][32 items][T bytes] (low nibble = even subspace) -> device dword layout
__global__ void pack_codes_kernel(const uint8_t *in, int64_t nblk, int T, int nd, uint32_t *out)
{
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = nblk * nd * 64;
    if (gid >= total) return;
    int lane = (int)(gid & 63);
    int64_t bw = gid >> 6;
    int w = (int)(bw % nd);
    int64_t b = bw / nd;
    int g = lane >> 5, item = lane & 31;
    const uint8_t *row = in + ((size_t)b * 32 + item) * T;
    uint32_t v = 0;
    for (int n = 0; n < 8; n++) {
        int t = 8 * w + n;
        if (t < T) {
            uint32_t byte = row[t];
            uint32_t nib = g ? (byte >> 4) : (byte & 15u);
            v |= nib << (4 * n);
        }
    }
    out[gid] = v;
}

__global__ void pack_ids_kernel(const int64_t *in, int64_t n, uint32_t *out)
{
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < n) out[gid] = in[gid] < 0 ? RAIRS_EMPTY_ID : (uint32_t)in[gid];
}

// (id, other-list tag) of every slot side by side, so that the selection gathers one 8-byte word
// per survivor instead of two 4-byte words from different arrays
__global__ void pair_ids_kernel(const uint32_t *ids, const int32_t *other, int64_t n, uint2 *out)
{
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < n) out[gid] = make_uint2(ids[gid], (uint32_t)other[gid]);
}

int rairs_launch_pair_ids(const uint32_t *ids, const int32_t *other, int64_t n, uint2 *out, hipStream_t s)
{
    if (n == 0) return RAIRS_OK;
    hipLaunchKernelGGL(pair_ids_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, ids, other, n, out);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

int rairs_launch_pack(const uint8_t *d_codes, const int64_t *d_ids64, int64_t blk0, int64_t nblk,
                      int M, int nd, uint32_t *codes, uint32_t *ids, hipStream_t s)
{
    if (nblk == 0) return RAIRS_OK;
    int64_t total = nblk * nd * 64;
    hipLaunchKernelGGL(pack_codes_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       d_codes, nblk, M / 2, nd, codes + (size_t)blk0 * nd * 64);
    int64_t n = nblk * 32;
    hipLaunchKernelGGL(pack_ids_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                       d_ids64, n, ids + (size_t)blk0 * 32);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

__global__ void transpose_kernel(const float *in, int rows, int cols, float *out)
{
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (int64_t)rows * cols) return;
    int r = (int)(gid / cols), c = (int)(gid % cols);
    out[(size_t)c * rows + r] = in[gid];
}

int rairs_launch_transpose(const float *d_in, int rows, int cols, float *d_out, hipStream_t s)
{
    int64_t n = (int64_t)rows * cols;
    hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, d_in,
                       rows, cols, d_out);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

// ---------------------------------------------------------------------------------------------
// coarse quantizer: FindNearestLists for the batch (Alg. 2)
// ---------------------------------------------------------------------------------------------
//
// The result is defined by the direct form: dist(q, l) = sum_i (q_i - c_li)^2 in fp32, summed as 64
// interleaved partial sums over the dimensions (class = dimension mod 64) folded pairwise at
// strides 32..1; the nprobe smallest (dist, list id) win.  With the inner-product metric the score
// of a list is -sum_i q_i c_li in the same order (the nprobe largest products win, ties to the
// smaller list id) and everything below holds with that score in place of the distance, the
// matrix-core form being s(q, l) = -q.c_l without centring.  Scores travel as order-preserving
// unsigned keys (f32_key), so negative ones sort correctly.  Two routes compute it:
//   full:      every (query, list) distance in the direct form, then a selection;
//   shortlist: s(q, l) = |c_l|^2 - 2 q.c_l for all pairs on the fp32 matrix cores, the lists whose
//              s is within a rounding-error margin of the nprobe-th smallest s are re-scored in the
//              direct form, and the selection is made among those.  The margin makes the shortlist
//              a superset of the true winners, so both routes return the same bits; a query whose
//              shortlist does not fit falls back to the full route.

typedef float v16f __attribute__((ext_vector_type(16)));

// order-preserving map of an fp32 value to an unsigned key, and back
static __device__ __forceinline__ uint32_t f32_key(float x)
{
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
static __device__ __forceinline__ float key_f32(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

// direct-form score (squared distance, or minus the inner product) of a query to list l of the
// transposed centroid matrix ct[d][nlist]
static __device__ __forceinline__ float direct_l2_t(const float *__restrict__ qq,
                                                    const float *__restrict__ ct, int d, int nlist, int l,
                                                    int metric)
{
    float p[64];
#pragma unroll
    for (int j = 0; j < 64; j++) p[j] = 0.0f;
    for (int i0 = 0; i0 < d; i0 += 64) {
#pragma unroll
        for (int j = 0; j < 64; j++) {
            int i = i0 + j;
            if (i < d) {
                const float c = ct[(size_t)i * nlist + l];
                float diff = qq[i] - c;
                float sq = metric ? qq[i] * c : diff * diff;
                p[j] = p[j] + sq;
            }
        }
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
#pragma unroll
        for (int j = 0; j < s; j++) p[j] = p[j] + p[j + s];
    }
    return metric ? -p[0] : p[0];
}

// Full route, distances: one lane per (query, list), lists strided over the y dimension of the
// grid.  With only_flagged set, queries whose flag is zero are left alone.
__global__ __launch_bounds__(WG) void coarse_dist_kernel(const float *__restrict__ q,
                                                         const float *__restrict__ ct, int d,
                                                         int nlist, uint32_t *__restrict__ dmat,
                                                         const uint32_t *__restrict__ only_flagged,
                                                         int metric)
{
    const int64_t qi = blockIdx.x;
    if (only_flagged && only_flagged[qi] == 0) return;
    const float *qq = q + (size_t)qi * d;
    for (int l = blockIdx.y * WG + threadIdx.x; l < nlist; l += gridDim.y * WG)
        dmat[(size_t)qi * nlist + l] = f32_key(direct_l2_t(qq, ct, d, nlist, l, metric));
}

// Full route, selection: the nprobe smallest (score, list id) of a row by radix select on the
// order-preserving keys, then sorted.  One workgroup per query.
__global__ __launch_bounds__(WG) void coarse_select_kernel(uint32_t *dmat,
                                                           int nlist, int nprobe,
                                                           int32_t *__restrict__ probe_ids,
                                                           float *__restrict__ probe_dists,
                                                           const uint32_t *__restrict__ only_flagged,
                                                           const float *__restrict__ q,
                                                           const float *__restrict__ ct, int d, int metric)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_prefix, s_remaining, s_cnt;
    __shared__ int wcnt[WG / 64];
    __shared__ uint64_t sel[RAIRS_MAX_NPROBE];
    const int tid = threadIdx.x;
    if (only_flagged && only_flagged[blockIdx.x] == 0) return;
    if (q) {
        // the row's distances first (same arithmetic as coarse_dist_kernel), by this workgroup
        uint32_t *drow = dmat + (size_t)blockIdx.x * nlist;
        const float *qq = q + (size_t)blockIdx.x * d;
        for (int l = tid; l < nlist; l += WG) drow[l] = f32_key(direct_l2_t(qq, ct, d, nlist, l, metric));
        __threadfence_block();
        __syncthreads();
    }
    const uint32_t *row = dmat + (size_t)blockIdx.x * nlist;

    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)nprobe;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < nlist; i += WG) {
            uint32_t key = row[i];
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t cum = 0;
            for (int b = 0; b < 256; b++) {
                uint32_t h = hist[b];
                if (cum + h >= remaining) {
                    s_prefix = prefix | ((uint32_t)b << shift);
                    s_remaining = remaining - cum;
                    break;
                }
                cum += h;
            }
        }
        __syncthreads();
        prefix = s_prefix;
        remaining = s_remaining;
        mask |= 255u << shift;
        __syncthreads();
    }
    // prefix is now the key of the nprobe-th smallest score; `remaining` of the keys
    // equal to it are needed, the ones with the smallest list ids.
    const uint32_t kth = prefix;
    if (tid == 0) s_cnt = 0;
    __syncthreads();
    for (int i = tid; i < nlist; i += WG) {
        uint32_t key = row[i];
        if (key < kth) {
            uint32_t pos = atomicAdd(&s_cnt, 1u);
            sel[pos] = ((uint64_t)key << 32) | (uint32_t)i;
        }
    }
    __syncthreads();
    const uint32_t base = s_cnt;
    uint32_t running = 0;
    const int wave = tid >> 6, lane = tid & 63;
    for (int i0 = 0; i0 < nlist && running < remaining; i0 += WG) {
        int i = i0 + tid;
        bool flag = i < nlist && row[i] == kth;
        unsigned long long b = __ballot(flag);
        if (lane == 0) wcnt[wave] = __popcll(b);
        __syncthreads();
        uint32_t off = running + (uint32_t)__popcll(b & ((1ull << lane) - 1ull));
        uint32_t tot = 0;
        for (int w = 0; w < WG / 64; w++) {
            if (w < wave) off += wcnt[w];
            tot += wcnt[w];
        }
        if (flag && off < remaining) sel[base + off] = ((uint64_t)kth << 32) | (uint32_t)i;
        running += tot;
        __syncthreads();
    }
    const int n2 = next_pow2(nprobe);
    for (int i = nprobe + tid; i < n2; i += WG) sel[i] = ~0ull;
    __syncthreads();
    bitonic_sort_lds(sel, n2);
    for (int i = tid; i < nprobe; i += WG) {
        uint64_t key = sel[i];
        probe_ids[(size_t)blockIdx.x * nprobe + i] = (int32_t)(uint32_t)key;
        if (probe_dists) {
            const float sc = key_f32((uint32_t)(key >> 32));
            probe_dists[(size_t)blockIdx.x * nprobe + i] = metric ? -sc : sc;    // reported: the product itself
        }
    }
}

// Shortlist route, scores: keys[q][l] = f32_key(|c'_l|^2 - 2 q'.c'_l) with v_mfma_f32_32x32x2f32,
// where q' = fl(q - cmean) and c' = fl(c - cmean) are the centred query and centroid.
// A workgroup takes 128 queries (32 per wave, kept in registers: lane (row i, half k) holds
// q_i[k*D/2 + s], s < D/2) and walks over tiles of 32 lists.  A tile's centroids are staged in LDS
// in operand order, element (s, k, j) = ct[k*D/2 + s][l0 + j] at s*64 + k*32 + j, so that the B
// operand of step s is one conflict-free 4-byte read per lane; the next tile is fetched into
// registers while the current one is multiplied (two LDS buffers, one barrier per tile).
// Result register r of lane (k, j) is row 8*(r/4) + 4*k + r%4, column j.
#define GEMM_QWG 128
template <int D>
__global__ __launch_bounds__(WG) __attribute__((amdgpu_waves_per_eu(D <= 128 ? 3 : 2))) void coarse_gemm_kernel(const float *__restrict__ q,
                                                         const float *__restrict__ ct,
                                                         const float *__restrict__ cmean,
                                                         const float *__restrict__ cnorm, int nlist,
                                                         int csplits, int tiles_per_split, int64_t nq,
                                                         uint32_t *__restrict__ keys, float alpha)
{
    constexpr int H = D / 2;
    constexpr int PER = D * 32 / WG;                    // staged elements per thread and tile
    __shared__ float Bs[2][D * 32];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, i = lane & 31, k = lane >> 5;
    // workgroups that share an L2 (consecutive ids go round the 8 dies) take the same lists
    int qblock, csplit;
    if ((csplits & 7) == 0) {
        const int per = csplits >> 3, x = blockIdx.x & 7, y = blockIdx.x >> 3;
        csplit = x * per + y % per;
        qblock = y / per;
    } else {
        csplit = blockIdx.x % csplits;
        qblock = blockIdx.x / csplits;
    }
    const int64_t q0 = (int64_t)qblock * GEMM_QWG + wave * 32;
    const int64_t qrow = q0 + i < nq ? q0 + i : nq - 1;
    float A[H];                                         // centred: fl(q - cmean)
    {
        const float4 *src = (const float4 *)(q + (size_t)qrow * D + k * H);
        const float4 *mu = (const float4 *)(cmean + k * H);
#pragma unroll
        for (int s4 = 0; s4 < H / 4; s4++) {
            const float4 x = src[s4], m = mu[s4];
            A[4 * s4] = x.x - m.x; A[4 * s4 + 1] = x.y - m.y; A[4 * s4 + 2] = x.z - m.z; A[4 * s4 + 3] = x.w - m.w;
        }
    }
    const int ntiles = (nlist + 31) >> 5;
    const int t_begin = csplit * tiles_per_split;
    const int t_end = t_begin + tiles_per_split < ntiles ? t_begin + tiles_per_split : ntiles;
    if (t_begin >= t_end) return;                       // uniform for the workgroup
    // staging: thread -> column sj, rows sr + 8 * e (row = dimension k*H + s)
    const int sj = threadIdx.x & 31, sr = threadIdx.x >> 5;
    float st[PER];
    // (a uniform row pointer plus one 32-bit offset per thread: sixteen 64-bit addresses per
    // thread would cost the registers that decide whether a third wave fits a SIMD)
    auto fetch = [&](int t) {
        const int l = t * 32 + sj;
        const uint32_t off = (uint32_t)sr * (uint32_t)nlist + (uint32_t)(l < nlist ? l : nlist - 1);
#pragma unroll
        for (int e = 0; e < PER; e++) {
            const float *rows = ct + (size_t)(8 * e) * nlist;       // uniform
            st[e] = rows[off];
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int e = 0; e < PER; e++) {
            const int row = sr + 8 * e, kk = row >= H ? 1 : 0, ss = row - kk * H;
            Bs[buf][ss * 64 + kk * 32 + sj] = st[e];
        }
    };
    fetch(t_begin);
    stage(0);
    __syncthreads();
    int buf = 0;
    // all 32 rows of the wave are queries of the batch (else: the last block, stores checked one by one)
    const bool whole = q0 + 32 <= nq;
    for (int t = t_begin; t < t_end; t++) {
        const bool more = t + 1 < t_end;
        if (more) fetch(t + 1);
        const int l = t * 32 + i;
        const float cn = cnorm[l < nlist ? l : nlist - 1];          // asked for before the products, used after
        v16f acc;
#pragma unroll
        for (int r = 0; r < 16; r++) acc[r] = 0.0f;
        const float *bl = &Bs[buf][lane];
#pragma unroll
        for (int s = 0; s < H; s++)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(A[s], bl[s * 64], acc, 0, 0, 0);
        // alpha = 2: |c'|^2 - 2 q'.c'; alpha = 1 with zero norms: -q.c
        if (l < nlist) {
            if (whole) {
                // a uniform row pointer per result register plus one 32-bit offset per lane
                const uint32_t off = (uint32_t)(4 * k) * (uint32_t)nlist + (uint32_t)l;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    uint32_t *rowp = keys + (size_t)(q0 + 8 * (r >> 2) + (r & 3)) * nlist;      // uniform
                    rowp[off] = f32_key(cn - alpha * acc[r]);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int64_t qq = q0 + 8 * (r >> 2) + 4 * k + (r & 3);
                    if (qq < nq) keys[(size_t)qq * nlist + l] = f32_key(cn - alpha * acc[r]);
                }
            }
        }
        if (more) stage(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
}

// The same scores for any dimension that is a multiple of 8: the dimensions are taken in chunks of
// GEMM_CD; a wave holds the chunk of its 32 queries in registers, the chunk of a list tile is staged
// in LDS, and the NT tiles of the workgroup keep their accumulators across the chunks.
#define GEMM_CD 128
template <int NT>
__global__ __launch_bounds__(WG) void coarse_gemm_chunk_kernel(const float *__restrict__ q,
                                                               const float *__restrict__ ct,
                                                               const float *__restrict__ cmean,
                                                               const float *__restrict__ cnorm, int d,
                                                               int nlist, int ngroups, int64_t nq,
                                                               uint32_t *__restrict__ keys, float alpha)
{
    __shared__ float Bs[GEMM_CD * 32];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, i = lane & 31, k = lane >> 5;
    const int qblock = blockIdx.x / ngroups, grp = blockIdx.x % ngroups;
    const int64_t q0 = (int64_t)qblock * GEMM_QWG + wave * 32;
    const int64_t qrow = q0 + i < nq ? q0 + i : nq - 1;
    const int ntiles = (nlist + 31) >> 5;
    const int sj = threadIdx.x & 31, sr = threadIdx.x >> 5;
    v16f acc[NT];
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[t][r] = 0.0f;
    for (int c0 = 0; c0 < d; c0 += GEMM_CD) {
        const int cd = d - c0 < GEMM_CD ? d - c0 : GEMM_CD;      // multiple of 8
        const int h = cd >> 1;                                   // multiple of 4
        float A[GEMM_CD / 2];
        {
            const float4 *src = (const float4 *)(q + (size_t)qrow * d + c0 + k * h);
            const float4 *mu = (const float4 *)(cmean + c0 + k * h);
#pragma unroll
            for (int s4 = 0; s4 < GEMM_CD / 8; s4++) {
                float4 x = make_float4(0.0f, 0.0f, 0.0f, 0.0f), m = x;
                if (4 * s4 < h) { x = src[s4]; m = mu[s4]; }
                A[4 * s4] = x.x - m.x; A[4 * s4 + 1] = x.y - m.y; A[4 * s4 + 2] = x.z - m.z; A[4 * s4 + 3] = x.w - m.w;
            }
        }
#pragma unroll
        for (int t = 0; t < NT; t++) {
            const int tile = grp * NT + t;
            if (tile < ntiles) {                                 // uniform for the workgroup
                __syncthreads();                                 // the previous chunk has been consumed
                const int l = tile * 32 + sj;
                const float *src = ct + (size_t)c0 * nlist + (l < nlist ? l : nlist - 1);
#pragma unroll
                for (int e = 0; e < GEMM_CD / 8; e++) {
                    const int row = sr + 8 * e;
                    if (row < cd) {
                        const int kk = row >= h ? 1 : 0, ss = row - kk * h;
                        Bs[ss * 64 + kk * 32 + sj] = src[(size_t)row * nlist];
                    }
                }
                __syncthreads();
#pragma unroll
                for (int s = 0; s < GEMM_CD / 2; s++)
                    if (s < h) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(A[s], Bs[s * 64 + lane], acc[t], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < NT; t++) {
        const int l = (grp * NT + t) * 32 + i;
        if (l < nlist) {
            const float cn = cnorm[l];
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int64_t qq = q0 + 8 * (r >> 2) + 4 * k + (r & 3);
                const float two = alpha * acc[t][r];
                if (qq < nq) keys[(size_t)qq * nlist + l] = f32_key(cn - two);
            }
        }
    }
}

// Shortlist route, selection.  One wave per query (four per workgroup, each with its own LDS
// region and no workgroup barrier): find the nprobe-th smallest key, widen it by the margin, gather
// the lists up to there, re-score them in the direct form, sort by (distance, list id), keep nprobe.
//
// Margin.  With u = 2^-24, a = q - cmean, b = c - cmean, N = |a|^2 + max |b|^2 and the exact
// D = |q - c|^2 = |a - b|^2 <= 2 N: the direct form is within (d + 2) u D of D; rounding a and b
// to fp32 moves |a - b|^2 by at most about 4 u N; the GEMM form's dot product is within
// d u |a'||b'|, the norm within u |b'|^2 and the final subtraction within u |s|.  Together
// |direct - (s + |a'|^2)| stays below 4 (d + 4) u N =: e, and every list among the nprobe best by
// the direct form has s <= (nprobe-th smallest s) + 2 e.  The kernel uses 16 (d + 4) u N, twice
// that, against accumulation orders inside the matrix core that are not documented.
//
// The nprobe-th smallest key is found in one pass over the row when a sample allows it: the
// ksamp-th smallest key `est` of the row's first `nsamp` keys is, with ksamp chosen well above the
// sample's share of nprobe, above the nprobe-th smallest of the row; every key <= est is gathered
// (with its list) and sorted, which yields the nprobe-th smallest exactly.  If fewer than nprobe
// keys were gathered, or they do not fit, or est is below the widened threshold, the wave falls back
// to a radix select over the whole row (four passes), which always works.
#define SHORTLIST_SAMPLE 512
template <bool IP>
__global__ __launch_bounds__(WG) void coarse_shortlist_kernel(const uint32_t *__restrict__ keys,
                                                              const float *__restrict__ q,
                                                              const float *__restrict__ cent, int d,
                                                              int nlist, int nprobe, int cap,
                                                              int nsamp, int ksamp,
                                                              const float *__restrict__ cmean,
                                                              float cmax2, int64_t nq,
                                                              int32_t *__restrict__ probe_ids,
                                                              float *__restrict__ probe_dists,
                                                              uint32_t *__restrict__ flags)
{
    __shared__ uint32_t hist_s[WG / 64][256];
    extern __shared__ __align__(16) uint64_t sel_dyn[];      // [WG / 64][cap], cap a power of two
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t qi = (int64_t)blockIdx.x * (WG / 64) + wave;
    if (qi >= nq) return;                                // no workgroup barrier below
    const uint32_t *row = keys + (size_t)qi * nlist;
    uint32_t *hist = hist_s[wave];
    uint64_t *sel = sel_dyn + (size_t)wave * cap;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;

    // |q|^2 and the margin
    const float *qq = q + (size_t)qi * d;
    float qn = 0.0f;
    for (int t = lane; t < d; t += 64) {
        const float a = qq[t] - cmean[t];
        qn += a * a;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) qn += __shfl_xor(qn, off);
    const float margin = 16.0f * (float)(d + 4) * 5.9604645e-8f * (qn + cmax2);
    const bool margin_ok = !(margin != margin) && margin < 3.0e38f;

    uint32_t nc = 0;                                     // lists in the shortlist (their ids in sel[0..nc))
    bool have = false;
    if (nsamp > 0 && margin_ok) {
        // est: the ksamp-th smallest of the sample, by bisection on the key bits (keys in registers)
        // (fetching the row's first 1,024 keys once, for the sample and for the gathering pass
        // below, was slower: 16 more registers held across the bisection)
        uint32_t ks[SHORTLIST_SAMPLE / 64];
#pragma unroll
        for (int u = 0; u < SHORTLIST_SAMPLE / 64; u++) {
            const int l = 64 * u + lane;
            ks[u] = l < nsamp ? row[l] : 0xFFFFFFFFu;
        }
        // (only an upper estimate is needed: the top 20 bits -- sign, exponent, 11 bits of the
        // fraction -- are found and the rest set, which overshoots by under a 2000th of the score)
        uint32_t est = 0;
        for (int bit = 31; bit >= 12; bit--) {
            const uint32_t cand = est | (1u << bit);
            uint32_t below = 0;
#pragma unroll
            for (int u = 0; u < SHORTLIST_SAMPLE / 64; u++) below += (uint32_t)__popcll(__ballot(ks[u] < cand));
            if (below < (uint32_t)ksamp) est = cand;
        }
        est |= 0xFFFu;
        // every key <= est, with its list
        uint32_t ng = 0;
        for (int l0 = 0; l0 < nlist; l0 += 64 * 16) {
            uint32_t kk[16];
#pragma unroll
            for (int u = 0; u < 16; u++) {
                const int l = l0 + 64 * u + lane;
                kk[u] = row[l < nlist ? l : nlist - 1];
            }
#pragma unroll
            for (int u = 0; u < 16; u++) {
                const int l = l0 + 64 * u + lane;
                const bool in = l < nlist && kk[u] <= est;
                const unsigned long long m = __ballot(in);
                const uint32_t pos = ng + (uint32_t)__popcll(m & lt_mask);
                if (in && pos < (uint32_t)cap) sel[pos] = ((uint64_t)kk[u] << 32) | (uint32_t)l;
                ng += (uint32_t)__popcll(m);
            }
        }
        if (ng >= (uint32_t)nprobe && ng <= 256u && ng <= (uint32_t)cap) {
            // few entries: no sort.  They go back into registers, the nprobe-th smallest key is
            // found bit by bit, and the entries up to the widened threshold are packed.
            wave_lds_sync();
            uint64_t mine[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const uint32_t i = 64u * u + lane;
                mine[u] = i < ng ? sel[i] : ~0ull;
            }
            uint32_t kth = 0;                            // largest t with fewer than nprobe keys below it
            for (int bit = 31; bit >= 0; bit--) {
                const uint32_t cand = kth | (1u << bit);
                uint32_t below = 0;
#pragma unroll
                for (int u = 0; u < 4; u++)
                    if (64u * u < ng) below += (uint32_t)__popcll(__ballot((uint32_t)(mine[u] >> 32) < cand));
                if (below < (uint32_t)nprobe) kth = cand;
            }
            const uint32_t thr = f32_key(key_f32(kth) + margin);
            if (thr <= est) {
                wave_lds_sync();                         // every lane holds its entries
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    if (64u * u < ng) {
                        const bool in = 64u * u + lane < ng && (uint32_t)(mine[u] >> 32) <= thr;
                        const unsigned long long m = __ballot(in);
                        if (in) sel[nc + (uint32_t)__popcll(m & lt_mask)] = (uint64_t)(uint32_t)mine[u];
                        nc += (uint32_t)__popcll(m);
                    }
                }
                have = true;
            }
        } else if (ng >= (uint32_t)nprobe && ng <= (uint32_t)cap) {
            const int n2 = next_pow2((int)ng < 2 ? 2 : (int)ng);
            for (int e = (int)ng + lane; e < n2; e += 64) sel[e] = ~0ull;
            wave_lds_sync();
            wave_bitonic_sort_lds(sel, n2, lane);
            const uint32_t kth = (uint32_t)(sel[nprobe - 1] >> 32);
            const uint32_t thr = f32_key(key_f32(kth) + margin);
            if (thr <= est) {
                // the sorted entries up to thr are the shortlist
                for (int e0 = 0; e0 < (int)ng; e0 += 64) {
                    const int e = e0 + lane;
                    nc += (uint32_t)__popcll(__ballot(e < (int)ng && (uint32_t)(sel[e] >> 32) <= thr));
                }
                have = true;
            }
        }
    }
    bool fits = true;
    if (!have) {
        // radix select of the nprobe-th smallest key over the whole row
        uint32_t prefix = 0, mask = 0, remaining = (uint32_t)nprobe;
        for (int shift = 24; shift >= 0; shift -= 8) {
            for (int b = lane; b < 256; b += 64) hist[b] = 0;
            wave_lds_sync();
            // sixteen keys per lane are fetched together so that their latencies overlap
            for (int l0 = 0; l0 < nlist; l0 += 64 * 16) {
                uint32_t kk[16];
#pragma unroll
                for (int u = 0; u < 16; u++) {
                    const int l = l0 + 64 * u + lane;
                    kk[u] = row[l < nlist ? l : nlist - 1];
                }
#pragma unroll
                for (int u = 0; u < 16; u++)
                    if (l0 + 64 * u + lane < nlist && (kk[u] & mask) == prefix)
                        atomicAdd(&hist[(kk[u] >> shift) & 255u], 1u);
            }
            wave_lds_sync();
            // the bin where the running count reaches `remaining`: four bins per lane + wave scan
            uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
            uint32_t tot = h0 + h1 + h2 + h3, incl = tot;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                uint32_t up = (uint32_t)__shfl_up((int)incl, off);
                if (lane >= off) incl += up;
            }
            const uint32_t excl = incl - tot;
            const bool here = excl < remaining && incl >= remaining;       // exactly one lane
            uint32_t bin = 0, rem = 0;
            if (here) {
                uint32_t cum = excl;
                if (cum + h0 >= remaining) { bin = 4 * lane; rem = remaining - cum; }
                else if (cum + h0 + h1 >= remaining) { bin = 4 * lane + 1; rem = remaining - cum - h0; }
                else if (cum + h0 + h1 + h2 >= remaining) { bin = 4 * lane + 2; rem = remaining - cum - h0 - h1; }
                else { bin = 4 * lane + 3; rem = remaining - cum - h0 - h1 - h2; }
            }
            const unsigned long long who = __ballot(here);
            const int src = __ffsll((long long)who) - 1;
            bin = (uint32_t)__shfl((int)bin, src);
            rem = (uint32_t)__shfl((int)rem, src);
            prefix |= bin << shift;
            remaining = rem;
            mask |= 255u << shift;
            wave_lds_sync();
        }
        const uint32_t thr = f32_key(key_f32(prefix) + margin);
        // gather the shortlist
        for (int l0 = 0; l0 < nlist; l0 += 64 * 16) {
            uint32_t kk[16];
#pragma unroll
            for (int u = 0; u < 16; u++) {
                const int l = l0 + 64 * u + lane;
                kk[u] = row[l < nlist ? l : nlist - 1];
            }
#pragma unroll
            for (int u = 0; u < 16; u++) {
                const int l = l0 + 64 * u + lane;
                const bool in = l < nlist && kk[u] <= thr;
                const unsigned long long m = __ballot(in);
                const uint32_t pos = nc + (uint32_t)__popcll(m & lt_mask);
                if (in && pos < (uint32_t)cap) sel[pos] = (uint64_t)(uint32_t)l;
                nc += (uint32_t)__popcll(m);
            }
        }
        fits = nc <= (uint32_t)cap && margin_ok;
        if (!fits) nc = 0;
    }
    if (lane == 0) flags[qi] = fits ? 0u : 1u;
    wave_lds_sync();
    // Re-score in the direct form, eight lists per step, two per group of 16 lanes: lane l of a
    // group sums the dimensions of the classes l, l + 16, l + 32, l + 48 (mod 64) in four
    // registers, so the strides 32 and 16 of the defined butterfly are sums inside the lane (the
    // same operands in the same pairing) and only strides 8 to 1 cross lanes.
    {
        constexpr int RU = 2;
        const int grp = lane >> 4, l16 = lane & 15;
        for (uint32_t c0 = 0; c0 < nc; c0 += 4 * RU) {
            uint32_t ls[RU];
            float p[RU][4];
            const float *crow[RU];
#pragma unroll
            for (int u = 0; u < RU; u++) {
                const uint32_t c = c0 + 4 * u + grp;
                ls[u] = (uint32_t)sel[c < nc ? c : nc - 1];
                crow[u] = cent + (size_t)ls[u] * d;
                p[u][0] = p[u][1] = p[u][2] = p[u][3] = 0.0f;
            }
            int i0 = 0;
            for (; i0 + 64 <= d; i0 += 64) {             // whole rounds of 64 dimensions: no lane checks
                float qv[4], x[RU][4];
#pragma unroll
                for (int cc = 0; cc < 4; cc++) {
                    qv[cc] = qq[i0 + l16 + 16 * cc];
#pragma unroll
                    for (int u = 0; u < RU; u++) x[u][cc] = crow[u][i0 + l16 + 16 * cc];
                }
#pragma unroll
                for (int u = 0; u < RU; u++)
#pragma unroll
                    for (int cc = 0; cc < 4; cc++) {
                        float sq;
                        if (IP) sq = qv[cc] * x[u][cc];
                        else { const float diff = qv[cc] - x[u][cc]; sq = diff * diff; }
                        p[u][cc] = p[u][cc] + sq;
                    }
            }
            if (i0 < d) {                                // the last, partial round
#pragma unroll
                for (int cc = 0; cc < 4; cc++) {
                    const int i = i0 + l16 + 16 * cc;
                    if (i < d) {
                        const float qv = qq[i];
#pragma unroll
                        for (int u = 0; u < RU; u++) {
                            const float x = crow[u][i];
                            float sq;
                            if (IP) sq = qv * x;
                            else { const float diff = qv - x; sq = diff * diff; }
                            p[u][cc] = p[u][cc] + sq;
                        }
                    }
                }
            }
            wave_lds_sync();                             // every list of the step was read before an entry is rewritten
#pragma unroll
            for (int u = 0; u < RU; u++) {
                const uint32_t c = c0 + 4 * u + grp;
                const float a = p[u][0] + p[u][2], b = p[u][1] + p[u][3];    // stride 32
                float t = a + b;                         // stride 16
                t = t + lane_xor8(t);
                t = t + lane_xor4(t);
                t = t + lane_xor2(t);
                t = t + lane_xor1(t);
                const float dist = IP ? -t : t;
                if (l16 == 0 && c < nc) sel[c] = ((uint64_t)f32_key(dist) << 32) | ls[u];
            }
            wave_lds_sync();
        }
    }
    if (nc <= 64u) {
        // a lane per list: its place in the (distance, list id) order is the number of smaller keys
        wave_lds_sync();
        const uint64_t mine = lane < (int)nc ? sel[lane] : ~0ull;
        int rank = 0;
        for (int j = 0; j < (int)nc; j++) rank += sel[j] < mine ? 1 : 0;      // one address: a broadcast
        if (fits && lane < (int)nc && rank < nprobe) {
            probe_ids[(size_t)qi * nprobe + rank] = (int32_t)(uint32_t)mine;
            if (probe_dists) {
                const float sc = key_f32((uint32_t)(mine >> 32));
                probe_dists[(size_t)qi * nprobe + rank] = IP ? -sc : sc;
            }
        }
        return;
    }
    const int n2 = next_pow2((int)nc < 2 ? 2 : (int)nc);
    for (int e = (int)nc + lane; e < n2; e += 64) sel[e] = ~0ull;
    wave_lds_sync();
    wave_bitonic_sort_lds(sel, n2, lane);
    if (fits)
        for (int e = lane; e < nprobe; e += 64) {
            uint64_t key = sel[e];
            probe_ids[(size_t)qi * nprobe + e] = (int32_t)(uint32_t)key;
            if (probe_dists) {
                const float sc = key_f32((uint32_t)(key >> 32));
                probe_dists[(size_t)qi * nprobe + e] = IP ? -sc : sc;
            }
        }
}

#define SHORTLIST_MAX_NPROBE 1024
static bool coarse_shortlist_ok(const IndexView &v, int nprobe)
{
    return v.d % 8 == 0 && nprobe <= SHORTLIST_MAX_NPROBE && v.nlist >= 64;
}

// The list with the smallest key of every query's row of the score matrix: where the bound's sample
// is taken when it is to start before the probe lists exist.  The keys carry the matrix core's
// rounding, so this list is nearly always, but not provably, the nearest; whoever uses it checks
// that it is among the query's probe lists.  One wave per query.
__global__ __launch_bounds__(WG) void coarse_first_kernel(const uint32_t *__restrict__ keys, int nlist,
                                                          int64_t nq, int32_t *__restrict__ first)
{
    const int lane = threadIdx.x & 63;
    const int64_t qi = (int64_t)blockIdx.x * (WG / 64) + (threadIdx.x >> 6);
    if (qi >= nq) return;
    const uint32_t *row = keys + (size_t)qi * nlist;
    uint64_t best = ~0ull;
    for (int l0 = 0; l0 < nlist; l0 += 64 * 16) {
        uint32_t kk[16];
#pragma unroll
        for (int u = 0; u < 16; u++) {
            const int l = l0 + 64 * u + lane;
            kk[u] = row[l < nlist ? l : nlist - 1];
        }
#pragma unroll
        for (int u = 0; u < 16; u++) {
            const int l = l0 + 64 * u + lane;
            const uint64_t x = ((uint64_t)kk[u] << 32) | (uint32_t)l;
            if (l < nlist && x < best) best = x;
        }
    }
    best = wave_min_u64(best);
    if (lane == 0) first[qi] = (int32_t)(uint32_t)best;
}

bool rairs_coarse_has_scores(const IndexView &v, int nprobe, const float *q)
{
    return coarse_shortlist_ok(v, nprobe) && ((uintptr_t)q & 15) == 0;
}

int rairs_launch_coarse_first(const IndexView &v, const float *dmat, int64_t nq, int32_t *first, hipStream_t s)
{
    hipLaunchKernelGGL(coarse_first_kernel, dim3((unsigned)((nq + WG / 64 - 1) / (WG / 64))), dim3(WG), 0, s,
                       (const uint32_t *)dmat, v.nlist, nq, first);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

int rairs_launch_coarse(const IndexView &v, const float *q, int64_t nq, int nprobe, float *dmat,
                        int32_t *probe_ids, float *probe_dists, uint32_t *flags, hipStream_t s,
                        hipEvent_t scored, hipStream_t s_select)
{
    const int groups = (v.nlist + WG - 1) / WG;
    if (!coarse_shortlist_ok(v, nprobe) || !flags || ((uintptr_t)q & 15) != 0) {
        hipLaunchKernelGGL(coarse_dist_kernel, dim3((unsigned)nq, groups), dim3(WG), 0, s, q,
                           v.centroids_t, v.d, v.nlist, (uint32_t *)dmat, nullptr, v.metric);
        hipLaunchKernelGGL(coarse_select_kernel, dim3((unsigned)nq), dim3(WG), 0, s, (uint32_t *)dmat, v.nlist,
                           nprobe, probe_ids, probe_dists, nullptr, nullptr, nullptr, 0, v.metric);
        RAIRS_HIP(hipGetLastError());
        return RAIRS_OK;
    }
    // each workgroup: 128 queries x a run of list tiles; enough workgroups to fill the chip twice
    // over, but at least 4 tiles per run so that the query registers are loaded rarely
    const int ntiles = (v.nlist + 31) / 32;
    const unsigned qblocks = (unsigned)((nq + GEMM_QWG - 1) / GEMM_QWG);
    int csplits = (int)((1024 + qblocks - 1) / qblocks);
    if (csplits > (ntiles + 3) / 4) csplits = (ntiles + 3) / 4;
    if (csplits >= 8) csplits = csplits / 8 * 8;
    if (csplits < 1) csplits = 1;
    const int tiles_per_split = (ntiles + csplits - 1) / csplits;
    const dim3 grid(qblocks * csplits);
    uint32_t *keys = (uint32_t *)dmat;
    const float alpha = v.metric ? 1.0f : 2.0f;
#define GEMM_CASE(D)                                                                              \
    case D:                                                                                       \
        hipLaunchKernelGGL(coarse_gemm_kernel<D>, grid, dim3(WG), 0, s, q, v.centroids_ct, v.cmean, v.cnorm, \
                           v.nlist, csplits, tiles_per_split, nq, keys, alpha);                   \
        break
    switch (v.d) {
        GEMM_CASE(32);
        GEMM_CASE(64);
        GEMM_CASE(96);
        GEMM_CASE(128);
        GEMM_CASE(256);
    default: {
        // any other multiple of 8: chunked kernel, four list tiles per workgroup when that still
        // gives the chip enough workgroups, else one
        const int g4 = (ntiles + 3) / 4;
        if ((int64_t)qblocks * g4 >= 512)
            hipLaunchKernelGGL(coarse_gemm_chunk_kernel<4>, dim3(qblocks * g4), dim3(WG), 0, s, q,
                               v.centroids_ct, v.cmean, v.cnorm, v.d, v.nlist, g4, nq, keys, alpha);
        else
            hipLaunchKernelGGL(coarse_gemm_chunk_kernel<1>, dim3(qblocks * ntiles), dim3(WG), 0, s, q,
                               v.centroids_ct, v.cmean, v.cnorm, v.d, v.nlist, ntiles, nq, keys, alpha);
    }
    }
#undef GEMM_CASE
    if (scored) {
        // the score matrix is complete; the selection goes on on the other stream
        RAIRS_HIP(hipEventRecord(scored, s));
        RAIRS_HIP(hipStreamWaitEvent(s_select, scored, 0));
        s = s_select;
    }
    // LDS room per query: the lists inside the margin (half more than nprobe, at least 64), or,
    // when the sample route is used, the keys up to the sample's estimate (about 2-4 x nprobe)
    const int extra = nprobe / 2 > 64 ? nprobe / 2 : 64;
    int cap = next_pow2(nprobe + extra);
    if (cap < 64) cap = 64;
    int nsamp = 0, ksamp = 0;
    if (nprobe <= 496 && v.nlist >= 4 * SHORTLIST_SAMPLE / 2 && 8 * nprobe <= v.nlist) {
        nsamp = SHORTLIST_SAMPLE;
        // the sample's expected share of the nprobe best, plus three standard deviations and a bit
        const double share = (double)nprobe * nsamp / v.nlist;
        ksamp = (int)(share + 3.0 * sqrt(share) + 4.0);
        if (ksamp > nsamp) ksamp = nsamp;
        const int cap2 = next_pow2(4 * nprobe + 64);
        if (cap2 > cap) cap = cap2;
    }
    const size_t sel_bytes = (size_t)cap * 8 * (WG / 64);
#define SHORTLIST_LAUNCH(IP_)                                                                     \
    do {                                                                                          \
        if (sel_bytes > 32 * 1024)                                                                \
            RAIRS_HIP(hipFuncSetAttribute((const void *)coarse_shortlist_kernel<IP_>,              \
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)sel_bytes)); \
        hipLaunchKernelGGL(coarse_shortlist_kernel<IP_>, dim3((unsigned)((nq + WG / 64 - 1) / (WG / 64))), \
                           dim3(WG), sel_bytes, s, keys, q, v.centroids, v.d, v.nlist, nprobe, cap, nsamp, \
                           ksamp, v.cmean, v.cmax2, nq, probe_ids, probe_dists, flags);           \
    } while (0)
    if (v.metric) SHORTLIST_LAUNCH(true);
    else SHORTLIST_LAUNCH(false);
#undef SHORTLIST_LAUNCH
    // queries whose shortlist did not fit (many lists at nearly the same distance): full route,
    // both steps by the query's own workgroup
    hipLaunchKernelGGL(coarse_select_kernel, dim3((unsigned)nq), dim3(WG), 0, s, (uint32_t *)dmat, v.nlist, nprobe,
                       probe_ids, probe_dists, flags, q, v.centroids_t, v.d, v.metric);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

// probe set of each query as a bitmap over list ids (listVisited of Alg. 5, made order-free)
__global__ __launch_bounds__(WG) void bitmap_kernel(const int32_t *__restrict__ probe_ids,
                                                    int nprobe, int nlist, int bmwords,
                                                    uint32_t *__restrict__ bitmap,
                                                    uint32_t *__restrict__ hist)
{
    uint32_t *bm = bitmap + (size_t)blockIdx.x * bmwords;
    for (int i = threadIdx.x; i < bmwords; i += WG) bm[i] = 0;
    // the query's survivor histogram starts empty as well
    if (hist && threadIdx.x < RAIRS_HIST_BINS) hist[(size_t)blockIdx.x * RAIRS_HIST_BINS + threadIdx.x] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < nprobe; i += WG) {
        int32_t l = probe_ids[(size_t)blockIdx.x * nprobe + i];
        if (l >= 0 && l < nlist) atomicOr(&bm[l >> 5], 1u << (l & 31));
    }
}

int rairs_launch_bitmap(const IndexView &v, const int32_t *probe_ids, int64_t nq, int nprobe,
                        uint32_t *bitmap, int bmwords, uint32_t *hist, hipStream_t s)
{
    hipLaunchKernelGGL(bitmap_kernel, dim3((unsigned)nq), dim3(WG), 0, s, probe_ids, nprobe,
                       v.nlist, bmwords, bitmap, hist);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

// ---------------------------------------------------------------------------------------------
// lookup tables: ComputeLookupTable (Alg. 2) + 8-bit quantisation
// ---------------------------------------------------------------------------------------------

// A workgroup builds the tables of LUT_QPW queries, one after the other.  A thread owns groups of
// four consecutive codes of one sub-quantizer (group eg = tid + WG r: sub-quantizer eg / 4, codes
// 4 (eg % 4) ..+3), so the 16 entries of a sub-quantizer sit in four neighbouring lanes: its
// offset and width are a minimum and a maximum over those lanes (register moves), the largest
// width a maximum over the wave and then over the waves (one barrier per query), and a group's
// four bytes leave as one store.  The codewords of a thread's groups are the same for every query
// and stay in registers when a sub-vector has at most four dimensions.  The arithmetic per entry
// is unchanged: squared differences (or products) summed in dimension order.
#define LUT_QPW 8
#define LUT_GROUPS_MAX (RAIRS_MAX_M * 4 / WG)           // groups per thread at the largest M
template <bool IP, int DSUB>                            // DSUB: dimensions of a sub-vector, 0 = any (codewords re-read)
__global__ __launch_bounds__(WG) void lut_kernel(const float *__restrict__ q,
                                                 const float *__restrict__ codebook, int d, int M,
                                                 int64_t nq, uint8_t *__restrict__ lut,
                                                 float *__restrict__ bias_sum,
                                                 float *__restrict__ scale)
{
    __shared__ float wave_span[2][WG / 64];             // alternating by query: one barrier per query
    __shared__ float bias_s[RAIRS_MAX_M];               // only for the stage call's sum of the offsets
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int dsub = DSUB > 0 ? DSUB : d / M;
    const int ngroups = M * 4;
    constexpr int CW = DSUB > 0 ? DSUB : 1;
    float cw[LUT_GROUPS_MAX][4][CW];
    if (DSUB > 0) {
#pragma unroll
        for (int r = 0; r < LUT_GROUPS_MAX; r++) {
            const int eg = tid + WG * r;
#pragma unroll
            for (int k = 0; k < 4; k++)
#pragma unroll
                for (int t = 0; t < CW; t++)
                    cw[r][k][t] = eg < ngroups ? codebook[((size_t)eg * 4 + k) * DSUB + t] : 0.0f;
        }
    }
    const int64_t q0 = (int64_t)blockIdx.x * LUT_QPW;
    for (int qi = 0; qi < LUT_QPW && q0 + qi < nq; qi++) {
        const int64_t qid = q0 + qi;
        const float *qq = q + (size_t)qid * d;
        float T[LUT_GROUPS_MAX][4], lo[LUT_GROUPS_MAX], span = 0.0f;
#pragma unroll
        for (int r = 0; r < LUT_GROUPS_MAX; r++) {
            const int eg = tid + WG * r;
            lo[r] = 0.0f;
            if (eg < ngroups) {                         // (r = 0: every thread when M >= 64)
                const int m = eg >> 2;
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    float acc;
                    if (DSUB > 0) {
                        const float x0 = qq[m * DSUB];
                        const float a = x0 - cw[r][k][0];
                        acc = IP ? x0 * cw[r][k][0] : a * a;
#pragma unroll
                        for (int t = 1; t < CW; t++) {
                            const float xt = qq[m * DSUB + t];
                            const float b = xt - cw[r][k][t];
                            const float sq = IP ? xt * cw[r][k][t] : b * b;
                            acc = acc + sq;
                        }
                    } else {
                        const float *c = codebook + ((size_t)eg * 4 + k) * dsub;
                        const float a = qq[m * dsub] - c[0];
                        acc = IP ? qq[m * dsub] * c[0] : a * a;
                        for (int t = 1; t < dsub; t++) {
                            const float b = qq[m * dsub + t] - c[t];
                            const float sq = IP ? qq[m * dsub + t] * c[t] : b * b;
                            acc = acc + sq;
                        }
                    }
                    T[r][k] = IP ? -acc : acc;          // inner product: minus the product, smaller is better
                }
                float mn = T[r][0], mx = T[r][0];
#pragma unroll
                for (int k = 1; k < 4; k++) {
                    mn = T[r][k] < mn ? T[r][k] : mn;
                    mx = T[r][k] > mx ? T[r][k] : mx;
                }
                // over the four lanes of the sub-quantizer (a minimum and a maximum: order-free)
                float o = lane_xor1(mn); mn = o < mn ? o : mn;
                o = lane_xor2(mn); mn = o < mn ? o : mn;
                o = lane_xor1(mx); mx = o > mx ? o : mx;
                o = lane_xor2(mx); mx = o > mx ? o : mx;
                lo[r] = mn;
                const float width = mx - mn;
                span = width > span ? width : span;
                if (bias_sum && (tid & 3) == 0) bias_s[m] = mn;
            }
        }
        // the largest width over the workgroup
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float o = __shfl_xor(span, off);
            span = o > span ? o : span;
        }
        float *ws = wave_span[qi & 1];
        if (lane == 0) ws[wave] = span;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < WG / 64; w++) span = ws[w] > span ? ws[w] : span;
        const float s = span > 0.0f ? __fdiv_rn(255.0f, span) : 0.0f;
        if (tid == 0 && scale) scale[qid] = s;
        if (tid == 64 && bias_sum) {
            // the sum of the offsets is defined in sub-quantizer order; only the stage call asks for it
            float bsum = 0.0f;
            for (int m = 0; m < M; m++) bsum = bsum + bias_s[m];
            bias_sum[qid] = bsum;
        }
#pragma unroll
        for (int r = 0; r < LUT_GROUPS_MAX; r++) {
            const int eg = tid + WG * r;
            if (eg < ngroups) {
                uint32_t packed = 0;
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const float x = T[r][k] - lo[r];
                    const float y = x * s;
                    float rr = rintf(y);
                    rr = rr > 255.0f ? 255.0f : rr;
                    packed |= (uint32_t)rr << (8 * k);
                }
                ((uint32_t *)(lut + (size_t)qid * M * 16))[eg] = packed;
            }
        }
        if (bias_sum) __syncthreads();                  // bias_s is rewritten by the next query
    }
}

int rairs_launch_lut(const IndexView &v, const float *q, int64_t nq, uint8_t *lut, float *bias_sum,
                     float *scale, hipStream_t s)
{
    const dim3 grid((unsigned)((nq + LUT_QPW - 1) / LUT_QPW));
    const int dsub = v.d / v.M;
#define LUT_LAUNCH(IP_, DS_)                                                                      \
    hipLaunchKernelGGL((lut_kernel<IP_, DS_>), grid, dim3(WG), 0, s, q, v.codebook, v.d, v.M, nq, lut, bias_sum, scale)
#define LUT_METRIC(DS_)                                                                           \
    do { if (v.metric) LUT_LAUNCH(true, DS_); else LUT_LAUNCH(false, DS_); } while (0)
    switch (dsub) {
    case 1: LUT_METRIC(1); break;
    case 2: LUT_METRIC(2); break;
    case 4: LUT_METRIC(4); break;
    default: LUT_METRIC(0); break;
    }
#undef LUT_METRIC
#undef LUT_LAUNCH
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

// ---------------------------------------------------------------------------------------------
// PQEncoding (Alg. 1, Section 2.2): codes of a batch of vectors (index construction)
// ---------------------------------------------------------------------------------------------

// code[m] = the nearest of the 16 codewords of sub-quantizer m, the first one on a tie; distances
// in the table build's arithmetic (fp32, sequential over the sub-vector, no fused multiply-add).
// One thread per output byte -- sub-quantizers 2b and 2b+1 of one vector -- and the thread keeps
// the 32 codewords of its byte position b in registers for all its vectors: the grid's stride over
// (vector, byte) pairs is a multiple of M/2, so b never changes.  Adjacent threads read adjacent
// sub-vectors and write adjacent bytes; the kernel streams the vectors once (HBM bound).
template <int DSUB>
__global__ __launch_bounds__(WG) void pq_encode_reg_kernel(const float *__restrict__ cb, int M,
                                                           const float *__restrict__ x, int64_t n,
                                                           uint8_t *__restrict__ codes)
{
    const int hb = M / 2, d = M * DSUB;
    const int64_t gtid = (int64_t)blockIdx.x * WG + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * WG;       // a multiple of hb (the launcher sees to it)
    const int b = (int)(gtid % hb);
    float cw[2][16][DSUB];
#pragma unroll
    for (int h = 0; h < 2; h++)
#pragma unroll
        for (int c = 0; c < 16; c++)
#pragma unroll
            for (int t = 0; t < DSUB; t++) cw[h][c][t] = cb[((size_t)(2 * b + h) * 16 + c) * DSUB + t];
    const int64_t vstep = stride / hb;
#pragma unroll 2
    for (int64_t v = gtid / hb; v < n; v += vstep) {
        float xs[2 * DSUB];
        const float *xv = x + (size_t)v * d + (size_t)b * 2 * DSUB;
#pragma unroll
        for (int t = 0; t < 2 * DSUB; t++) xs[t] = xv[t];
        uint32_t out = 0;
#pragma unroll
        for (int h = 0; h < 2; h++) {
            int best = 0;
            float bestd = 0.0f;
#pragma unroll
            for (int c = 0; c < 16; c++) {
                const float a0 = xs[h * DSUB] - cw[h][c][0];
                float acc = a0 * a0;
#pragma unroll
                for (int t = 1; t < DSUB; t++) {
                    const float a = xs[h * DSUB + t] - cw[h][c][t];
                    const float sq = a * a;
                    acc = acc + sq;
                }
                if (c == 0 || acc < bestd) { best = c; bestd = acc; }
            }
            out |= (uint32_t)best << (4 * h);
        }
        codes[(size_t)v * hb + b] = (uint8_t)out;
    }
}

// Any sub-vector length: the codebook sits in LDS as [half][codeword][dimension][byte position], so
// that the lanes of a wave (adjacent byte positions) read adjacent words.
__global__ __launch_bounds__(WG) void pq_encode_lds_kernel(const float *__restrict__ cb, int d, int M,
                                                           const float *__restrict__ x, int64_t n,
                                                           uint8_t *__restrict__ codes)
{
    extern __shared__ float pq_cb[];                     // 16 d floats
    const int hb = M / 2, dsub = d / M;
    for (int i = threadIdx.x; i < 16 * d; i += WG) {
        const int t = i % dsub, c = (i / dsub) % 16, m = i / (dsub * 16);
        pq_cb[(((m & 1) * 16 + c) * dsub + t) * hb + (m >> 1)] = cb[i];
    }
    __syncthreads();
    const int64_t total = n * hb;
    for (int64_t e = (int64_t)blockIdx.x * WG + threadIdx.x; e < total; e += (int64_t)gridDim.x * WG) {
        const int64_t v = e / hb;
        const int b = (int)(e % hb);
        const float *xv = x + (size_t)v * d + (size_t)b * 2 * dsub;
        uint32_t out = 0;
        for (int h = 0; h < 2; h++) {
            int best = 0;
            float bestd = 0.0f;
            for (int c = 0; c < 16; c++) {
                const float *cwp = pq_cb + (size_t)((h * 16 + c) * dsub) * hb + b;
                const float a0 = xv[h * dsub] - cwp[0];
                float acc = a0 * a0;
                for (int t = 1; t < dsub; t++) {
                    const float a = xv[h * dsub + t] - cwp[(size_t)t * hb];
                    const float sq = a * a;
                    acc = acc + sq;
                }
                if (c == 0 || acc < bestd) { best = c; bestd = acc; }
            }
            out |= (uint32_t)best << (4 * h);
        }
        codes[e] = (uint8_t)out;
    }
}

int rairs_launch_pq_encode(const float *cb, int d, int M, const float *x, int64_t n, uint8_t *codes,
                           hipStream_t s)
{
    const int hb = M / 2, dsub = d / M;
    // threads in the grid: a multiple of lcm(WG, hb), about eight workgroups per compute unit
    int g = hb, r = WG;
    while (r) { const int tmp = g % r; g = r; r = tmp; }             // gcd(hb, WG)
    const int64_t unit = (int64_t)hb / g;                // workgroups per lcm(WG, hb) threads
    int64_t grid = (2048 + unit - 1) / unit * unit;
    const int64_t need = (n * hb + WG - 1) / WG;
    if (need < grid) grid = (need + unit - 1) / unit * unit;
    if (grid < unit) grid = unit;
    switch (dsub) {
    case 1: hipLaunchKernelGGL(pq_encode_reg_kernel<1>, dim3((unsigned)grid), dim3(WG), 0, s, cb, M, x, n, codes); break;
    case 2: hipLaunchKernelGGL(pq_encode_reg_kernel<2>, dim3((unsigned)grid), dim3(WG), 0, s, cb, M, x, n, codes); break;
    case 4: hipLaunchKernelGGL(pq_encode_reg_kernel<4>, dim3((unsigned)grid), dim3(WG), 0, s, cb, M, x, n, codes); break;
    default: {
        const size_t lds = (size_t)16 * d * sizeof(float);
        if (lds > 48 * 1024)
            RAIRS_HIP(hipFuncSetAttribute((const void *)pq_encode_lds_kernel,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(pq_encode_lds_kernel, dim3((unsigned)grid), dim3(WG), lds, s, cb, d, M, x, n, codes);
    }
    }
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

// ---------------------------------------------------------------------------------------------
// RairAssign (Alg. 3): the AIR loss over the nearest lists of a vector (index construction)
// ---------------------------------------------------------------------------------------------

// cand[v][0 .. nc) are the vector's nearest lists from the coarse quantizer.  One thread per
// (vector, candidate): loss = ||r_i||^2 + lambda <r_0, r_i>, r_i = centroid_i - v, in float64 with
// both sums sequential over the dimensions; the first thread of a vector's group then takes the
// first minimum over candidates 1.. (strict) or 0.. and writes the pair ordered by list id.
__global__ __launch_bounds__(WG) void air_assign_kernel(IndexView v, const float *__restrict__ x,
                                                        int64_t n, int nc, int group, double lambda,
                                                        int strict, const int32_t *__restrict__ cand,
                                                        int32_t *__restrict__ out)
{
    __shared__ double loss_s[WG];
    const int tid = threadIdx.x, g = tid / group, i = tid % group;
    const int64_t vec = (int64_t)blockIdx.x * (WG / group) + g;
    const int d = v.d;
    double loss = 0.0;
    if (vec < n && i < nc) {
        const float *xv = x + (size_t)vec * d;
        const float *p0 = v.centroids + (size_t)cand[(size_t)vec * nc] * d;
        const float *pi = v.centroids + (size_t)cand[(size_t)vec * nc + i] * d;
        double l2 = 0.0, ip = 0.0;
        int t = 0;
        if ((d & 3) == 0) {
            // four dimensions per load (rows of d floats, d a multiple of 4, are 16-byte aligned);
            // the sums still run over the dimensions one after the other
            for (; t < d; t += 4) {
                const float4 xa = *(const float4 *)(xv + t), a0 = *(const float4 *)(p0 + t),
                             ai = *(const float4 *)(pi + t);
                const float xs[4] = {xa.x, xa.y, xa.z, xa.w}, c0[4] = {a0.x, a0.y, a0.z, a0.w},
                            ci[4] = {ai.x, ai.y, ai.z, ai.w};
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const double xt = (double)xs[u];
                    const double r0 = (double)c0[u] - xt, r = (double)ci[u] - xt;
                    const double rr = r * r, r0r = r0 * r;
                    l2 = l2 + rr;
                    ip = ip + r0r;
                }
            }
        }
        for (; t < d; t++) {
            const double xt = (double)xv[t];
            const double r0 = (double)p0[t] - xt, r = (double)pi[t] - xt;
            const double rr = r * r, r0r = r0 * r;
            l2 = l2 + rr;
            ip = ip + r0r;
        }
        const double scaled = lambda * ip;
        loss = l2 + scaled;
    }
    loss_s[tid] = loss;
    __syncthreads();
    if (vec < n && i == 0) {
        const int32_t first = cand[(size_t)vec * nc];
        int best = -1;
        double bestloss = 0.0;
        for (int j = strict ? 1 : 0; j < nc; j++) {
            const double lj = loss_s[g * group + j];
            if (best < 0 || lj < bestloss) { best = j; bestloss = lj; }
        }
        const int32_t second = best < 0 ? first : cand[(size_t)vec * nc + best];
        out[2 * vec] = first < second ? first : second;
        out[2 * vec + 1] = first < second ? second : first;
    }
}

int rairs_launch_air_assign(const IndexView &v, const float *x, int64_t n, int nc, double lambda,
                            int strict, const int32_t *cand, int32_t *out, hipStream_t s)
{
    const int group = next_pow2(nc);                     // <= 32: several vectors per workgroup
    const int per_wg = WG / group;
    hipLaunchKernelGGL(air_assign_kernel, dim3((unsigned)((n + per_wg - 1) / per_wg)), dim3(WG), 0, s, v, x,
                       n, nc, group, lambda, strict, cand, out);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

// ---------------------------------------------------------------------------------------------
// Refine (Alg. 2, the refine step): exact distances of the candidates, K smallest by (distance, id)
// ---------------------------------------------------------------------------------------------

#define REFINE_TAKE_MAX_K 16                // up to here the k results are taken one by one, else a full sort
// One wave per query, no workgroup barrier: the wave takes the query's candidates four at a time,
// one per group of 16 lanes, keeps their keys in its own LDS region and selects there.  The sum
// is the defined one -- 64 interleaved partial sums p_j over the dimensions i = j (mod 64), i
// increasing, then p_j + p_(j xor 32), xor 16, ... xor 1 -- arranged so that most of it stays in
// a lane: lane l of a group holds p_l, p_(l+16), p_(l+32), p_(l+48), so the strides 32 and 16 of
// the butterfly are sums inside the lane (same operands, so the same bits) and only strides 8 to
// 1 cross lanes, as register moves within the group's row of 16.  (A whole wave per row with the
// four rows folded together took 22 instructions per four candidates for the fold, this takes 9,
// and no selects to route ids and flags to the lane that writes the key.)
// (the metric and the row type are template arguments: as run-time flags they cost a select per
// element -- both the product and the squared difference were computed -- a third of the loop)
// (D: the dimension when it is 64, 96 or 128 -- the query's values then stay in registers and the
// rounds are unrolled with constant offsets -- else 0: any dimension, by loops)
template <bool IP, typename RowT, int D>
__global__ __launch_bounds__(WG) void refine_kernel(IndexView v, const float *__restrict__ q,
                                                    const int64_t *__restrict__ cand_ids, int64_t nq,
                                                    int refine_k, int k,
                                                    int64_t *__restrict__ out_ids,
                                                    float *__restrict__ out_dists)
{
    extern __shared__ __align__(16) uint64_t refine_keys[];      // [WG / 64][n2]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t qi = (int64_t)blockIdx.x * (WG / 64) + wave;
    if (qi >= nq) return;                                // waves are independent of each other
    const float *qq = q + (size_t)qi * v.d;
    const int n2 = next_pow2(refine_k < 2 ? 2 : refine_k);
    uint64_t *keys = refine_keys + (size_t)wave * n2;
    const int grp = lane >> 4, l16 = lane & 15;
    const int64_t *my_ids = cand_ids + (size_t)qi * refine_k;
    // Two candidates per group and step (eight per wave), so that sixteen row loads are in flight
    // together: a wave's steps are a serial chain of memory round trips, and this halves it.  The
    // ids of a step are fetched one step ahead of their rows.
    constexpr int RU = 2;
    const int n_used = refine_k < n2 ? refine_k : n2;    // candidates that exist; the rest of the keys are empty
    for (int e = n_used + lane; e < n2; e += 64) keys[e] = ~0ull;
    static_assert(D % 16 == 0, "a known dimension is a whole number of 16-lane rows");
    constexpr int NQV = D > 0 ? D / 16 : 1;
    float qreg[NQV];                                     // the query's values of this lane's classes
    if (D > 0) {
#pragma unroll
        for (int t = 0; t < NQV; t++) qreg[t] = qq[l16 + 16 * t];
    }
    int64_t id_next[RU];
#pragma unroll
    for (int u = 0; u < RU; u++) id_next[u] = 4 * u + grp < n_used ? my_ids[4 * u + grp] : -1;
    for (int c0 = 0; c0 < n_used; c0 += 4 * RU) {
        int64_t id[RU];
        bool ok[RU];
        float p[RU][4];
        const RowT *row[RU];
#pragma unroll
        for (int u = 0; u < RU; u++) {
            const int c = c0 + 4 * u + grp;              // this group's candidates of the step
            id[u] = id_next[u];
            id_next[u] = c + 4 * RU < n_used ? my_ids[c + 4 * RU] : -1;
            ok[u] = c < n_used && id[u] >= 0 && id[u] < v.ntotal;
            if (!ok[u]) id[u] = 0;                       // row 0 is read and discarded
            p[u][0] = p[u][1] = p[u][2] = p[u][3] = 0.0f;
            row[u] = (const RowT *)v.raw + (size_t)id[u] * v.d;
        }
        int i0 = 0;
        if (D > 0) {
            // every (round, class) pair that exists, in dimension order; which exist is known here
#pragma unroll
            for (int r = 0; r < (D + 63) / 64; r++) {
                float x[RU][4];
#pragma unroll
                for (int cc = 0; cc < 4; cc++)
                    if (64 * r + 16 * cc < D)
#pragma unroll
                        for (int u = 0; u < RU; u++) x[u][cc] = (float)row[u][64 * r + l16 + 16 * cc];
#pragma unroll
                for (int u = 0; u < RU; u++)
#pragma unroll
                    for (int cc = 0; cc < 4; cc++)
                        if (64 * r + 16 * cc < D) {
                            const float qv = qreg[4 * r + cc];
                            float sq;
                            if (IP) sq = qv * x[u][cc];
                            else { const float diff = qv - x[u][cc]; sq = diff * diff; }
                            p[u][cc] = p[u][cc] + sq;
                        }
            }
            i0 = D;
        }
        for (; i0 + 64 <= v.d; i0 += 64) {               // whole rounds of 64 dimensions: no lane checks
            float qv[4], x[RU][4];
#pragma unroll
            for (int cc = 0; cc < 4; cc++) {             // class l16 + 16 cc, dimensions increasing
                qv[cc] = qq[i0 + l16 + 16 * cc];
#pragma unroll
                for (int u = 0; u < RU; u++) x[u][cc] = (float)row[u][i0 + l16 + 16 * cc];
            }
#pragma unroll
            for (int u = 0; u < RU; u++)
#pragma unroll
                for (int cc = 0; cc < 4; cc++) {
                    float sq;
                    if (IP) sq = qv[cc] * x[u][cc];
                    else { const float diff = qv[cc] - x[u][cc]; sq = diff * diff; }
                    p[u][cc] = p[u][cc] + sq;
                }
        }
        if (i0 < v.d) {                                  // the last, partial round
#pragma unroll
            for (int cc = 0; cc < 4; cc++) {
                const int i = i0 + l16 + 16 * cc;
                if (i < v.d) {
                    const float qv = qq[i];
#pragma unroll
                    for (int u = 0; u < RU; u++) {
                        const float x = (float)row[u][i];
                        float sq;
                        if (IP) sq = qv * x;
                        else { const float diff = qv - x; sq = diff * diff; }
                        p[u][cc] = p[u][cc] + sq;
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < RU; u++) {
            const int c = c0 + 4 * u + grp;
            const float a = p[u][0] + p[u][2], b = p[u][1] + p[u][3];    // stride 32: classes j and j + 32
            float t = a + b;                             // stride 16
            t = t + lane_xor8(t);
            t = t + lane_xor4(t);
            t = t + lane_xor2(t);
            t = t + lane_xor1(t);
            const float dist = IP ? -t : t;              // inner product: ordered by minus the product
            // empty: all ones, above every key
            if (l16 == 0 && c < n_used) keys[c] = ok[u] ? (((uint64_t)f32_key(dist) << 32) | (uint32_t)id[u]) : ~0ull;
        }
    }
    wave_lds_sync();
    if (k <= REFINE_TAKE_MAX_K) {
        // few results of many candidates: find them by their rank instead of sorting all
        if (n2 <= 128) {
            uint64_t key;
            int rank, m;
            if (wave_rank_smallest(keys, n2, k, lane, &key, &rank, &m)) {
                if (lane < m && rank < k) {
                    out_ids[(size_t)qi * k + rank] = (int64_t)(uint32_t)key;
                    const float sc = key_f32((uint32_t)(key >> 32));
                    out_dists[(size_t)qi * k + rank] = IP ? -sc : sc;
                }
                for (int r = m + lane; r < k; r += 64) {     // fewer than k candidates exist
                    out_ids[(size_t)qi * k + r] = -1;
                    out_dists[(size_t)qi * k + r] = IP ? -__builtin_inff() : __builtin_inff();
                }
                return;
            }
        }
        const uint64_t key = wave_take_smallest(keys, n2, k, lane);
        if (lane < k) {
            const bool ok = key != ~0ull;
            out_ids[(size_t)qi * k + lane] = ok ? (int64_t)(uint32_t)key : -1;
            const float sc = ok ? key_f32((uint32_t)(key >> 32)) : __builtin_inff();
            out_dists[(size_t)qi * k + lane] = IP ? -sc : sc;
        }
        return;
    }
    wave_bitonic_sort_lds(keys, n2, lane);
    for (int i = lane; i < k; i += 64) {
        const uint64_t key = keys[i];
        const bool ok = key != ~0ull;
        out_ids[(size_t)qi * k + i] = ok ? (int64_t)(uint32_t)key : -1;
        const float sc = ok ? key_f32((uint32_t)(key >> 32)) : __builtin_inff();
        out_dists[(size_t)qi * k + i] = IP ? -sc : sc;       // inner product: the product itself, missing -inf
    }
}

#define REFINE_WAVE_MIN_QUERIES 4096        // batches from this size on: one wave per query
// The same for small batches: one workgroup per query, its four waves share the candidates (wave w
// takes candidates w, w + 4, ...) and the workgroup sorts the keys.  With few queries this keeps
// four times as many waves at work, which is what counts when every wave waits for its row loads.
__global__ __launch_bounds__(WG) void refine_wg_kernel(IndexView v, const float *__restrict__ q,
                                                    const int64_t *__restrict__ cand_ids,
                                                    int refine_k, int k,
                                                    int64_t *__restrict__ out_ids,
                                                    float *__restrict__ out_dists)
{
    __shared__ uint64_t keys[RAIRS_MAX_REFINE_K];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t qi = blockIdx.x;
    const float *qq = q + (size_t)qi * v.d;
    const int n2 = next_pow2(refine_k < 2 ? 2 : refine_k);
    // Candidate wave + 4 m is the wave's m-th; lane l first fetches the id of the (mb + l)-th
    // for 64 of them at once, so that the row loads below do not wait for an id load each time.
    // Four candidates at a time, so that their row loads are in flight together.
    const int per_wave = n2 / (WG / 64);                 // n2 is a power of two >= 2; 0 for n2 = 2
    for (int mb = 0; mb < (per_wave > 0 ? per_wave : 1); mb += 64) {
    int64_t myid = -1;
    {
        const int c = wave + (WG / 64) * (mb + lane);
        if (c < refine_k) myid = cand_ids[(size_t)qi * refine_k + c];
    }
    for (int m0 = mb; m0 < mb + 64 && wave + (WG / 64) * m0 < n2; m0 += 4) {
        const int c0 = wave + (WG / 64) * m0;
        int64_t id[4];
        bool ok[4];
        float p[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int src = m0 - mb + u;                 // < 64: four at a time from a multiple of four
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)myid, src);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)myid >> 32), src);
            id[u] = (int64_t)(((uint64_t)hi << 32) | lo);
        }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            ok[u] = id[u] >= 0 && id[u] < v.ntotal;
            if (!ok[u]) id[u] = 0;                       // row 0 is read and discarded
            p[u] = 0.0f;
        }
        const bool any = ok[0] || ok[1] || ok[2] || ok[3];       // wave-uniform
        if (!any) {
            // nothing to read (also keeps an empty index untouched)
        } else if (v.raw_u8) {
            for (int i = lane; i < v.d; i += 64) {
                const float qv = qq[i];
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const float x = (float)((const uint8_t *)v.raw)[(size_t)id[u] * v.d + i];
                    float diff = qv - x;
                    float sq = v.metric ? qv * x : diff * diff;
                    p[u] = p[u] + sq;
                }
            }
        } else {
            for (int i = lane; i < v.d; i += 64) {
                const float qv = qq[i];
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const float x = ((const float *)v.raw)[(size_t)id[u] * v.d + i];
                    float diff = qv - x;
                    float sq = v.metric ? qv * x : diff * diff;
                    p[u] = p[u] + sq;
                }
            }
        }
        const float folded = fold_four_rows(p[0], p[1], p[2], p[3], lane);     // row lane >> 4
        const float dist = v.metric ? -folded : folded;
        {
            const int u = lane >> 4, c = c0 + u * (WG / 64);
            const bool oku = u == 0 ? ok[0] : (u == 1 ? ok[1] : (u == 2 ? ok[2] : ok[3]));
            const int64_t idu = u == 0 ? id[0] : (u == 1 ? id[1] : (u == 2 ? id[2] : id[3]));
            // empty: distance bits in the NaN region, id = all ones
            if ((lane & 15) == 0 && c < n2)
                keys[c] = oku ? (((uint64_t)f32_key(dist) << 32) | (uint32_t)idu) : ~0ull;
        }
    }
    }
    __syncthreads();
    bitonic_sort_lds(keys, n2);
    for (int i = tid; i < k; i += WG) {
        uint64_t key = keys[i];
        bool ok = key != ~0ull;
        out_ids[(size_t)qi * k + i] = ok ? (int64_t)(uint32_t)key : -1;
        const float sc = ok ? key_f32((uint32_t)(key >> 32)) : __builtin_inff();
        out_dists[(size_t)qi * k + i] = v.metric ? -sc : sc;
    }
}

int rairs_launch_refine(const IndexView &v, const float *q, const int64_t *cand_ids, int64_t nq,
                        int refine_k, int k, int64_t *out_ids, float *out_dists, hipStream_t s)
{
    const int n2 = next_pow2(refine_k < 2 ? 2 : refine_k);
    if (nq >= REFINE_WAVE_MIN_QUERIES)
    {
        const dim3 grid((unsigned)((nq + WG / 64 - 1) / (WG / 64)));
        const size_t lds = (size_t)(WG / 64) * n2 * 8;
#define REFINE_LAUNCH(IP_, ROW_, D_)                                                              \
    hipLaunchKernelGGL((refine_kernel<IP_, ROW_, D_>), grid, dim3(WG), lds, s, v, q, cand_ids, nq, refine_k, k, \
                       out_ids, out_dists)
#define REFINE_DIM(IP_, ROW_)                                                                     \
    do {                                                                                          \
        if (v.d == 128) REFINE_LAUNCH(IP_, ROW_, 128);                                            \
        else if (v.d == 96) REFINE_LAUNCH(IP_, ROW_, 96);                                         \
        else if (v.d == 64) REFINE_LAUNCH(IP_, ROW_, 64);                                         \
        else REFINE_LAUNCH(IP_, ROW_, 0);                                                         \
    } while (0)
        if (v.metric) { if (v.raw_u8) REFINE_DIM(true, uint8_t); else REFINE_DIM(true, float); }
        else          { if (v.raw_u8) REFINE_DIM(false, uint8_t); else REFINE_DIM(false, float); }
#undef REFINE_DIM
#undef REFINE_LAUNCH
    }
    else
        hipLaunchKernelGGL(refine_wg_kernel, dim3((unsigned)nq), dim3(WG), 0, s, v, q, cand_ids, refine_k,
                           k, out_ids, out_dists);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}
