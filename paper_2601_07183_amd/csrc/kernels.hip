// HIP kernels (gfx950, wave64) of the RAIRS query path: coarse quantizer, lookup tables,
// exact SEIL scan with a bounded top-bigK queue, refinement.  Built with -ffp-contract=off:
// the fp32 operation order below is part of the result's definition.
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
// coarse quantizer: FindNearestLists for the batch (Alg. 2 line 5)
// ---------------------------------------------------------------------------------------------

// One lane per (query, centroid).  The squared distance is summed as 64 interleaved partial
// sums over the dimensions (class = dimension mod 64), folded pairwise at strides 32..1.
__global__ __launch_bounds__(WG) void coarse_dist_kernel(const float *__restrict__ q,
                                                         const float *__restrict__ ct, int d,
                                                         int nlist, int groups,
                                                         float *__restrict__ dmat)
{
    int qi = blockIdx.x / groups;
    int l = (blockIdx.x % groups) * WG + threadIdx.x;
    const float *qq = q + (size_t)qi * d;
    int lc = l < nlist ? l : nlist - 1;
    float p[64];
#pragma unroll
    for (int j = 0; j < 64; j++) p[j] = 0.0f;
    for (int i0 = 0; i0 < d; i0 += 64) {
#pragma unroll
        for (int j = 0; j < 64; j++) {
            int i = i0 + j;
            if (i < d) {
                float diff = qq[i] - ct[(size_t)i * nlist + lc];
                float sq = diff * diff;
                p[j] = p[j] + sq;
            }
        }
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
#pragma unroll
        for (int j = 0; j < s; j++) p[j] = p[j] + p[j + s];
    }
    if (l < nlist) dmat[(size_t)qi * nlist + l] = p[0];
}

// Per query: the nprobe smallest (distance, list id) by radix select on the fp32 bit pattern
// (distances are >= +0, so the unsigned order of the bits is the numeric order), then sorted.
__global__ __launch_bounds__(WG) void coarse_select_kernel(const float *__restrict__ dmat,
                                                           int nlist, int nprobe,
                                                           int32_t *__restrict__ probe_ids,
                                                           float *__restrict__ probe_dists)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_prefix, s_remaining, s_cnt;
    __shared__ int wcnt[WG / 64];
    __shared__ uint64_t sel[RAIRS_MAX_NPROBE];
    const int tid = threadIdx.x;
    const uint32_t *row = (const uint32_t *)(dmat + (size_t)blockIdx.x * nlist);

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
    // prefix is now the bit pattern of the nprobe-th smallest distance; `remaining` of the keys
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
        if (probe_dists) probe_dists[(size_t)blockIdx.x * nprobe + i] = __uint_as_float((uint32_t)(key >> 32));
    }
}

// Same distances with the lane's centroid held in registers and a block of queries streamed past
// it: the centroid matrix is then read once per 32 queries instead of once per query.
#define COARSE_QB 32
template <int D>
__global__ __launch_bounds__(WG) void coarse_dist_reg_kernel(const float *__restrict__ q,
                                                             const float *__restrict__ ct,
                                                             int nlist, int groups, int64_t nq,
                                                             float *__restrict__ dmat)
{
    constexpr int NP = D < 64 ? D : 64;      // partial-sum classes in use
    const int64_t q0 = (int64_t)(blockIdx.x / groups) * COARSE_QB;
    const int l = (blockIdx.x % groups) * WG + threadIdx.x;
    const int lc = l < nlist ? l : nlist - 1;
    float c[D];
#pragma unroll
    for (int i = 0; i < D; i++) c[i] = ct[(size_t)i * nlist + lc];
    const int64_t q1 = q0 + COARSE_QB < nq ? q0 + COARSE_QB : nq;
    for (int64_t qi = q0; qi < q1; qi++) {
        const float *qq = q + (size_t)qi * D;
        float p[NP];
#pragma unroll
        for (int j = 0; j < NP; j++) {
            float diff = qq[j] - c[j];
            p[j] = diff * diff;
        }
#pragma unroll
        for (int i = NP; i < D; i++) {
            float diff = qq[i] - c[i];
            float sq = diff * diff;
            p[i & 63] = p[i & 63] + sq;
        }
        // classes NP..63 are +0 and adding +0 changes nothing (all terms are >= +0)
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) {
#pragma unroll
            for (int j = 0; j < s; j++)
                if (j + s < NP) p[j] = p[j] + p[j + s];
        }
        if (l < nlist) dmat[(size_t)qi * nlist + l] = p[0];
    }
}

// One wave per query (four queries per workgroup): same selection as coarse_select_kernel for
// nprobe <= 1024.  All loops have trip counts that depend only on nlist and nprobe, so the
// workgroup barriers are reached uniformly.
#define SELW_MAX_NPROBE 1024
__global__ __launch_bounds__(WG) void coarse_select_wave_kernel(const float *__restrict__ dmat,
                                                                int nlist, int nprobe, int64_t nq,
                                                                int32_t *__restrict__ probe_ids,
                                                                float *__restrict__ probe_dists)
{
    __shared__ uint32_t hist_s[WG / 64][256];
    __shared__ uint64_t sel_s[WG / 64][SELW_MAX_NPROBE];
    __shared__ uint32_t cnt_s[WG / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t qi0 = (int64_t)blockIdx.x * (WG / 64) + wave;
    const int64_t qi = qi0 < nq ? qi0 : nq - 1;          // surplus waves redo the last query
    const uint32_t *row = (const uint32_t *)(dmat + (size_t)qi * nlist);
    uint32_t *hist = hist_s[wave];
    uint64_t *sel = sel_s[wave];

    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)nprobe;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int i = lane; i < 256; i += 64) hist[i] = 0;
        __syncthreads();
        for (int i = lane; i < nlist; i += 64) {
            uint32_t key = row[i];
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
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
        __syncthreads();
    }
    const uint32_t kth = prefix;
    // keys below the nprobe-th distance in any order, then `remaining` keys equal to it, the ones
    // with the smallest list ids (lists are walked in increasing id)
    uint32_t nless = 0, neq = 0;
    for (int i0 = 0; i0 < nlist; i0 += 64) {
        const int i = i0 + lane;
        const uint32_t key = i < nlist ? row[i] : 0xFFFFFFFFu;
        const bool less = i < nlist && key < kth;
        const bool eq = i < nlist && key == kth;
        const unsigned long long ml = __ballot(less), me = __ballot(eq);
        const unsigned long long below = (1ull << lane) - 1ull;
        if (less) sel[nless + __popcll(ml & below)] = ((uint64_t)key << 32) | (uint32_t)i;
        nless += (uint32_t)__popcll(ml);
        if (eq) {
            const uint32_t r = neq + (uint32_t)__popcll(me & below);
            // slots after the (nprobe - remaining) smaller keys
            if (r < remaining) sel[(uint32_t)nprobe - remaining + r] = ((uint64_t)kth << 32) | (uint32_t)i;
        }
        neq += (uint32_t)__popcll(me);
    }
    const int n2 = next_pow2(nprobe < 2 ? 2 : nprobe);
    for (int i = nprobe + lane; i < n2; i += 64) sel[i] = ~0ull;
    __syncthreads();
    // bitonic sort by the wave alone
    for (int k = 2; k <= n2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = lane; i < n2; i += 64) {
                int p = i ^ j;
                if (p > i) {
                    bool up = (i & k) == 0;
                    uint64_t x = sel[i], y = sel[p];
                    if ((x > y) == up) { sel[i] = y; sel[p] = x; }
                }
            }
            __syncthreads();
        }
    if (qi0 < nq)
        for (int i = lane; i < nprobe; i += 64) {
            uint64_t key = sel[i];
            probe_ids[(size_t)qi * nprobe + i] = (int32_t)(uint32_t)key;
            if (probe_dists) probe_dists[(size_t)qi * nprobe + i] = __uint_as_float((uint32_t)(key >> 32));
        }
    (void)cnt_s;
}

int rairs_launch_coarse(const IndexView &v, const float *q, int64_t nq, int nprobe, float *dmat,
                        int32_t *probe_ids, float *probe_dists, hipStream_t s)
{
    int groups = (v.nlist + WG - 1) / WG;
    const unsigned qblocks = (unsigned)((nq + COARSE_QB - 1) / COARSE_QB);
    switch (v.d) {
    case 32:
        hipLaunchKernelGGL(coarse_dist_reg_kernel<32>, dim3(qblocks * groups), dim3(WG), 0, s, q,
                           v.centroids_t, v.nlist, groups, nq, dmat);
        break;
    case 96:
        hipLaunchKernelGGL(coarse_dist_reg_kernel<96>, dim3(qblocks * groups), dim3(WG), 0, s, q,
                           v.centroids_t, v.nlist, groups, nq, dmat);
        break;
    case 128:
        hipLaunchKernelGGL(coarse_dist_reg_kernel<128>, dim3(qblocks * groups), dim3(WG), 0, s, q,
                           v.centroids_t, v.nlist, groups, nq, dmat);
        break;
    default:
        hipLaunchKernelGGL(coarse_dist_kernel, dim3((unsigned)(nq * groups)), dim3(WG), 0, s, q,
                           v.centroids_t, v.d, v.nlist, groups, dmat);
    }
    if (nprobe <= SELW_MAX_NPROBE)
        hipLaunchKernelGGL(coarse_select_wave_kernel, dim3((unsigned)((nq + WG / 64 - 1) / (WG / 64))),
                           dim3(WG), 0, s, dmat, v.nlist, nprobe, nq, probe_ids, probe_dists);
    else
        hipLaunchKernelGGL(coarse_select_kernel, dim3((unsigned)nq), dim3(WG), 0, s, dmat, v.nlist,
                           nprobe, probe_ids, probe_dists);
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
// lookup tables: ComputeLookupTable (Alg. 2 line 4) + 8-bit quantisation
// ---------------------------------------------------------------------------------------------

__global__ __launch_bounds__(WG) void lut_kernel(const float *__restrict__ q,
                                                 const float *__restrict__ codebook, int d, int M,
                                                 uint8_t *__restrict__ lut,
                                                 float *__restrict__ bias_sum,
                                                 float *__restrict__ scale)
{
    __shared__ float Ts[RAIRS_MAX_M * 16];
    __shared__ float bias[RAIRS_MAX_M];
    __shared__ float width[RAIRS_MAX_M];
    __shared__ float s_scale;
    const int tid = threadIdx.x;
    const int dsub = d / M;
    const float *qq = q + (size_t)blockIdx.x * d;
    for (int e = tid; e < M * 16; e += WG) {
        int m = e >> 4;
        const float *cw = codebook + (size_t)e * dsub;
        float a = qq[m * dsub] - cw[0];
        float acc = a * a;
        for (int t = 1; t < dsub; t++) {
            float b = qq[m * dsub + t] - cw[t];
            float sq = b * b;
            acc = acc + sq;
        }
        Ts[e] = acc;
    }
    __syncthreads();
    for (int m = tid; m < M; m += WG) {
        float lo = Ts[m * 16], hi = lo;
        for (int c = 1; c < 16; c++) {
            float x = Ts[m * 16 + c];
            lo = x < lo ? x : lo;
            hi = x > hi ? x : hi;
        }
        bias[m] = lo;
        width[m] = hi - lo;
    }
    __syncthreads();
    if (tid == 0) {
        float span = 0.0f, bsum = 0.0f;
        for (int m = 0; m < M; m++) {
            span = width[m] > span ? width[m] : span;
            bsum = bsum + bias[m];
        }
        float s = span > 0.0f ? __fdiv_rn(255.0f, span) : 0.0f;
        s_scale = s;
        if (bias_sum) bias_sum[blockIdx.x] = bsum;
        if (scale) scale[blockIdx.x] = s;
    }
    __syncthreads();
    const float s = s_scale;
    for (int e = tid; e < M * 16; e += WG) {
        float x = Ts[e] - bias[e >> 4];
        float y = x * s;
        float r = rintf(y);
        r = r > 255.0f ? 255.0f : r;
        lut[(size_t)blockIdx.x * M * 16 + e] = (uint8_t)r;
    }
}

int rairs_launch_lut(const IndexView &v, const float *q, int64_t nq, uint8_t *lut, float *bias_sum,
                     float *scale, hipStream_t s)
{
    hipLaunchKernelGGL(lut_kernel, dim3((unsigned)nq), dim3(WG), 0, s, q, v.codebook, v.d, v.M,
                       lut, bias_sum, scale);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}

// ---------------------------------------------------------------------------------------------
// Refine (Alg. 2 line 7): exact distances of the candidates, K smallest by (distance, id)
// ---------------------------------------------------------------------------------------------

// One wave per candidate row: lane j sums the dimensions i = j (mod 64) in increasing order,
// then the 64 partial sums are folded across lanes at strides 32..1.
__global__ __launch_bounds__(WG) void refine_kernel(IndexView v, const float *__restrict__ q,
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
    for (int c = wave; c < n2; c += WG / 64) {
        int64_t id = c < refine_k ? cand_ids[(size_t)qi * refine_k + c] : -1;
        uint64_t key = ~0ull;               // distance bits of NaN/inf region, id = empty
        if (id >= 0 && id < v.ntotal) {
            float p = 0.0f;
            if (v.raw_u8) {
                const uint8_t *row = (const uint8_t *)v.raw + (size_t)id * v.d;
                for (int i = lane; i < v.d; i += 64) {
                    float diff = qq[i] - (float)row[i];
                    float sq = diff * diff;
                    p = p + sq;
                }
            } else {
                const float *row = (const float *)v.raw + (size_t)id * v.d;
                for (int i = lane; i < v.d; i += 64) {
                    float diff = qq[i] - row[i];
                    float sq = diff * diff;
                    p = p + sq;
                }
            }
#pragma unroll
            for (int s = 32; s >= 1; s >>= 1) p = p + __shfl_xor(p, s);
            key = ((uint64_t)__float_as_uint(p) << 32) | (uint32_t)id;
        }
        if (lane == 0) keys[c] = key;
    }
    __syncthreads();
    bitonic_sort_lds(keys, n2);
    for (int i = tid; i < k; i += WG) {
        uint64_t key = keys[i];
        bool ok = key != ~0ull;
        out_ids[(size_t)qi * k + i] = ok ? (int64_t)(uint32_t)key : -1;
        out_dists[(size_t)qi * k + i] = ok ? __uint_as_float((uint32_t)(key >> 32)) : __builtin_inff();
    }
}

int rairs_launch_refine(const IndexView &v, const float *q, const int64_t *cand_ids, int64_t nq,
                        int refine_k, int k, int64_t *out_ids, float *out_dists, hipStream_t s)
{
    hipLaunchKernelGGL(refine_kernel, dim3((unsigned)nq), dim3(WG), 0, s, v, q, cand_ids, refine_k,
                       k, out_ids, out_dists);
    RAIRS_HIP(hipGetLastError());
    return RAIRS_OK;
}
