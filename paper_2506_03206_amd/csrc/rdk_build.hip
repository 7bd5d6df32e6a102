// Construction of the token-affinity kernel M (section 3 of the paper, Eq. 2), run once at
// preprocessing time:  M_ij = exp(Omega_ij / tau) / sum_k exp(Omega_ik / tau), i kept, j any target id,
// with Omega_ij the cosine similarity of embedding rows.  All affinity arithmetic here is fp64: the
// exponent Omega / tau amplifies rounding by 1 / tau, and speed is secondary for a one-off step.
//
// Sparse (top-k) form: for each pruned id the k most similar kept slots are found by a blocked sweep
// over the kept embeddings; Eq. 2 is then normalised over the retained entries of each row.  Row sums
// are accumulated in 2^-40 fixed point so that the result does not depend on the order of the atomics.
#include "rdk_device.hpp"

namespace rdk {

namespace {

constexpr int kTile = 64;       // ids / slots per tile side
constexpr int kDepth = 32;      // embedding columns per LDS stage
constexpr double kFixScale = 1099511627776.0;  // 2^40

struct BuildWs {
    double *inv_norm;           // [N]
    unsigned long long *zfix;   // [n]   sum of unnormalised neighbour weights, fixed point
    int32_t *pruned_ids;        // [N-n]
    double *nbr_a;              // [(N-n), k]  unnormalised weights exp((Omega-1)/tau)
    int32_t *nbr_s;             // [(N-n), k]
    double *row_sum;            // [n]   dense build
};

BuildWs carve(const rdk_kernel_desc_t &d, void *ws)
{
    BuildWs w;
    char *p = (char *)ws;
    const size_t np = (size_t)(d.N - d.n), k = (size_t)(d.k > 0 ? d.k : 0);
    w.inv_norm = (double *)p; p += align_up((size_t)d.N * 8, 256);
    w.zfix = (unsigned long long *)p; p += align_up((size_t)d.n * 8, 256);
    w.pruned_ids = (int32_t *)p; p += align_up((np + 1) * 4, 256);
    w.nbr_a = (double *)p; p += align_up((np * k + 1) * 8, 256);
    w.nbr_s = (int32_t *)p; p += align_up((np * k + 1) * 4, 256);
    w.row_sum = (double *)p;
    return w;
}

__global__ void slot_of_kernel(const int32_t *kept_ids, int n, int N, int32_t *slot_of)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= N) return;
    int lo = 0, hi = n;   // first slot whose id is >= j
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (kept_ids[mid] < j) lo = mid + 1; else hi = mid;
    }
    slot_of[j] = (lo < n && kept_ids[lo] == j) ? lo : -((j - lo) + 1);
}

__global__ void check_kept_kernel(const int32_t *kept_ids, int n, int N, int32_t *flag)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n) return;
    const int v = kept_ids[s];
    if (v < 0 || v >= N || (s > 0 && kept_ids[s - 1] >= v)) atomicOr(flag, 1);
}

__global__ void fill_zero_kernel(unsigned long long *x, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) x[i] = 0ull;
}

__global__ void fill_flag_kernel(int32_t *x) { *x = 0; }

__global__ void inv_norm_kernel(const float *E, int N, int d, double *inv_norm)
{
    const int j = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (j >= N) return;
    double s = 0.0;
    for (int c = lane_id(); c < d; c += kWave) {
        const double v = (double)E[(int64_t)j * d + c];
        s += v * v;
    }
    s = wave_sum(s);
    if (lane_id() == 0) inv_norm[j] = 1.0 / sqrt(s);
}

// Token features from T sampled score rows (Sec. 3: Omega estimated from data):  F[j, t] = z[t, j] - mean_t z[., j].
// One workgroup owns 64 tokens: column means in fp64 (thread x of each quarter reads z[t, j0 + x], coalesced over x),
// then 64 x 64 tiles are turned through LDS so that both the reads of z and the writes of F are coalesced.
template <int KIND>
__global__ __launch_bounds__(256) void features_from_scores_kernel(const void *z, int64_t ldz, int T, int N, float *F, int64_t ldf)
{
    __shared__ double part[4][64];
    __shared__ float mean[64];
    __shared__ float tile[64][65];
    const int x = threadIdx.x % 64, y = threadIdx.x / 64;
    const int j0 = blockIdx.x * 64;
    const bool col_ok = j0 + x < N;
    double acc = 0.0;
    if (col_ok)
        for (int t = y; t < T; t += 4) acc += (double)load1<KIND>(row_ptr<KIND>(z, ldz, t), j0 + x);
    part[y][x] = acc;
    __syncthreads();
    if (y == 0) mean[x] = (float)(((part[0][x] + part[1][x]) + (part[2][x] + part[3][x])) / (double)T);
    __syncthreads();
    for (int t0 = 0; t0 < T; t0 += 64) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {   // rows t0 + y + 4 r of z, columns j0 + x
            const int t = t0 + y + 4 * r;
            tile[y + 4 * r][x] = (col_ok && t < T) ? load1<KIND>(row_ptr<KIND>(z, ldz, t), j0 + x) - mean[x] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 16; ++r) {   // rows j0 + y + 4 r of F, columns t0 + x
            const int j = j0 + y + 4 * r;
            if (j < N && t0 + x < T) F[(int64_t)j * ldf + t0 + x] = tile[x][y + 4 * r];
        }
        __syncthreads();
    }
}

// chunk_lo[c] = number of kept ids below c * kChunk (kept ids ascend, so the ids of chunk c hold the slots
// chunk_lo[c] .. chunk_lo[c + 1] - 1, a contiguous piece of every drafter row).
__global__ void chunk_lo_kernel(const int32_t *kept_ids, int n, int nchunks, int32_t *chunk_lo)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c > nchunks) return;
    const int64_t first = (int64_t)c * kChunk;
    int lo = 0, hi = n;   // lower bound of `first` in kept_ids
    while (lo < hi) {
        const int mid = (lo + hi) / 2;
        if (kept_ids[mid] < first) lo = mid + 1;
        else hi = mid;
    }
    chunk_lo[c] = lo;
}

__global__ void pruned_ids_kernel(const int32_t *slot_of, int N, int n, int32_t *pruned_ids)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= N || slot_of[j] >= 0) return;
    const int u = -slot_of[j] - 1;
    if (u < N - n) pruned_ids[u] = j;   // always true for ascending kept ids; an unchecked list must not write past the table
}

// The kept slots in pieces of at most 64 that stay inside one chunk (a chunk with m kept ids gives ceil(m / 64) pieces):
// one workgroup counts the pieces of 1024 chunks at a time, numbers them with a prefix sum and writes them out.
__global__ __launch_bounds__(1024) void row_items_kernel(const int32_t *chunk_lo, int nchunks, int32_t *item_lo, int2 *row_items)
{
    __shared__ int wave_total[1024 / kWave];
    __shared__ int carry;
    const int lane = lane_id(), wid = threadIdx.x / kWave;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < nchunks; base += 1024) {
        const int c = base + threadIdx.x;
        int lo = 0, hi = 0;
        if (c < nchunks) {
            lo = chunk_lo[c];
            hi = chunk_lo[c + 1];
        }
        const int cnt = (hi - lo + 63) / 64;
        int incl = cnt;
        for (int off = 1; off < kWave; off <<= 1) {
            const int o = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += o;
        }
        if (lane == kWave - 1) wave_total[wid] = incl;
        __syncthreads();
        int before = carry;
        for (int w = 0; w < wid; ++w) before += wave_total[w];
        const int first = before + incl - cnt;
        if (c < nchunks) {
            item_lo[c] = first;
            for (int k = 0; k < cnt; ++k)
                row_items[first + k] = make_int2(lo + 64 * k, c | ((lo & 3) << 22) | (min(64, hi - lo - 64 * k) << 24));
        }
        __syncthreads();
        if (threadIdx.x == 1023) carry = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) item_lo[nchunks] = carry;
}

// Per chunk and lane the kept mask of the lane's 16 ids and the kept ids of the chunk below each of its four groups.
__global__ void lane_map_kernel(const int32_t *slot_of, const int32_t *chunk_lo, int N, int n, uint64_t *lane_map)
{
    const int c = blockIdx.x, l = threadIdx.x;
    const int lo = chunk_lo[c];
    uint64_t rec = 0;
    for (int i = 0; i < 4; ++i) {
        const int j0 = c * kChunk + 256 * i + 4 * l;
        int below = n;                                     // kept ids below j0 in the whole vocabulary
        if (j0 < N) {
            const int s = slot_of[j0];
            below = s >= 0 ? s : j0 - (-s - 1);
        }
        rec |= (uint64_t)(below - lo) << (16 + 12 * i);
        for (int e = 0; e < 4; ++e)
            if (j0 + e < N && slot_of[j0 + e] >= 0) rec |= (uint64_t)1 << (4 * i + e);
    }
    lane_map[(int64_t)c * kWave + l] = rec;
}

// Cosine similarities of a 64 x 64 tile: rows = ids `row_ids[r0..]`, columns = ids `col_ids[c0..]`
// (NULL id list = the identity).  256 threads, each a 4 x 4 micro-tile in fp64; the result is left in
// om[64][65].  Entries outside the ranges are -2 (below any cosine).
__device__ __forceinline__ void affinity_tile(const float *E, int d, const double *inv_norm, const int32_t *row_ids, int r0,
                                              int n_rows, const int32_t *col_ids, int c0, int n_cols,
                                              float (*ea)[kDepth + 1], float (*eb)[kDepth + 1], double (*om)[kTile + 1])
{
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    double acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
    for (int dc = 0; dc < d; dc += kDepth) {
        __syncthreads();
        for (int t = threadIdx.x; t < kTile * kDepth; t += blockDim.x) {
            const int r = t / kDepth, c = t % kDepth;
            float va = 0.f, vb = 0.f;
            if (dc + c < d) {
                if (r0 + r < n_rows) va = E[(int64_t)(row_ids ? row_ids[r0 + r] : r0 + r) * d + dc + c];
                if (c0 + r < n_cols) vb = E[(int64_t)(col_ids ? col_ids[c0 + r] : c0 + r) * d + dc + c];
            }
            ea[r][c] = va;
            eb[r][c] = vb;
        }
        __syncthreads();
#pragma unroll 4
        for (int c = 0; c < kDepth; ++c) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = (double)ea[ty * 4 + i][c];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = (double)eb[tx * 4 + j][c];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = ty * 4 + i;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = tx * 4 + j;
            double v = -2.0;
            if (r0 + r < n_rows && c0 + c < n_cols) {
                const int ir = row_ids ? row_ids[r0 + r] : r0 + r;
                const int ic = col_ids ? col_ids[c0 + c] : c0 + c;
                v = acc[i][j] * inv_norm[ir] * inv_norm[ic];
            }
            om[r][c] = v;
        }
    }
    __syncthreads();
}

// Top-k kept slots per pruned id.  One workgroup owns 64 pruned ids and sweeps all kept slots in tiles
// of 64; after each tile one thread per id merges the 64 new affinities into its sorted list (falling
// affinity, ties by rising slot: a later slot never displaces an equal earlier one).
__global__ __launch_bounds__(256) void topk_kernel(const float *E, int d, const double *inv_norm, const int32_t *pruned_ids,
                                                   int n_pruned, const int32_t *kept_ids, int n, int k, double inv_tau,
                                                   double *nbr_a, int32_t *nbr_s, unsigned long long *zfix)
{
    __shared__ float ea[kTile][kDepth + 1], eb[kTile][kDepth + 1];
    __shared__ double om[kTile][kTile + 1];
    extern __shared__ unsigned char dyn[];
    double *best_v = (double *)dyn;                        // [64][k]
    int32_t *best_s = (int32_t *)(best_v + kTile * k);     // [64][k]
    const int r0 = blockIdx.x * kTile;
    int filled = 0;
    for (int c0 = 0; c0 < n; c0 += kTile) {
        affinity_tile(E, d, inv_norm, pruned_ids, r0, n_pruned, kept_ids, c0, n, ea, eb, om);
        if (threadIdx.x < kTile && r0 + threadIdx.x < n_pruned) {
            double *bv = best_v + threadIdx.x * k;
            int32_t *bs = best_s + threadIdx.x * k;
            const int lim = min(kTile, n - c0);
            for (int c = 0; c < lim; ++c) {
                const double v = om[threadIdx.x][c];
                if (filled < k || v > bv[k - 1]) {
                    int pos = filled < k ? filled : k - 1;
                    while (pos > 0 && bv[pos - 1] < v) {
                        bv[pos] = bv[pos - 1];
                        bs[pos] = bs[pos - 1];
                        --pos;
                    }
                    bv[pos] = v;
                    bs[pos] = c0 + c;
                    if (filled < k) ++filled;
                }
            }
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < kTile * k; t += blockDim.x) {
        const int r = t / k, e = t % k;
        if (r0 + r >= n_pruned) continue;
        const double a = exp((best_v[r * k + e] - 1.0) * inv_tau);
        const int s = best_s[r * k + e];
        nbr_a[(int64_t)(r0 + r) * k + e] = a;
        nbr_s[(int64_t)(r0 + r) * k + e] = s;
        atomicAdd(&zfix[s], (unsigned long long)(a * kFixScale + 0.5));
    }
}

// Normalise over the retained entries (Eq. 2 on the retained set).  Stored layout: per pruned slot u a
// row of kk (kept slot, weight) pairs (the k real ones, then padding with slot 0 and weight 0), and
// per kept slot its diagonal weight.
__global__ void sparse_finish_kernel(int n_pruned, int n, int k, int kk, const double *nbr_a, const int32_t *nbr_s,
                                     const unsigned long long *zfix, int2 *nbr, float *self_w)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) self_w[t] = (float)(1.0 / (1.0 + (double)zfix[t] / kFixScale));
    if (t >= (int64_t)n_pruned * kk) return;
    const int64_t u = t / kk;
    const int e = (int)(t % kk);
    int idx = 0;
    float w = 0.f;
    if (e < k) {
        idx = nbr_s[u * k + e];
        w = (float)(nbr_a[u * k + e] / (1.0 + (double)zfix[idx] / kFixScale));
    }
    nbr[t] = make_int2(idx, __float_as_int(w));
}

// Copy between the caller's [.., k] tables and the padded [.., kk] tables of the storage blob.
__global__ void sparse_import_kernel(int n_pruned, int n, int k, int kk, const int32_t *sp_idx, const float *sp_w,
                                     const float *sp_self, int2 *nbr, float *self_w)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) self_w[t] = sp_self[t];
    if (t >= (int64_t)n_pruned * kk) return;
    const int64_t u = t / kk;
    const int e = (int)(t % kk);
    // slots are clamped into [0, n): a table that was not validated cannot send a gather outside the drafter rows
    nbr[t] = make_int2(e < k ? min(max(sp_idx[u * k + e], 0), n - 1) : 0, __float_as_int(e < k ? sp_w[u * k + e] : 0.f));
}

__global__ void sparse_export_kernel(int n_pruned, int n, int k, int kk, const int2 *nbr, const float *self_w,
                                     int32_t *sp_idx, float *sp_w, float *sp_self)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) sp_self[t] = self_w[t];
    if (t >= (int64_t)n_pruned * kk) return;
    const int64_t u = t / kk;
    const int e = (int)(t % kk);
    if (e < k) {
        sp_idx[u * k + e] = nbr[t].x;
        sp_w[u * k + e] = __int_as_float(nbr[t].y);
    }
}

// Dense Eq. 2, first pass: one workgroup owns 64 kept slots and sweeps the target ids in tiles of 64,
// storing exp((Omega - 1) / tau) and summing each row in a fixed order.
__global__ __launch_bounds__(256) void dense_rows_kernel(const float *E, int d, const double *inv_norm, const int32_t *kept_ids,
                                                         int n, int N, double inv_tau, float *M, int64_t ldm, double *row_sum)
{
    __shared__ float ea[kTile][kDepth + 1], eb[kTile][kDepth + 1];
    __shared__ double om[kTile][kTile + 1];
    __shared__ double part[kTile][4];
    const int r0 = blockIdx.x * kTile;
    const int r = threadIdx.x / 4, cq = threadIdx.x % 4;   // 4 threads per row, 16 columns each
    double sum = 0.0;
    for (int c0 = 0; c0 < N; c0 += kTile) {
        affinity_tile(E, d, inv_norm, kept_ids, r0, n, nullptr, c0, N, ea, eb, om);
        if (r0 + r < n) {
            for (int c = cq * 16; c < cq * 16 + 16; ++c) {
                if (c0 + c >= N) break;
                const double a = exp((om[r][c] - 1.0) * inv_tau);
                sum += a;
                M[(int64_t)(r0 + r) * ldm + c0 + c] = (float)a;
            }
        }
    }
    part[r][cq] = sum;
    __syncthreads();
    if (cq == 0 && r0 + r < n) row_sum[r0 + r] = (part[r][0] + part[r][1]) + (part[r][2] + part[r][3]);
}

__global__ void dense_scale_kernel(float *M, int64_t ldm, int n, int N, const double *row_sum)
{
    for (int s = blockIdx.y; s < n; s += gridDim.y) {   // rows beyond the grid's second dimension are looped over
        const double inv = 1.0 / row_sum[s];
        for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < N; j += (int64_t)gridDim.x * blockDim.x)
            M[(int64_t)s * ldm + j] = (float)((double)M[(int64_t)s * ldm + j] * inv);
    }
}

// Row sums and sign check of a supplied dense kernel.
__global__ void check_dense_kernel(const float *M, int64_t ldm, int N, int32_t *flag)
{
    const int s = blockIdx.x;
    double sum = 0.0;
    bool bad = false;
    for (int j = threadIdx.x; j < N; j += blockDim.x) {
        const float v = M[(int64_t)s * ldm + j];
        bad |= !(v >= 0.f);
        sum += (double)v;
    }
    sum = wave_sum(sum);
    __shared__ double sh[4];
    __shared__ int shb;
    if (threadIdx.x == 0) shb = 0;
    __syncthreads();
    if (lane_id() == 0) sh[threadIdx.x / kWave] = sum;
    if (bad) atomicOr(&shb, 1);
    __syncthreads();
    if (threadIdx.x == 0) {
        const double t = (sh[0] + sh[1]) + (sh[2] + sh[3]);
        if (shb || !(fabs(t - 1.0) <= 1e-3)) atomicOr(flag, 1);
    }
}

// Row sums of a sparse kernel: entry (idx, w) of a pruned id adds w to row idx; the diagonal adds self_w.
__global__ void check_sparse_accum_kernel(const int2 *nbr, int64_t count, const float *self_w, int n,
                                          unsigned long long *zfix, int32_t *flag)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) {
        const float sw = self_w[t];
        if (!(sw >= 0.f)) atomicOr(flag, 1);
        else atomicAdd(&zfix[t], (unsigned long long)((double)sw * kFixScale + 0.5));
    }
    if (t >= count) return;
    const float w = __int_as_float(nbr[t].y);
    const int s = nbr[t].x;
    if (!(w >= 0.f) || s < 0 || s >= n) {
        atomicOr(flag, 1);
        return;
    }
    if (w > 0.f) atomicAdd(&zfix[s], (unsigned long long)((double)w * kFixScale + 0.5));
}

__global__ void check_sparse_rows_kernel(const unsigned long long *zfix, int n, int32_t *flag)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s < n && !(fabs((double)zfix[s] / kFixScale - 1.0) <= 1e-3)) atomicOr(flag, 1);
}

}  // namespace

size_t build_workspace_bytes(const rdk_kernel_desc_t &d)
{
    const size_t np = (size_t)(d.N - d.n), k = (size_t)(d.k > 0 ? d.k : 0);
    return align_up((size_t)d.N * 8, 256) + align_up((size_t)d.n * 8, 256) + align_up((np + 1) * 4, 256) +
           align_up((np * k + 1) * 8, 256) + align_up((np * k + 1) * 4, 256) + align_up((size_t)d.n * 8, 256) + 256;
}

rdk_status_t launch_slot_of(const int32_t *kept_ids, int32_t n, int32_t N, int32_t *slot_of, hipStream_t st)
{
    hipLaunchKernelGGL(slot_of_kernel, dim3((N + 255) / 256), dim3(256), 0, st, kept_ids, n, N, slot_of);
    RDK_LAUNCH_CHECK("slot_of_kernel");
    return RDK_OK;
}

rdk_status_t launch_check_kept(const int32_t *kept_ids, int32_t n, int32_t N, int32_t *flag, hipStream_t st)
{
    hipLaunchKernelGGL(fill_flag_kernel, dim3(1), dim3(1), 0, st, flag);
    hipLaunchKernelGGL(check_kept_kernel, dim3((n + 255) / 256), dim3(256), 0, st, kept_ids, n, N, flag);
    RDK_LAUNCH_CHECK("check_kept_kernel");
    return RDK_OK;
}

rdk_status_t launch_features_from_scores(const void *z, rdk_input_kind_t kind, int64_t ldz, int32_t T, int32_t N, float *F,
                                         int64_t ldf, hipStream_t st)
{
    const dim3 grid((N + 63) / 64), block(256);
    switch (kind) {
        case RDK_PROB_F32:
        case RDK_LOGIT_F32:
            hipLaunchKernelGGL((features_from_scores_kernel<RDK_LOGIT_F32>), grid, block, 0, st, z, ldz, T, N, F, ldf);
            break;
        case RDK_LOGIT_BF16:
            hipLaunchKernelGGL((features_from_scores_kernel<RDK_LOGIT_BF16>), grid, block, 0, st, z, ldz, T, N, F, ldf);
            break;
        default: return RDK_ERR_DTYPE;
    }
    RDK_LAUNCH_CHECK("features_from_scores_kernel");
    return RDK_OK;
}

rdk_status_t launch_row_items(const int32_t *chunk_lo, int32_t N, int32_t *item_lo, int2 *row_items, hipStream_t st)
{
    const int nchunks = (N + kChunk - 1) / kChunk;
    hipLaunchKernelGGL(row_items_kernel, dim3(1), dim3(1024), 0, st, chunk_lo, nchunks, item_lo, row_items);
    RDK_LAUNCH_CHECK("row_items_kernel");
    return RDK_OK;
}

rdk_status_t launch_lane_map(const int32_t *slot_of, const int32_t *chunk_lo, int32_t N, int32_t n, uint64_t *lane_map,
                             hipStream_t st)
{
    const int nchunks = (N + kChunk - 1) / kChunk;
    hipLaunchKernelGGL(lane_map_kernel, dim3(nchunks), dim3(kWave), 0, st, slot_of, chunk_lo, N, n, lane_map);
    RDK_LAUNCH_CHECK("lane_map_kernel");
    return RDK_OK;
}

rdk_status_t launch_chunk_lo(const int32_t *kept_ids, int32_t n, int32_t N, int32_t *chunk_lo, hipStream_t st)
{
    const int nchunks = (N + kChunk - 1) / kChunk;
    hipLaunchKernelGGL(chunk_lo_kernel, dim3((nchunks + 256) / 256), dim3(256), 0, st, kept_ids, n, nchunks, chunk_lo);
    RDK_LAUNCH_CHECK("chunk_lo_kernel");
    return RDK_OK;
}

rdk_status_t launch_pruned_ids(const int32_t *slot_of, int32_t N, int32_t n, int32_t *pruned_ids, hipStream_t st)
{
    hipLaunchKernelGGL(pruned_ids_kernel, dim3((N + 255) / 256), dim3(256), 0, st, slot_of, N, n, pruned_ids);
    RDK_LAUNCH_CHECK("pruned_ids_kernel");
    return RDK_OK;
}

static unsigned table_blocks(int n_pruned, int kk, int n)
{
    int64_t count = (int64_t)n_pruned * kk;
    if (count < n) count = n;
    return (unsigned)((count + 255) / 256);
}

rdk_status_t launch_build_sparse(const rdk_kernel_desc_t &d, const int32_t *pruned_ids, int2 *nbr, float *self_w, int32_t kk,
                                 void *ws, hipStream_t st)
{
    BuildWs w = carve(d, ws);
    const int np = d.N - d.n;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((d.n + 255) / 256), dim3(256), 0, st, w.zfix, (int64_t)d.n);
    RDK_LAUNCH_CHECK("fill_zero_kernel");
    if (d.k > 0 && np > 0) {
        hipLaunchKernelGGL(inv_norm_kernel, dim3((d.N + 3) / 4), dim3(256), 0, st, d.embeddings, d.N, d.d, w.inv_norm);
        RDK_LAUNCH_CHECK("inv_norm_kernel");
        const size_t dyn = (size_t)kTile * d.k * (sizeof(double) + sizeof(int32_t));
        RDK_HIP(hipFuncSetAttribute((const void *)topk_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn));
        hipLaunchKernelGGL(topk_kernel, dim3((np + kTile - 1) / kTile), dim3(256), dyn, st, d.embeddings, d.d, w.inv_norm,
                           pruned_ids, np, d.kept_ids, d.n, d.k, 1.0 / (double)d.tau, w.nbr_a, w.nbr_s, w.zfix);
        RDK_LAUNCH_CHECK("topk_kernel");
    }
    hipLaunchKernelGGL(sparse_finish_kernel, dim3(table_blocks(np, kk, d.n)), dim3(256), 0, st, np, d.n, d.k, kk, w.nbr_a,
                       w.nbr_s, w.zfix, nbr, self_w);
    RDK_LAUNCH_CHECK("sparse_finish_kernel");
    return RDK_OK;
}

rdk_status_t launch_import_sparse(const rdk_kernel_desc_t &d, int2 *nbr, float *self_w, int32_t kk, hipStream_t st)
{
    const int np = d.N - d.n;
    hipLaunchKernelGGL(sparse_import_kernel, dim3(table_blocks(np, kk, d.n)), dim3(256), 0, st, np, d.n, d.k, kk,
                       d.sparse_idx, d.sparse_w, d.self_w, nbr, self_w);
    RDK_LAUNCH_CHECK("sparse_import_kernel");
    return RDK_OK;
}

rdk_status_t launch_export_sparse(const KernelHandle &h, int32_t *idx, float *w, float *self_w, hipStream_t st)
{
    const int np = h.N - h.n;
    hipLaunchKernelGGL(sparse_export_kernel, dim3(table_blocks(np, h.kk, h.n)), dim3(256), 0, st, np, h.n, h.k, h.kk,
                       h.nbr, h.self_w, idx, w, self_w);
    RDK_LAUNCH_CHECK("sparse_export_kernel");
    return RDK_OK;
}

rdk_status_t launch_build_dense(const rdk_kernel_desc_t &d, float *M, int64_t ldm, void *ws, hipStream_t st)
{
    BuildWs w = carve(d, ws);
    hipLaunchKernelGGL(inv_norm_kernel, dim3((d.N + 3) / 4), dim3(256), 0, st, d.embeddings, d.N, d.d, w.inv_norm);
    RDK_LAUNCH_CHECK("inv_norm_kernel");
    hipLaunchKernelGGL(dense_rows_kernel, dim3((d.n + kTile - 1) / kTile), dim3(256), 0, st, d.embeddings, d.d, w.inv_norm,
                       d.kept_ids, d.n, d.N, 1.0 / (double)d.tau, M, ldm, w.row_sum);
    RDK_LAUNCH_CHECK("dense_rows_kernel");
    hipLaunchKernelGGL(dense_scale_kernel, dim3(64, d.n < 32768 ? d.n : 32768), dim3(256), 0, st, M, ldm, d.n, d.N, w.row_sum);
    RDK_LAUNCH_CHECK("dense_scale_kernel");
    return RDK_OK;
}

rdk_status_t launch_check_stochastic_dense(const float *M, int64_t ldm, int32_t n, int32_t N, int32_t *flag, hipStream_t st)
{
    hipLaunchKernelGGL(fill_flag_kernel, dim3(1), dim3(1), 0, st, flag);
    hipLaunchKernelGGL(check_dense_kernel, dim3(n), dim3(256), 0, st, M, ldm, N, flag);
    RDK_LAUNCH_CHECK("check_dense_kernel");
    return RDK_OK;
}

rdk_status_t launch_check_stochastic_sparse(const KernelHandle &h, void *ws, int32_t *flag, hipStream_t st)
{
    unsigned long long *zfix = (unsigned long long *)ws;
    const int np = h.N - h.n;
    hipLaunchKernelGGL(fill_flag_kernel, dim3(1), dim3(1), 0, st, flag);
    hipLaunchKernelGGL(fill_zero_kernel, dim3((h.n + 255) / 256), dim3(256), 0, st, zfix, (int64_t)h.n);
    hipLaunchKernelGGL(check_sparse_accum_kernel, dim3(table_blocks(np, h.kk, h.n)), dim3(256), 0, st, h.nbr, (int64_t)np * h.kk,
                       h.self_w, h.n, zfix, flag);
    hipLaunchKernelGGL(check_sparse_rows_kernel, dim3((h.n + 255) / 256), dim3(256), 0, st, zfix, h.n, flag);
    RDK_LAUNCH_CHECK("check_sparse_rows_kernel");
    return RDK_OK;
}

}  // namespace rdk
