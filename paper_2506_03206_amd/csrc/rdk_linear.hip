// Linear-time redistribution (Alg. 1, steps 1-2) in its two forms:
//   * the first-order closed form, Eq. 3 of the paper (no matrix, needs the target row p);
//   * the product M^T q' with the top-k sparse kernel (k gathers per pruned id).
// Step 1 (token-level intersection, Eq. 1) is folded in: the drafter row is only ever used divided
// by its own sum over the kept slots.
#include "rdk_rowstats.hpp"

namespace rdk {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kPosBlock = 16;   // positions per gather in the sparse product: 16 fp32 = one 64-byte segment
constexpr int kIdsPerBlock = 256;

struct LinearWs {
    SoftStat *pstat;   // [B, p_splits]  target row softmax statistics (logit p only)
    SoftStat *qstat;   // [B]            drafter row: (max, sum exp) or (0, sum)
    SoftStat *qpart;   // [B, q_splits]  partials of the above (sparse product)
    float *tpart;      // [B, t_splits, 4]  Taylor partial sums
    float *qT;         // [ceil(B/16), n, 16] drafter weights, position-minor (sparse product)
    int p_splits, t_splits, q_splits;
};

LinearWs carve(const KernelHandle &h, int32_t B, void *ws)
{
    LinearWs w;
    w.p_splits = row_splits(B, h.N, kWaves);
    w.t_splits = w.p_splits;
    w.q_splits = row_splits(B, h.n, kWaves);
    char *p = (char *)ws;
    w.pstat = (SoftStat *)p; p += align_up((size_t)B * w.p_splits * sizeof(SoftStat), 256);
    w.qstat = (SoftStat *)p; p += align_up((size_t)B * sizeof(SoftStat), 256);
    w.qpart = (SoftStat *)p; p += align_up((size_t)B * kMaxSplits * sizeof(SoftStat), 256);
    w.tpart = (float *)p; p += align_up((size_t)B * w.t_splits * 4 * sizeof(float), 256);
    w.qT = (float *)p;
    return w;
}

// ------------------------------------------------------------------------------------------------
// Eq. 3, first pass.  For the ids of one split of a row:
//   Zq += q^_s, Tn += q^_s p_j, An += N q^_s / (N + p_j)   over kept ids j (slot s),
//   Bs += p_j / (N + p_j)                                    over all ids j.
// Then theta = Tn / Zq and sum_j pt_j = An / Zq + theta * Bs, because
//   pt_j = N q'_j / (N + p_j) + theta p_j / (N + p_j)  with q'_j = q^_s / Zq on kept ids, 0 elsewhere.
template <int PK, int QK>
__global__ __launch_bounds__(kThreads) void taylor_stats_kernel(const void *p, int64_t ldp, const void *q, int64_t ldq,
                                                                const int32_t *slot_of, int N, int splits, bool vec_p,
                                                                LinearWs w)
{
    const int64_t row = blockIdx.x / splits;
    const int split = blockIdx.x % splits;
    const int nchunks = (N + kChunk - 1) / kChunk;
    const int cpw = (nchunks + splits - 1) / splits;
    const int c_begin = split * cpw, c_end = min(nchunks, c_begin + cpw);
    const void *pr = row_ptr<PK>(p, ldp, row);
    const void *qr = row_ptr<QK>(q, ldq, row);
    const int wid = threadIdx.x / kWave, lane = lane_id();
    float pm = 0.f, pinv = 1.f;
    if (PK != RDK_PROB_F32) {
        const SoftStat rs = merged_row_stat<PK>(w.pstat, w.p_splits, row);
        pm = rs.m;
        pinv = 1.0f / rs.s;
    }
    const float qm = QK == RDK_PROB_F32 ? 0.f : w.qstat[row].m;
    const float pfill = PK == RDK_PROB_F32 ? 0.f : -INFINITY;
    const float fN = (float)N;
    float zq = 0.f, tn = 0.f, an = 0.f, bs = 0.f;
    for (int c = c_begin + wid; c < c_end; c += kWaves) {
        const int64_t base = (int64_t)c * kChunk + lane * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t idx = base + i * 256;
            const float4 pv = load4<PK>(pr, idx, N, vec_p, pfill);
            const float pe[4] = {to_weight<PK>(pv.x, pm, pinv), to_weight<PK>(pv.y, pm, pinv),
                                 to_weight<PK>(pv.z, pm, pinv), to_weight<PK>(pv.w, pm, pinv)};
            int4 sv = make_int4(-1, -1, -1, -1);
            if (idx + 3 < N) {
                sv = *(const int4 *)(slot_of + idx);
            } else {
                if (idx + 0 < N) sv.x = slot_of[idx + 0];
                if (idx + 1 < N) sv.y = slot_of[idx + 1];
                if (idx + 2 < N) sv.z = slot_of[idx + 2];
            }
            const int se[4] = {sv.x, sv.y, sv.z, sv.w};
            float qraw[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) qraw[e] = load1<QK>(qr, max(se[e], 0));   // unconditional: loads stay batched
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float r = 1.0f / (fN + pe[e]);
                bs += pe[e] * r;
                const float qh = se[e] >= 0 ? to_weight<QK>(qraw[e], qm, 1.f) : 0.f;
                zq += qh;
                tn += qh * pe[e];
                an += fN * qh * r;
            }
        }
    }
    zq = wave_sum(zq);
    tn = wave_sum(tn);
    an = wave_sum(an);
    bs = wave_sum(bs);
    __shared__ float sh[kWaves][4];
    if (lane == 0) {
        sh[wid][0] = zq; sh[wid][1] = tn; sh[wid][2] = an; sh[wid][3] = bs;
    }
    __syncthreads();
    if (threadIdx.x < 4) {
        float s = sh[0][threadIdx.x];
        for (int i = 1; i < kWaves; ++i) s += sh[i][threadIdx.x];
        w.tpart[(row * splits + split) * 4 + threadIdx.x] = s;
    }
}

// Eq. 3, second pass: out_j = ((N q'_j + theta p_j) / (N + p_j)) / sum_j pt_j.
template <int PK, int QK>
__global__ __launch_bounds__(kThreads) void taylor_write_kernel(const void *p, int64_t ldp, const void *q, int64_t ldq,
                                                                const int32_t *slot_of, int N, int splits, bool vec_p,
                                                                bool vec_o, LinearWs w, float *out, int64_t ldo)
{
    const int64_t row = blockIdx.x / splits;
    const int split = blockIdx.x % splits;
    const int nchunks = (N + kChunk - 1) / kChunk;
    const int cpw = (nchunks + splits - 1) / splits;
    const int c_begin = split * cpw, c_end = min(nchunks, c_begin + cpw);
    const void *pr = row_ptr<PK>(p, ldp, row);
    const void *qr = row_ptr<QK>(q, ldq, row);
    float *orow = out + row * ldo;
    const int wid = threadIdx.x / kWave, lane = lane_id();
    float pm = 0.f, pinv = 1.f;
    if (PK != RDK_PROB_F32) {
        const SoftStat rs = merged_row_stat<PK>(w.pstat, w.p_splits, row);
        pm = rs.m;
        pinv = 1.0f / rs.s;
    }
    const float qm = QK == RDK_PROB_F32 ? 0.f : w.qstat[row].m;
    // totals of the first pass, summed in split order by every wave alike
    float zq = 0.f, tn = 0.f, an = 0.f, bs = 0.f;
    {
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        for (int i = lane; i < splits; i += kWave) {
            const float4 t = *(const float4 *)(w.tpart + (row * splits + i) * 4);
            a0 += t.x; a1 += t.y; a2 += t.z; a3 += t.w;
        }
        zq = wave_sum(a0); tn = wave_sum(a1); an = wave_sum(a2); bs = wave_sum(a3);
    }
    const float inv_zq = 1.0f / zq;
    const float theta = tn * inv_zq;
    const float inv_S = 1.0f / (an * inv_zq + theta * bs);
    const float fN = (float)N;
    const float pfill = PK == RDK_PROB_F32 ? 0.f : -INFINITY;
    for (int c = c_begin + wid; c < c_end; c += kWaves) {
        const int64_t base = (int64_t)c * kChunk + lane * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t idx = base + i * 256;
            if (idx >= N) continue;
            const float4 pv = load4<PK>(pr, idx, N, vec_p, pfill);
            const float pe[4] = {to_weight<PK>(pv.x, pm, pinv), to_weight<PK>(pv.y, pm, pinv),
                                 to_weight<PK>(pv.z, pm, pinv), to_weight<PK>(pv.w, pm, pinv)};
            int4 sv = make_int4(-1, -1, -1, -1);
            if (idx + 3 < N) {
                sv = *(const int4 *)(slot_of + idx);
            } else {
                if (idx + 0 < N) sv.x = slot_of[idx + 0];
                if (idx + 1 < N) sv.y = slot_of[idx + 1];
                if (idx + 2 < N) sv.z = slot_of[idx + 2];
            }
            const int se[4] = {sv.x, sv.y, sv.z, sv.w};
            float o[4];
            float qraw[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) qraw[e] = load1<QK>(qr, max(se[e], 0));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float qp = se[e] >= 0 ? to_weight<QK>(qraw[e], qm, 1.f) * inv_zq : 0.f;
                o[e] = (fN * qp + theta * pe[e]) / (fN + pe[e]) * inv_S;
            }
            if (vec_o && idx + 3 < N) {
                *(float4 *)(orow + idx) = make_float4(o[0], o[1], o[2], o[3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (idx + e < N) orow[idx + e] = o[e];
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Identity kernel: q' scattered to the kept ids, zero elsewhere (token-level intersection, Eq. 1).
template <int QK>
__global__ __launch_bounds__(kThreads) void tli_scatter_kernel(const void *q, int64_t ldq, const int32_t *slot_of, int N,
                                                               const SoftStat *qstat, float *out, int64_t ldo)
{
    const int64_t row = blockIdx.y;
    const void *qr = row_ptr<QK>(q, ldq, row);
    const float qm = qstat[row].m, inv = 1.0f / qstat[row].s;
    for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < N; j += (int64_t)gridDim.x * kThreads) {
        const int s = slot_of[j];
        out[row * ldo + j] = s >= 0 ? to_weight<QK>(load1<QK>(qr, s), qm, 1.f) * inv : 0.f;
    }
}

// ------------------------------------------------------------------------------------------------
// Sparse product, preparation: drafter weights of 16 positions side by side,
//   qT[(pb * n + s) * 16 + r] = weight(q[pb*16 + r, s])   (zero for positions beyond B),
// so that one neighbour of one id is a single 64-byte read serving 16 positions.
template <int QK>
__global__ __launch_bounds__(kThreads) void q_transpose_kernel(const void *q, int64_t ldq, int n, int B, const SoftStat *qpart,
                                                               int q_splits, SoftStat *qstat, float *qT)
{
    __shared__ float tile[64][kPosBlock + 1];
    __shared__ SoftStat rowstat[kPosBlock];
    const int pb = blockIdx.y;
    const int s0 = blockIdx.x * 64;
    {   // merge the row statistics of the 16 positions (4 per wavefront); the first slot tile publishes them
        const int wid = threadIdx.x / kWave;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = wid * 4 + i;
            const int64_t b = (int64_t)pb * kPosBlock + r;
            SoftStat st;
            st.m = 0.f;
            st.s = 1.f;
            if (b < B) st = merged_row_stat<QK>(qpart, q_splits, b);
            if (lane_id() == 0) {
                rowstat[r] = st;
                if (blockIdx.x == 0 && b < B) qstat[b] = st;
            }
        }
    }
    __syncthreads();
    {   // read: 16 rows x 64 slots, 16 threads per row, 4 slots per thread
        const int r = threadIdx.x / 16, c4 = (threadIdx.x % 16) * 4;
        const int64_t b = (int64_t)pb * kPosBlock + r;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (b < B) {
            const void *qr = row_ptr<QK>(q, ldq, b);
            const float qm = rowstat[r].m;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (s0 + c4 + e < n) v[e] = to_weight<QK>(load1<QK>(qr, s0 + c4 + e), qm, 1.f);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) tile[c4 + e][r] = v[e];
    }
    __syncthreads();
    {   // write: 64 slots x 16 positions, contiguous
        const int sl = threadIdx.x / 4, pq = (threadIdx.x % 4) * 4;
        if (s0 + sl < n) {
            float4 o = make_float4(tile[sl][pq], tile[sl][pq + 1], tile[sl][pq + 2], tile[sl][pq + 3]);
            *(float4 *)(qT + ((int64_t)pb * n + s0 + sl) * kPosBlock + pq) = o;
        }
    }
}

// Broadcast within each group of four lanes: every lane receives the value held by lane `SRC` of its group.
template <int SRC>
__device__ __forceinline__ int quad_bcast(int v)
{
    return __builtin_amdgcn_mov_dpp(v, SRC * 0x55, 0xf, 0xf, true);
}

// Sparse product.  A wavefront covers 16 target ids x 16 positions: lane = 4 * (id within 16) + quarter,
// each lane accumulates four positions (one float4) of one id.  The four lanes of an id each load a
// quarter of its (slot, weight) row and pass the entries round by DPP.  Every gather is 16 bytes per
// lane, 64 bytes per id, out of the position-minor drafter table that stays in the L2 of the XCD the
// block runs on: blocks are numbered so that an XCD sweeps all id tiles of one position block before
// it moves to the next (consecutive block ids go to consecutive XCDs).
__global__ __launch_bounds__(kThreads) void sparse_product_kernel(const int32_t *ell_idx, const float *ell_w, int kk,
                                                                  const float *qT, const SoftStat *qstat, int N, int n, int B,
                                                                  int tiles, int per_xcd, int total_work, float *out,
                                                                  int64_t ldo, bool vec_o)
{
    __shared__ float stage[kPosBlock][kIdsPerBlock + 4];
    const int xcd = blockIdx.x % 8, rank = blockIdx.x / 8;
    const int work = xcd * per_xcd + rank;
    if (rank >= per_xcd || work >= total_work) return;
    const int pb = work / tiles, tile = work % tiles;
    const int wid = threadIdx.x / kWave, lane = lane_id();
    const int quarter = lane & 3, sub = lane >> 2;
    const float *qslab = qT + (int64_t)pb * n * kPosBlock + quarter * 4;

    float inv_z[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int b = pb * kPosBlock + quarter * 4 + e;
        inv_z[e] = b < B ? 1.0f / qstat[b].s : 0.f;
    }

#pragma unroll 1
    for (int step = 0; step < kIdsPerBlock / 64; ++step) {
        const int jl = step * 64 + wid * 16 + sub;           // id within the tile
        const int64_t j = (int64_t)tile * kIdsPerBlock + jl;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int t0 = 0; t0 < kk; t0 += 16) {
            int4 iv = make_int4(0, 0, 0, 0);
            float4 wv = make_float4(0.f, 0.f, 0.f, 0.f);
            if (j < N && t0 + quarter * 4 < kk) {
                iv = *(const int4 *)(ell_idx + j * kk + t0 + quarter * 4);
                wv = *(const float4 *)(ell_w + j * kk + t0 + quarter * 4);
            }
            const int ie[4] = {iv.x, iv.y, iv.z, iv.w};
            const int we[4] = {__float_as_int(wv.x), __float_as_int(wv.y), __float_as_int(wv.z), __float_as_int(wv.w)};
            // all sixteen gathers are issued before any is used; padding entries carry weight 0 and slot 0
            float4 g[16];
            float wt[16];
#define RDK_GATHER(SRC, E)                                                                       \
    {                                                                                            \
        const int s_ = quad_bcast<SRC>(ie[E]);                                                   \
        wt[SRC * 4 + E] = __int_as_float(quad_bcast<SRC>(we[E]));                                \
        g[SRC * 4 + E] = *(const float4 *)(qslab + (int64_t)s_ * kPosBlock);                     \
    }
#define RDK_QUARTER(SRC) RDK_GATHER(SRC, 0) RDK_GATHER(SRC, 1) RDK_GATHER(SRC, 2) RDK_GATHER(SRC, 3)
            RDK_QUARTER(0) RDK_QUARTER(1) RDK_QUARTER(2) RDK_QUARTER(3)
#undef RDK_QUARTER
#undef RDK_GATHER
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                acc.x += wt[t] * g[t].x; acc.y += wt[t] * g[t].y; acc.z += wt[t] * g[t].z; acc.w += wt[t] * g[t].w;
            }
        }
        stage[quarter * 4 + 0][jl] = acc.x * inv_z[0];
        stage[quarter * 4 + 1][jl] = acc.y * inv_z[1];
        stage[quarter * 4 + 2][jl] = acc.z * inv_z[2];
        stage[quarter * 4 + 3][jl] = acc.w * inv_z[3];
    }
    __syncthreads();
    // 16 rows x 256 ids: each thread writes four float4
    const int64_t j0 = (int64_t)tile * kIdsPerBlock;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int f = it * kThreads + threadIdx.x;   // float4 index within the tile
        const int r = f / (kIdsPerBlock / 4), c = (f % (kIdsPerBlock / 4)) * 4;
        const int b = pb * kPosBlock + r;
        if (b >= B) continue;
        float *o = out + (int64_t)b * ldo + j0 + c;
        if (vec_o && j0 + c + 3 < N) {
            *(float4 *)o = make_float4(stage[r][c], stage[r][c + 1], stage[r][c + 2], stage[r][c + 3]);
        } else {
            for (int e = 0; e < 4; ++e)
                if (j0 + c + e < N) o[e] = stage[r][c + e];
        }
    }
}

template <int PK, int QK>
rdk_status_t run_taylor(const KernelHandle &h, RowInput p, RowInput q, int32_t B, float *out, int64_t ldo, void *ws,
                        hipStream_t st)
{
    LinearWs w = carve(h, B, ws);
    rdk_status_t rc;
    if (PK != RDK_PROB_F32) {
        rc = launch_row_stats<PK>(p, h.N, B, w.p_splits, w.pstat, st);
        if (rc != RDK_OK) return rc;
    }
    if (QK != RDK_PROB_F32) {
        rc = launch_row_stats<QK>(q, h.n, B, 1, w.qstat, st);
        if (rc != RDK_OK) return rc;
    }
    const bool vec_p = rows_vectorisable(p.ptr, p.ld, p.kind);
    const bool vec_o = rows_vectorisable(out, ldo, RDK_PROB_F32);
    {
        TimedLaunch timed("taylor_stats_kernel", st);
        hipLaunchKernelGGL((taylor_stats_kernel<PK, QK>), dim3((unsigned)B * w.t_splits), dim3(kThreads), 0, st, p.ptr, p.ld,
                           q.ptr, q.ld, h.slot_of, h.N, w.t_splits, vec_p, w);
    }
    RDK_LAUNCH_CHECK("taylor_stats_kernel");
    {
        TimedLaunch timed("taylor_write_kernel", st);
        hipLaunchKernelGGL((taylor_write_kernel<PK, QK>), dim3((unsigned)B * w.t_splits), dim3(kThreads), 0, st, p.ptr, p.ld,
                           q.ptr, q.ld, h.slot_of, h.N, w.t_splits, vec_p, vec_o, w, out, ldo);
    }
    RDK_LAUNCH_CHECK("taylor_write_kernel");
    return RDK_OK;
}

template <int QK>
rdk_status_t run_sparse(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws, hipStream_t st)
{
    LinearWs w = carve(h, B, ws);
    if (h.format == RDK_IDENTITY) {
        rdk_status_t rc1 = launch_row_stats<QK>(q, h.n, B, 1, w.qstat, st);
        if (rc1 != RDK_OK) return rc1;
        const int bx = (h.N + kThreads * 4 - 1) / (kThreads * 4);
        {
            TimedLaunch timed("tli_scatter_kernel", st);
            hipLaunchKernelGGL((tli_scatter_kernel<QK>), dim3(bx, B), dim3(kThreads), 0, st, q.ptr, q.ld, h.slot_of, h.N, w.qstat,
                               out, ldo);
        }
        RDK_LAUNCH_CHECK("tli_scatter_kernel");
        return RDK_OK;
    }
    rdk_status_t rc = launch_row_stats<QK>(q, h.n, B, w.q_splits, w.qpart, st);
    if (rc != RDK_OK) return rc;
    const int pbs = (B + kPosBlock - 1) / kPosBlock;
    {
        TimedLaunch timed("q_transpose_kernel", st);
        hipLaunchKernelGGL((q_transpose_kernel<QK>), dim3((h.n + 63) / 64, pbs), dim3(kThreads), 0, st, q.ptr, q.ld, h.n, B,
                           w.qpart, w.q_splits, w.qstat, w.qT);
    }
    RDK_LAUNCH_CHECK("q_transpose_kernel");
    const int tiles = (h.N + kIdsPerBlock - 1) / kIdsPerBlock;
    const int total = pbs * tiles;
    const int per_xcd = (total + 7) / 8;
    {
        TimedLaunch timed("sparse_product_kernel", st);
        hipLaunchKernelGGL(sparse_product_kernel, dim3(8 * per_xcd), dim3(kThreads), 0, st, h.ell_idx, h.ell_w, h.kk, w.qT,
                           w.qstat, h.N, h.n, B, tiles, per_xcd, total, out, ldo, rows_vectorisable(out, ldo, RDK_PROB_F32));
    }
    RDK_LAUNCH_CHECK("sparse_product_kernel");
    return RDK_OK;
}

}  // namespace

size_t linear_workspace_bytes(const KernelHandle &h, int32_t B)
{
    const int splits = row_splits(B, h.N, kWaves);
    const size_t pbs = (B + kPosBlock - 1) / kPosBlock;
    return align_up((size_t)B * splits * sizeof(SoftStat), 256) + align_up((size_t)B * sizeof(SoftStat), 256) +
           align_up((size_t)B * kMaxSplits * sizeof(SoftStat), 256) +
           align_up((size_t)B * splits * 4 * sizeof(float), 256) + align_up(pbs * h.n * kPosBlock * sizeof(float), 256);
}

rdk_status_t launch_taylor(const KernelHandle &h, RowInput p, RowInput q, int32_t B, float *out, int64_t ldo, void *ws,
                           hipStream_t st)
{
#define RDK_T(PK, QK) \
    if (p.kind == PK && q.kind == QK) return run_taylor<PK, QK>(h, p, q, B, out, ldo, ws, st);
    RDK_T(RDK_PROB_F32, RDK_PROB_F32)
    RDK_T(RDK_PROB_F32, RDK_LOGIT_F32)
    RDK_T(RDK_PROB_F32, RDK_LOGIT_BF16)
    RDK_T(RDK_LOGIT_F32, RDK_PROB_F32)
    RDK_T(RDK_LOGIT_F32, RDK_LOGIT_F32)
    RDK_T(RDK_LOGIT_F32, RDK_LOGIT_BF16)
    RDK_T(RDK_LOGIT_BF16, RDK_PROB_F32)
    RDK_T(RDK_LOGIT_BF16, RDK_LOGIT_F32)
    RDK_T(RDK_LOGIT_BF16, RDK_LOGIT_BF16)
#undef RDK_T
    return RDK_ERR_DTYPE;
}

rdk_status_t launch_sparse(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws, hipStream_t st)
{
    switch (q.kind) {
        case RDK_PROB_F32: return run_sparse<RDK_PROB_F32>(h, q, B, out, ldo, ws, st);
        case RDK_LOGIT_F32: return run_sparse<RDK_LOGIT_F32>(h, q, B, out, ldo, ws, st);
        case RDK_LOGIT_BF16: return run_sparse<RDK_LOGIT_BF16>(h, q, B, out, ldo, ws, st);
    }
    return RDK_ERR_DTYPE;
}

}  // namespace rdk
