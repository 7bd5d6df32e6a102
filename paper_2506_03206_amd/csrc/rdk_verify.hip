// Verification of a batch of positions: Alg. 4 of the paper, steps 2 and 4-10, given the target
// rows p and the redistributed drafter rows q' (both over the N target ids).
//
// Two launches (three when p arrives as logits):
//   [row_softstats]   running (max, sum exp) of the logits, a few partials per row
//   verify_stream     one pass over p and q': per 1024-id block the sums of q', of max(0, p - q')
//                     and of min(p, q')  (Def. 2.1 and the residual of step 8)
//   verify_finalize   per row: totals, Philox uniforms, the two inverse-CDF draws (block located from
//                     the partial sums, then re-read), the accept test, and the per-sequence scan
// The streaming pass is bound by HBM: 8 bytes per (position, id), nothing is written but 12 bytes
// per 1024 ids.
#include "rdk_rowstats.hpp"

namespace rdk {

namespace {

constexpr int kStreamThreads = 256;
constexpr int kWavesPerBlock = kStreamThreads / kWave;

struct VerifyWs {
    float *part_q, *part_r, *part_a;  // [B, nchunks]
    SoftStat *pstat;                  // [B, stat_splits] (logit input only)
    int nchunks, stat_splits;
};

__host__ __device__ inline int chunks_of(int64_t N) { return (int)((N + kChunk - 1) / kChunk); }

VerifyWs carve(const rdk_verify_desc_t &d, void *ws)
{
    VerifyWs w;
    w.nchunks = chunks_of(d.N);
    w.stat_splits = row_splits(d.B, d.N, kWavesPerBlock);
    char *p = (char *)ws;
    size_t per = align_up((size_t)d.B * w.nchunks * sizeof(float), 256);
    w.part_q = (float *)p; p += per;
    w.part_r = (float *)p; p += per;
    w.part_a = (float *)p; p += per;
    w.pstat = (SoftStat *)p;
    return w;
}

// ------------------------------------------------------------------------------------------------
template <int KIND, bool HAS_Q>
__global__ __launch_bounds__(kStreamThreads) void verify_stream_kernel(const void *p, int64_t ldp, const float *q, int64_t ldq,
                                                                       int N, int splits, bool vec_p, bool vec_q, VerifyWs w)
{
    const int64_t row = blockIdx.x / splits;
    const int split = blockIdx.x % splits;
    const int cpw = (w.nchunks + splits - 1) / splits;
    const int c_begin = split * cpw, c_end = min(w.nchunks, c_begin + cpw);
    const void *pr = row_ptr<KIND>(p, ldp, row);
    const float *qr = HAS_Q ? q + row * ldq : nullptr;
    const int wid = threadIdx.x / kWave, lane = lane_id();
    float m = 0.f, inv = 1.f;
    if (KIND != RDK_PROB_F32) {
        const SoftStat rs = merged_row_stat<KIND>(w.pstat, w.stat_splits, row);
        m = rs.m;
        inv = 1.0f / rs.s;
    }
    const float pfill = KIND == RDK_PROB_F32 ? 0.f : -INFINITY;

    for (int c = c_begin + wid; c < c_end; c += kWavesPerBlock) {
        const int64_t base = (int64_t)c * kChunk + lane * 4;
        float4 pv[4], qv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) pv[i] = load4<KIND>(pr, base + i * 256, N, vec_p, pfill);
        if (HAS_Q) {
#pragma unroll
            for (int i = 0; i < 4; ++i) qv[i] = load4<RDK_PROB_F32>(qr, base + i * 256, N, vec_q, 0.f);
        }
        float sq = 0.f, sr = 0.f, sa = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float pe[4] = {to_weight<KIND>(pv[i].x, m, inv), to_weight<KIND>(pv[i].y, m, inv),
                                 to_weight<KIND>(pv[i].z, m, inv), to_weight<KIND>(pv[i].w, m, inv)};
            if (HAS_Q) {
                const float qe[4] = {qv[i].x, qv[i].y, qv[i].z, qv[i].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    sq += qe[e];
                    sr += fmaxf(pe[e] - qe[e], 0.f);
                    sa += fminf(pe[e], qe[e]);
                }
            } else {
                sr += (pe[0] + pe[1]) + (pe[2] + pe[3]);
            }
        }
        sr = wave_sum(sr);
        if (HAS_Q) {
            sq = wave_sum(sq);
            sa = wave_sum(sa);
        }
        if (lane == 0) {
            const int64_t o = row * w.nchunks + c;
            w.part_r[o] = sr;
            if (HAS_Q) {
                w.part_q[o] = sq;
                w.part_a[o] = sa;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Wave-level helpers of the finalize step.

// Sum of a row of block partials in fp64; lane l owns the `per_lane` consecutive blocks from l*per_lane.
__device__ __forceinline__ double lane_partial_sum(const float *part, int nchunks, int per_lane)
{
    const int c0 = lane_id() * per_lane;
    double s = 0.0;
    for (int t = 0; t < per_lane; ++t)
        if (c0 + t < nchunks) s += (double)part[c0 + t];
    return s;
}

// Locates the block in which the inclusive prefix of `part` first exceeds thr.  Returns the block and
// the prefix before it; block = -1 when no prefix exceeds thr.
__device__ __forceinline__ int locate_block(const float *part, int nchunks, int per_lane, double lane_sum, double thr,
                                            double &prefix_before)
{
    const double incl = wave_inclusive_scan(lane_sum);
    const unsigned long long hits = __ballot(incl > thr);
    if (hits == 0ull) return -1;
    const int src = __ffsll(hits) - 1;
    int blk = -1;
    double pre = incl - lane_sum;
    if (lane_id() == src) {
        const int c0 = src * per_lane;
        for (int t = 0; t < per_lane && c0 + t < nchunks; ++t) {
            const double v = (double)part[c0 + t];
            if (pre + v > thr) {
                blk = c0 + t;
                break;
            }
            pre += v;
        }
    }
    blk = __shfl(blk, src, kWave);
    prefix_before = __shfl(pre, src, kWave);
    return blk;
}

// Within one 1024-id block, the smallest id whose inclusive prefix of weights exceeds thr_local; if
// rounding leaves none, the last id of the block with a positive weight.  wv[i] holds the weights of
// ids blk*1024 + i*256 + lane*4 .. +3 (zero beyond the row), all loaded before the scan starts.
__device__ __forceinline__ int search_block(const float4 (&wv)[4], int blk, double thr_local)
{
    const int lane = lane_id();
    double carried = 0.0;
    int last_positive = -1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = blk * kChunk + i * 256 + lane * 4;
        const double l0 = (double)wv[i].x, l1 = l0 + (double)wv[i].y, l2 = l1 + (double)wv[i].z, l3 = l2 + (double)wv[i].w;
        const double incl = wave_inclusive_scan(l3);
        const double excl = carried + (incl - l3);
        const unsigned long long hits = __ballot(excl + l3 > thr_local);
        if (hits != 0ull) {
            const int src = __ffsll(hits) - 1;
            const int e = (excl + l0 > thr_local) ? 0 : (excl + l1 > thr_local) ? 1 : (excl + l2 > thr_local) ? 2 : 3;
            return __shfl(idx + e, src, kWave);
        }
        const int mine = wv[i].w > 0.f ? 3 : wv[i].z > 0.f ? 2 : wv[i].y > 0.f ? 1 : wv[i].x > 0.f ? 0 : -1;
        const unsigned long long pos = __ballot(mine >= 0);
        if (pos != 0ull) {
            const int src = 63 - __clzll(pos);
            last_positive = __shfl(idx + mine, src, kWave);
        }
        carried += __shfl(incl, kWave - 1, kWave);
    }
    return last_positive;
}

template <int KIND, bool HAS_Q>
__global__ void verify_finalize_kernel(rdk_verify_desc_t d, const void *p, int64_t ldp, const float *q, int64_t ldq,
                                       bool vec_p, bool vec_q, VerifyWs w, int rows_per_block, bool scan_here,
                                       int32_t *draft_ids, uint8_t *accept, float *alpha, float *resid_mass,
                                       int32_t *resid_ids, int32_t *n_accepted, int32_t *out_tokens)
{
    __shared__ int32_t sh_draft[16], sh_resid[16];
    __shared__ uint8_t sh_acc[16];
    const int wid = threadIdx.x / kWave, lane = lane_id();
    const int64_t row = (int64_t)blockIdx.x * rows_per_block + wid;
    const int N = d.N;
    if (row < d.B) {
        const void *pr = row_ptr<KIND>(p, ldp, row);
        const float *qr = HAS_Q ? q + row * ldq : nullptr;
        float m = 0.f, inv = 1.f;
        if (KIND != RDK_PROB_F32) {
            const SoftStat rs = merged_row_stat<KIND>(w.pstat, w.stat_splits, row);
            m = rs.m;
            inv = 1.0f / rs.s;
        }
        const float pfill = KIND == RDK_PROB_F32 ? 0.f : -INFINITY;
        const int per_lane = (w.nchunks + kWave - 1) / kWave;
        const float *pq = w.part_q + row * w.nchunks;
        const float *prr = w.part_r + row * w.nchunks;
        const float *pa = w.part_a + row * w.nchunks;
        const bool draw_draft = HAS_Q && d.sample_draft;

        // 1. block partials (one round trip), uniforms meanwhile
        const double lane_r = lane_partial_sum(prr, w.nchunks, per_lane);
        const double lane_q = draw_draft ? lane_partial_sum(pq, w.nchunks, per_lane) : 0.0;
        const double lane_a = HAS_Q ? lane_partial_sum(pa, w.nchunks, per_lane) : 0.0;
        int32_t dtok = (HAS_Q && !d.sample_draft) ? draft_ids[row] : -1;
        uint32_t words[4];
        position_words(d.seed, d.offset + (uint64_t)row, words);
        const double R = wave_sum(lane_r);
        const double Q = draw_draft ? wave_sum(lane_q) : 0.0;
        const double A = HAS_Q ? wave_sum(lane_a) : 0.0;

        // 2. the blocks that hold the two prefix-sum crossings
        double thr_d = 0.0, thr_r = 0.0, before_d = 0.0, before_r = 0.0;
        int blk_d = -1, blk_r = -1;
        if (draw_draft && Q > 0.0) {
            thr_d = word_to_unit(words[0]) * Q;
            blk_d = locate_block(pq, w.nchunks, per_lane, lane_q, thr_d, before_d);
        }
        if (R > 0.0) {
            thr_r = word_to_unit(words[HAS_Q ? 2 : 3]) * R;
            blk_r = locate_block(prr, w.nchunks, per_lane, lane_r, thr_r, before_r);
        }

        // 3. both blocks are fetched together (one round trip), then scanned
        float4 wd[4], wp[4], wq[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t id_d = (int64_t)max(blk_d, 0) * kChunk + i * 256 + lane * 4;
            const int64_t id_r = (int64_t)max(blk_r, 0) * kChunk + i * 256 + lane * 4;
            if (draw_draft) wd[i] = load4<RDK_PROB_F32>(qr, id_d, N, vec_q, 0.f);
            wp[i] = load4<KIND>(pr, id_r, N, vec_p, pfill);
            if (HAS_Q) wq[i] = load4<RDK_PROB_F32>(qr, id_r, N, vec_q, 0.f);
        }
        if (blk_d >= 0) dtok = search_block(wd, blk_d, thr_d - before_d);
        // 4. the accept test needs p and q' at the draft token: issue those loads before the second scan
        float pd_raw = 0.f, qd = 0.f;
        const bool d_ok = HAS_Q && dtok >= 0 && dtok < N;
        if (d_ok) {
            pd_raw = load1<KIND>(pr, dtok);
            qd = qr[dtok];
        }
        int32_t rtok = -1;
        if (blk_r >= 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                wp[i].x = to_weight<KIND>(wp[i].x, m, inv);
                wp[i].y = to_weight<KIND>(wp[i].y, m, inv);
                wp[i].z = to_weight<KIND>(wp[i].z, m, inv);
                wp[i].w = to_weight<KIND>(wp[i].w, m, inv);
                if (HAS_Q) {
                    wp[i].x = fmaxf(wp[i].x - wq[i].x, 0.f);
                    wp[i].y = fmaxf(wp[i].y - wq[i].y, 0.f);
                    wp[i].z = fmaxf(wp[i].z - wq[i].z, 0.f);
                    wp[i].w = fmaxf(wp[i].w - wq[i].w, 0.f);
                }
            }
            rtok = search_block(wp, blk_r, thr_r - before_r);
        }
        uint8_t acc = 0;
        if (d_ok) acc = (word_to_unit(words[1]) * (double)qd < (double)to_weight<KIND>(pd_raw, m, inv)) ? 1 : 0;
        if (lane == 0) {
            if (HAS_Q && d.sample_draft) draft_ids[row] = dtok;
            accept[row] = acc;
            if (alpha) alpha[row] = (float)A;
            if (resid_mass) resid_mass[row] = (float)R;
            resid_ids[row] = rtok;
            if (scan_here) {
                sh_draft[wid] = dtok;
                sh_resid[wid] = rtok;
                sh_acc[wid] = acc;
            }
        }
    }
    if (scan_here) {  // the block holds exactly one sequence: steps 4-10 of Alg. 4
        __syncthreads();
        if (threadIdx.x == 0) {
            const int g = d.gamma;
            int j = 0;
            while (j < g && sh_acc[j]) ++j;
            if (n_accepted) n_accepted[blockIdx.x] = j;
            if (out_tokens) {
                int32_t *o = out_tokens + (int64_t)blockIdx.x * (g + 1);
                for (int i = 0; i <= g; ++i) o[i] = i < j ? sh_draft[i] : (i == j && j < g) ? sh_resid[i] : -1;
            }
        }
    }
}

// Per-sequence scan as a launch of its own (sequences longer than one workgroup's waves).
__global__ void sequence_scan_kernel(int S, int gamma, const int32_t *draft_ids, const uint8_t *accept,
                                     const int32_t *resid_ids, int32_t *n_accepted, int32_t *out_tokens)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= S) return;
    const int64_t b0 = (int64_t)s * gamma;
    int j = 0;
    while (j < gamma && accept[b0 + j]) ++j;
    if (n_accepted) n_accepted[s] = j;
    if (out_tokens) {
        int32_t *o = out_tokens + (int64_t)s * (gamma + 1);
        for (int i = 0; i <= gamma; ++i) o[i] = i < j ? draft_ids[b0 + i] : (i == j && j < gamma) ? resid_ids[b0 + i] : -1;
    }
}

__global__ void philox_words_kernel(uint64_t seed, uint64_t offset, int count, uint32_t *words)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    uint32_t w[4];
    position_words(seed, offset + (uint64_t)i, w);
    for (int j = 0; j < 4; ++j) words[(int64_t)i * 4 + j] = w[j];
}

template <int KIND, bool HAS_Q>
rdk_status_t run_verify(const rdk_verify_desc_t &d, RowInput p, const float *q, int64_t ldq, int32_t *draft_ids,
                        uint8_t *accept, float *alpha, float *resid_mass, int32_t *resid_ids, int32_t *n_accepted,
                        int32_t *out_tokens, void *ws, hipStream_t st)
{
    VerifyWs w = carve(d, ws);
    const bool vec_p = rows_vectorisable(p.ptr, p.ld, p.kind);
    const bool vec_q = HAS_Q ? rows_vectorisable(q, ldq, RDK_PROB_F32) : false;
    const int splits = row_splits(d.B, d.N, kWavesPerBlock);
    if (KIND != RDK_PROB_F32) {
        rdk_status_t rc = launch_row_stats<KIND>(p, d.N, d.B, w.stat_splits, w.pstat, st);
        if (rc != RDK_OK) return rc;
    }
    {
        TimedLaunch timed("verify_stream_kernel", st);
        hipLaunchKernelGGL((verify_stream_kernel<KIND, HAS_Q>), dim3((unsigned)d.B * splits), dim3(kStreamThreads), 0, st, p.ptr,
                           p.ld, q, ldq, d.N, splits, vec_p, vec_q, w);
    }
    RDK_LAUNCH_CHECK("verify_stream_kernel");
    const bool scan_here = d.gamma >= 1 && d.gamma <= 16;
    const int rows_per_block = scan_here ? d.gamma : 4;
    const int blocks = (d.B + rows_per_block - 1) / rows_per_block;
    {
        TimedLaunch timed("verify_finalize_kernel", st);
        hipLaunchKernelGGL((verify_finalize_kernel<KIND, HAS_Q>), dim3(blocks), dim3(rows_per_block * kWave), 0, st, d, p.ptr,
                           p.ld, q, ldq, vec_p, vec_q, w, rows_per_block, scan_here, draft_ids, accept, alpha, resid_mass,
                           resid_ids, n_accepted, out_tokens);
    }
    RDK_LAUNCH_CHECK("verify_finalize_kernel");
    if (d.gamma > 16 && (n_accepted || out_tokens)) {
        const int S = d.B / d.gamma;
        {
            TimedLaunch timed("sequence_scan_kernel", st);
            hipLaunchKernelGGL(sequence_scan_kernel, dim3((S + 63) / 64), dim3(64), 0, st, S, d.gamma, draft_ids, accept,
                               resid_ids, n_accepted, out_tokens);
        }
        RDK_LAUNCH_CHECK("sequence_scan_kernel");
    }
    return RDK_OK;
}

}  // namespace

size_t verify_workspace_bytes(const rdk_verify_desc_t &d)
{
    const int nchunks = chunks_of(d.N);
    const size_t per = align_up((size_t)d.B * nchunks * sizeof(float), 256);
    return 3 * per + align_up((size_t)d.B * row_splits(d.B, d.N, kWavesPerBlock) * sizeof(SoftStat), 256);
}

rdk_status_t launch_verify(const rdk_verify_desc_t &d, RowInput p, const float *q_prime, int64_t ldq, int32_t *draft_ids,
                           uint8_t *accept, float *alpha, float *resid_mass, int32_t *resid_ids, int32_t *n_accepted,
                           int32_t *out_tokens, void *ws, hipStream_t st)
{
#define RDK_VERIFY_CASE(K)                                                                                                  \
    case K:                                                                                                                 \
        return q_prime ? run_verify<K, true>(d, p, q_prime, ldq, draft_ids, accept, alpha, resid_mass, resid_ids,           \
                                             n_accepted, out_tokens, ws, st)                                                \
                       : run_verify<K, false>(d, p, q_prime, ldq, draft_ids, accept, alpha, resid_mass, resid_ids,          \
                                              n_accepted, out_tokens, ws, st);
    switch (p.kind) {
        RDK_VERIFY_CASE(RDK_PROB_F32)
        RDK_VERIFY_CASE(RDK_LOGIT_F32)
        RDK_VERIFY_CASE(RDK_LOGIT_BF16)
    }
#undef RDK_VERIFY_CASE
    return RDK_ERR_DTYPE;
}

rdk_status_t launch_philox_words(uint64_t seed, uint64_t offset, int32_t count, uint32_t *words, hipStream_t st)
{
    hipLaunchKernelGGL(philox_words_kernel, dim3((count + 255) / 256), dim3(256), 0, st, seed, offset, count, words);
    RDK_LAUNCH_CHECK("philox_words_kernel");
    return RDK_OK;
}

}  // namespace rdk
