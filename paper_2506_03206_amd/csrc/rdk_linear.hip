// Linear-time redistribution (Alg. 1, steps 1-2) in its two forms:
//   * the first-order closed form, Eq. 3 of the paper (no matrix, needs the target row p);
//   * (the product M^T q' with the top-k sparse kernel lives in rdk_sparse.hip);
//   * the identity kernel: token-level intersection itself.
// Step 1 (token-level intersection, Eq. 1) is folded in: the drafter row is only ever used divided
// by its own sum over the kept slots.
#include "rdk_finalize.hpp"

namespace rdk {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

struct LinearWs {
    SoftStat *pstat;   // [B, p_splits]  target row softmax statistics (logit p only)
    SoftStat *qstat;   // [B]            drafter row: (max, sum exp) or (0, sum)
    float *tpart;      // [B, t_splits, 8]  Taylor partial sums (4 used by the two-pass form, 8 by the one-pass form)
    int p_splits, t_splits;
};

LinearWs carve(const KernelHandle &h, int32_t B, void *ws)
{
    LinearWs w;
    w.p_splits = row_splits(B, h.N, kWaves);
    w.t_splits = w.p_splits;
    char *p = (char *)ws;
    w.pstat = (SoftStat *)p; p += align_up((size_t)B * w.p_splits * sizeof(SoftStat), 256);
    w.qstat = (SoftStat *)p; p += align_up((size_t)B * sizeof(SoftStat), 256);
    w.tpart = (float *)p;
    return w;
}

// ------------------------------------------------------------------------------------------------
// The kept ids ascend, so the kept ids inside one chunk of kChunk target ids own a contiguous run of slots
// lo .. hi-1 (chunk_lo of the kernel handle).  A wavefront reads that run of the drafter row and of kept_ids with
// coalesced loads and scatters it through a private LDS array (kChunk words + one spare word per lane) into id
// order; afterwards lane l holds the unnormalised drafter weights of the ids  base + i*256 + l*4 .. +3  (i = 0..3),
// the same ids whose target values it loads; ids that are not kept get 0.  This replaces one gather per id.
__device__ __forceinline__ void wave_lds_sync()
{
    // LDS operations of one wavefront execute in order: only the compiler has to be kept from moving them
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int QK>
__device__ __forceinline__ void stage_chunk(float *lds, const void *qr, bool vec_q, int n, float qm, const int32_t *kept, int lo,
                                            int hi, int base, float4 (&qd)[4])
{
    const int lane = lane_id();
    float4 *l4 = (float4 *)lds;
#pragma unroll
    for (int i = 0; i < 4; ++i) l4[i * kWave + lane] = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_sync();
    // All quads of the run lie inside the row (true for every chunk but, when n is not a multiple of four, the last):
    // the same answer for the whole wavefront.  Then the sweep over the run is uniform too: lanes past its end are
    // sent to the last quad of the row (they repeat what its own lane stores), and no load or store sits behind a
    // per-lane branch.
    if (vec_q && ((hi + 3) & ~3) <= n) {
        const int last_quad = (n & ~3) - 4;
        for (int s0 = lo & ~3; s0 < hi; s0 += 4 * kWave) {
            const int s = min(s0 + lane * 4, last_quad);
            const int4 kv = *(const int4 *)(kept + s);
            const float4 qv = load4_full<QK>(qr, s);
            const int ke[4] = {kv.x, kv.y, kv.z, kv.w};
            const float qe[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool mine = s + e >= lo && s + e < hi;
                lds[mine ? ((ke[e] - base) & (kChunk - 1)) : kChunk + lane] = to_weight<QK>(qe[e], qm, 1.f);
            }
        }
    } else {
        for (int s = (lo & ~3) + lane * 4; s < hi; s += 4 * kWave) {
            int4 kv = make_int4(0, 0, 0, 0);
            if (s + 3 < n) {
                kv = *(const int4 *)(kept + s);
            } else {
                if (s + 0 < n) kv.x = kept[s + 0];
                if (s + 1 < n) kv.y = kept[s + 1];
                if (s + 2 < n) kv.z = kept[s + 2];
            }
            const float4 qv = load4<QK>(qr, s, n, vec_q, QK == RDK_PROB_F32 ? 0.f : -INFINITY);
            const int ke[4] = {kv.x, kv.y, kv.z, kv.w};
            const float qe[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {   // the weight is formed here, once per kept slot rather than once per target id
                const bool mine = s + e >= lo && s + e < hi;   // others go to a spare word per lane: no branch
                lds[mine ? ((ke[e] - base) & (kChunk - 1)) : kChunk + lane] = to_weight<QK>(qe[e], qm, 1.f);
            }
        }
    }
    wave_lds_sync();
#pragma unroll
    for (int i = 0; i < 4; ++i) qd[i] = l4[i * kWave + lane];
}

// Both passes hide memory latency by occupancy alone: they are held to 64 registers (eight wavefronts per SIMD).
// Eq. 3, first pass.  For the ids of one split of a row:
//   Zq += q^_s, Tn += q^_s p_j, An += N q^_s / (N + p_j)   over kept ids j (slot s),
//   Bs += p_j / (N + p_j)                                    over all ids j.
// Then theta = Tn / Zq and sum_j pt_j = An / Zq + theta * Bs, because
//   pt_j = N q'_j / (N + p_j) + theta p_j / (N + p_j)  with q'_j = q^_s / Zq on kept ids, 0 elsewhere.
// KEEP_P: the target rows are loaded as data that will be used again (the fused call: the second pass is their last
// reader and a batch fits the memory-side cache); otherwise they are streamed like every other single-use row.
template <int PK, int QK, bool KEEP_P>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(8))) void taylor_stats_kernel(
    const void *p, int64_t ldp, const void *q, int64_t ldq,
                                                                const int32_t *kept, const int32_t *chunk_lo, int N, int n,
                                                                int splits, bool vec_p, bool vec_q, LinearWs w)
{
    __shared__ __attribute__((aligned(16))) float qchunk[kWaves][kChunk + kWave];
    const int64_t row = blockIdx.x / splits;
    const int split = blockIdx.x % splits;
    const int nchunks = (N + kChunk - 1) / kChunk;
    const int cpw = (nchunks + splits - 1) / splits;
    const int c_begin = split * cpw, c_end = min(nchunks, c_begin + cpw);
    const void *pr = row_ptr<PK>(p, ldp, row);
    const void *qr = row_ptr<QK>(q, ldq, row);
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = lane_id();
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
    // the slot run of the next chunk is looked up one iteration ahead, so that no load of a chunk waits for another
    int c = c_begin + wid;
    int lo = 0, hi = 0;
    if (c < c_end) {
        lo = chunk_lo[c];
        hi = chunk_lo[c + 1];
    }
    for (; c < c_end; c += kWaves) {
        const int base = c * kChunk;
        float4 pv[4], qd[4];
        load_chunk<PK, !KEEP_P>(pr, base, N, vec_p, pfill, pv);
        const int lo_now = lo, hi_now = hi;
        if (c + kWaves < c_end) {
            lo = chunk_lo[c + kWaves];
            hi = chunk_lo[c + kWaves + 1];
        }
        stage_chunk<QK>(qchunk[wid], qr, vec_q, n, qm, kept, lo_now, hi_now, base, qd);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float pe[4] = {to_weight<PK>(pv[i].x, pm, pinv), to_weight<PK>(pv[i].y, pm, pinv),
                                 to_weight<PK>(pv[i].z, pm, pinv), to_weight<PK>(pv[i].w, pm, pinv)};
            const float qe[4] = {qd[i].x, qd[i].y, qd[i].z, qd[i].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float r = __builtin_amdgcn_rcpf(fN + pe[e]);
                bs += pe[e] * r;
                const float qh = qe[e];                            // zero on ids that are not kept
                zq += qh;
                tn += qh * pe[e];
                an += qh * r;                                      // times N at the end
            }
        }
    }
    an *= fN;
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

// Eq. 3, first pass for LOGIT target rows without a softmax pass of its own.  The sums of the pass above need the
// normalised p inside 1 / (N + p), i.e. the row maximum and normaliser first.  But p / N <= 1 / N, so with x = p / N
//   N / (N + p) = 1 - x + x^2 - x^3 + O(N^-4),      p / (N + p) = x - x^2 + x^3 + O(N^-4),
// and every term is a power sum of e = exp(z - m) that can be carried under a running maximum m and rescaled when
// the maximum grows (a factor exp(k (m_old - m_new)) for the k-th power).  Per split of a row, relative to the
// split's own maximum m:   S_k = sum_j e_j^k  and  Q_k = sum over kept ids of q^_s e_j^k,  k = 1..3,  and Q_0 = sum q^_s.
// The record (m, S1, S2, S3, Q0, Q1, Q2, Q3) goes to tpart, and (m, S1) also to pstat: the softmax statistics every
// later kernel reads, in the layout of the softmax pass this kernel replaces.  Used for N >= kOnePassMinN, where the
// truncation (a relative N^-3 of the smaller sum) is far below fp32 rounding.
constexpr int kOnePassMinN = 1024;

template <int PK, int QK, bool KEEP_P>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(8))) void taylor_stats_onepass_kernel(
    const void *p, int64_t ldp, const void *q, int64_t ldq, const int32_t *kept, const int32_t *chunk_lo, int N, int n,
    int splits, bool vec_p, bool vec_q, LinearWs w)
{
    static_assert(PK != RDK_PROB_F32, "probabilities need no normaliser: the two-pass kernel serves them");
    __shared__ __attribute__((aligned(16))) float qchunk[kWaves][kChunk + kWave];
    const int64_t row = blockIdx.x / splits;
    const int split = blockIdx.x % splits;
    const int nchunks = (N + kChunk - 1) / kChunk;
    const int cpw = (nchunks + splits - 1) / splits;
    const int c_begin = split * cpw, c_end = min(nchunks, c_begin + cpw);
    const void *pr = row_ptr<PK>(p, ldp, row);
    const void *qr = row_ptr<QK>(q, ldq, row);
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = lane_id();
    const float qm = QK == RDK_PROB_F32 ? 0.f : w.qstat[row].m;
    float m = -INFINITY;                                         // running maximum, the same in all lanes
    float s1 = 0.f, s2 = 0.f, s3 = 0.f, q0 = 0.f, q1 = 0.f, q2 = 0.f, q3 = 0.f;
    int c = c_begin + wid;
    int lo = 0, hi = 0;
    if (c < c_end) {
        lo = chunk_lo[c];
        hi = chunk_lo[c + 1];
    }
    for (; c < c_end; c += kWaves) {
        const int base = c * kChunk;
        float4 pv[4], qd[4];
        load_chunk<PK, !KEEP_P>(pr, base, N, vec_p, -INFINITY, pv);
        const int lo_now = lo, hi_now = hi;
        if (c + kWaves < c_end) {
            lo = chunk_lo[c + kWaves];
            hi = chunk_lo[c + kWaves + 1];
        }
        stage_chunk<QK>(qchunk[wid], qr, vec_q, n, qm, kept, lo_now, hi_now, base, qd);
        float cm = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) cm = fmaxf(cm, fmaxf(fmaxf(pv[i].x, pv[i].y), fmaxf(pv[i].z, pv[i].w)));
        cm = wave_max(cm);                                       // finite: a chunk holds at least one id
        if (cm > m) {                                            // the same decision in all lanes
            const float f = soft_exp(m - cm), f2 = f * f, f3 = f2 * f;   // 0 on the first chunk (m = -inf)
            s1 *= f; s2 *= f2; s3 *= f3;
            q1 *= f; q2 *= f2; q3 *= f3;
            m = cm;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float pe[4] = {soft_exp(pv[i].x - m), soft_exp(pv[i].y - m), soft_exp(pv[i].z - m), soft_exp(pv[i].w - m)};
            const float qe[4] = {qd[i].x, qd[i].y, qd[i].z, qd[i].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float e1 = pe[e], e2 = e1 * e1, e3 = e2 * e1;   // exp(-inf) = 0 beyond N
                const float qh = qe[e];                                // zero on ids that are not kept
                s1 += e1; s2 += e2; s3 += e3;
                q0 += qh; q1 += qh * e1; q2 += qh * e2; q3 += qh * e3;
            }
        }
    }
    s1 = wave_sum(s1); s2 = wave_sum(s2); s3 = wave_sum(s3);
    q0 = wave_sum(q0); q1 = wave_sum(q1); q2 = wave_sum(q2); q3 = wave_sum(q3);
    __shared__ float sh[kWaves][8];
    if (lane == 0) {
        sh[wid][0] = m; sh[wid][1] = s1; sh[wid][2] = s2; sh[wid][3] = s3;
        sh[wid][4] = q0; sh[wid][5] = q1; sh[wid][6] = q2; sh[wid][7] = q3;
    }
    __syncthreads();
    if (threadIdx.x == 0) {   // wavefronts without a chunk hold m = -inf and zeros: their factor is 0
        float mm = sh[0][0];
        for (int i = 1; i < kWaves; ++i) mm = fmaxf(mm, sh[i][0]);
        float r[8] = {mm, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int i = 0; i < kWaves; ++i) {
            const float f = sh[i][0] > -INFINITY ? soft_exp(sh[i][0] - mm) : 0.f, f2 = f * f, f3 = f2 * f;
            r[1] += sh[i][1] * f; r[2] += sh[i][2] * f2; r[3] += sh[i][3] * f3;
            r[4] += sh[i][4]; r[5] += sh[i][5] * f; r[6] += sh[i][6] * f2; r[7] += sh[i][7] * f3;
        }
        float *dst = w.tpart + (row * splits + split) * 8;
        *(float4 *)dst = make_float4(r[0], r[1], r[2], r[3]);
        *(float4 *)(dst + 4) = make_float4(r[4], r[5], r[6], r[7]);
        SoftStat st;
        st.m = mm;
        st.s = r[1];
        w.pstat[row * splits + split] = st;
    }
}

// Everything the second pass of Eq. 3 needs about one row; built by all lanes of a wavefront alike.
struct TaylorArgs {
    const void *p, *q;
    int64_t ldp, ldq;
    const int32_t *slot_of, *kept, *chunk_lo;
    int N, n, splits;
    bool vec_p, vec_q;
    bool onepass;   // the first pass was the one-pass kernel: tpart holds its eight-word records
    LinearWs w;
};

template <int PK, int QK>
struct TaylorRow {
    const void *pr, *qr;
    const int32_t *slot_of;
    int N;
    bool vec_p;
    float pm, pinv, qm, inv_zq, theta, inv_S, fN, nzs, ths;   // nzs = N / (Zq S), ths = theta / S

    // Eq. 3 for one id: qh = unnormalised drafter weight of the id (0 if it is not kept), pe = its target weight
    __device__ __forceinline__ float value(float qh, float pe) const
    {
        return (nzs * qh + ths * pe) * __builtin_amdgcn_rcpf(fN + pe);
    }

    // q' of ids idx .. idx+3 (Eq. 3) in two steps: target values and slots first, then the drafter values
    struct Pending {
        float4 pv;
        int4 sv;
        float qraw[4];
    };
    template <int K>
    __device__ __forceinline__ void stage(Pending &t, int64_t idx) const
    {
        if (K == 0) {
            t.pv = rdk::load4<PK>(pr, idx, N, vec_p, PK == RDK_PROB_F32 ? 0.f : -INFINITY);
            t.sv = make_int4(-1, -1, -1, -1);
            if (idx + 3 < N) {
                t.sv = *(const int4 *)(slot_of + idx);
            } else {
                if (idx + 0 < N) t.sv.x = slot_of[idx + 0];
                if (idx + 1 < N) t.sv.y = slot_of[idx + 1];
                if (idx + 2 < N) t.sv.z = slot_of[idx + 2];
            }
        } else {
            const int se[4] = {t.sv.x, t.sv.y, t.sv.z, t.sv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) t.qraw[e] = rdk::load1<QK>(qr, max(se[e], 0));   // unconditional: loads stay batched
        }
    }
    __device__ __forceinline__ float4 result(Pending &t, int64_t idx) const
    {
        const float pe[4] = {to_weight<PK>(t.pv.x, pm, pinv), to_weight<PK>(t.pv.y, pm, pinv), to_weight<PK>(t.pv.z, pm, pinv),
                             to_weight<PK>(t.pv.w, pm, pinv)};
        const int se[4] = {t.sv.x, t.sv.y, t.sv.z, t.sv.w};
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float qh = se[e] >= 0 ? to_weight<QK>(t.qraw[e], qm, 1.f) : 0.f;
            o[e] = idx + e < N ? value(qh, pe[e]) : 0.f;
        }
        return make_float4(o[0], o[1], o[2], o[3]);
    }
    __device__ __forceinline__ float load1(int j) const
    {
        const float pe = to_weight<PK>(rdk::load1<PK>(pr, j), pm, pinv);
        const int s = slot_of[j];
        const float qh = s >= 0 ? to_weight<QK>(rdk::load1<QK>(qr, max(s, 0)), qm, 1.f) : 0.f;
        return value(qh, pe);
    }
};

template <int PK, int QK>
__device__ __forceinline__ TaylorRow<PK, QK> make_taylor_row(const TaylorArgs &a, int64_t row)
{
    TaylorRow<PK, QK> r;
    r.pr = row_ptr<PK>(a.p, a.ldp, row);
    r.qr = row_ptr<QK>(a.q, a.ldq, row);
    r.slot_of = a.slot_of;
    r.N = a.N;
    r.vec_p = a.vec_p;
    r.pm = 0.f;
    r.pinv = 1.f;
    if (PK != RDK_PROB_F32) {
        const SoftStat rs = merged_row_stat<PK>(a.w.pstat, a.w.p_splits, row);
        r.pm = rs.m;
        r.pinv = 1.0f / rs.s;
    }
    r.qm = QK == RDK_PROB_F32 ? 0.f : a.w.qstat[row].m;
    // totals of the first pass, summed in split order by every wavefront alike
    r.fN = (float)a.N;
    float zq, tn, an, bs;
    if (PK != RDK_PROB_F32 && a.onepass) {
        // power sums relative to each split's own maximum, brought to the row maximum; then the series in x = p / N
        float s2 = 0.f, s3 = 0.f, q0 = 0.f, q1 = 0.f, q2 = 0.f, q3 = 0.f;
        for (int i = lane_id(); i < a.splits; i += kWave) {
            const float *rec = a.w.tpart + (row * a.splits + i) * 8;
            const float4 t0 = *(const float4 *)rec, t1 = *(const float4 *)(rec + 4);
            const float f = soft_exp(t0.x - r.pm), f2 = f * f, f3 = f2 * f;   // 0 for a split without ids
            s2 += t0.z * f2; s3 += t0.w * f3;
            q0 += t1.x; q1 += t1.y * f; q2 += t1.z * f2; q3 += t1.w * f3;
        }
        s2 = wave_sum(s2); s3 = wave_sum(s3);
        q0 = wave_sum(q0); q1 = wave_sum(q1); q2 = wave_sum(q2); q3 = wave_sum(q3);
        const float c = r.pinv / r.fN, c2 = c * c, c3 = c2 * c;               // x_j = e_j c
        zq = q0;
        tn = q1 * r.pinv;                                                     // sum q^ p
        an = q0 - q1 * c + q2 * c2 - q3 * c3;                                 // sum q^ N / (N + p)
        bs = 1.0f / r.fN - s2 * c2 + s3 * c3;                                 // sum p / (N + p);  sum x = 1 / N
    } else {
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        for (int i = lane_id(); i < a.splits; i += kWave) {
            const float4 t = *(const float4 *)(a.w.tpart + (row * a.splits + i) * 4);
            a0 += t.x; a1 += t.y; a2 += t.z; a3 += t.w;
        }
        zq = wave_sum(a0); tn = wave_sum(a1); an = wave_sum(a2); bs = wave_sum(a3);
    }
    r.inv_zq = inv_mass(zq);                                   // a drafter row without mass gives the zero row
    r.theta = tn * r.inv_zq;
    r.inv_S = inv_mass(an * r.inv_zq + r.theta * bs);
    r.nzs = r.fN * r.inv_zq * r.inv_S;
    r.ths = r.theta * r.inv_S;
    return r;
}

// Eq. 3, second pass: q'_j = ((N q0_j + theta p_j) / (N + p_j)) / sum_j pt_j.  WRITE_Q stores it; FUSE adds the
// verification sums per 1024-id block (sum q', sum max(0, p - q'), sum min(p, q')).  Whether q' is stored (out != NULL)
// is decided at run time, so that the sums do not depend on it by a single bit.
template <int PK, int QK, bool FUSE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(8))) void taylor_write_kernel(
    TaylorArgs a, bool vec_o, float *out, int64_t ldo, float *part_q,
                                                                float *part_r, float *part_a)
{
    __shared__ __attribute__((aligned(16))) float qchunk[kWaves][kChunk + kWave];
    const int64_t row = blockIdx.x / a.splits;
    const int split = blockIdx.x % a.splits;
    const int nchunks = (a.N + kChunk - 1) / kChunk;
    const int cpw = (nchunks + a.splits - 1) / a.splits;
    const int c_begin = split * cpw, c_end = min(nchunks, c_begin + cpw);
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = lane_id();
    const float pfill = PK == RDK_PROB_F32 ? 0.f : -INFINITY;
    int c = c_begin + wid;
    int lo = 0, hi = 0;
    if (c < c_end) {   // requested before the row constants below are waited for
        lo = a.chunk_lo[c];
        hi = a.chunk_lo[c + 1];
    }
    const TaylorRow<PK, QK> tr = make_taylor_row<PK, QK>(a, row);
    float *orow = out ? out + row * ldo : nullptr;
    for (; c < c_end; c += kWaves) {
        const int base = c * kChunk;
        float4 pv[4], qd[4];
        load_chunk<PK>(tr.pr, base, a.N, a.vec_p, pfill, pv);
        const int lo_now = lo, hi_now = hi;
        if (c + kWaves < c_end) {
            lo = a.chunk_lo[c + kWaves];
            hi = a.chunk_lo[c + kWaves + 1];
        }
        stage_chunk<QK>(qchunk[wid], tr.qr, a.vec_q, a.n, tr.qm, a.kept, lo_now, hi_now, base, qd);
        float sq = 0.f, sr = 0.f, sa = 0.f;
        const bool full_o = vec_o && base + kChunk <= a.N;   // the whole chunk is stored with 16-byte stores
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t idx = (int64_t)base + i * 256 + lane * 4;
            const float pe[4] = {to_weight<PK>(pv[i].x, tr.pm, tr.pinv), to_weight<PK>(pv[i].y, tr.pm, tr.pinv),
                                 to_weight<PK>(pv[i].z, tr.pm, tr.pinv), to_weight<PK>(pv[i].w, tr.pm, tr.pinv)};
            const float qe[4] = {qd[i].x, qd[i].y, qd[i].z, qd[i].w};
            float oe[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float qh = qe[e];                              // zero on ids that are not kept
                oe[e] = tr.value(qh, pe[e]);   // ids beyond N: both weights are zero, and so is the value
            }
            if (orow) {
                if (full_o) {
                    *(float4 *)(orow + idx) = make_float4(oe[0], oe[1], oe[2], oe[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (idx + e < a.N) orow[idx + e] = oe[e];
                }
            }
            if (FUSE) {
                sq += (oe[0] + oe[1]) + (oe[2] + oe[3]);
                sr += (fmaxf(pe[0] - oe[0], 0.f) + fmaxf(pe[1] - oe[1], 0.f)) +
                      (fmaxf(pe[2] - oe[2], 0.f) + fmaxf(pe[3] - oe[3], 0.f));
                sa += (fminf(pe[0], oe[0]) + fminf(pe[1], oe[1])) + (fminf(pe[2], oe[2]) + fminf(pe[3], oe[3]));
            }
        }
        if (FUSE) {
            sq = wave_sum(sq);
            sr = wave_sum(sr);
            sa = wave_sum(sa);
            if (lane == 0) {
                const int64_t o = row * nchunks + c;
                part_q[o] = sq;
                part_r[o] = sr;
                part_a[o] = sa;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Eq. 3 and the verification sums in ONE pass over the target row (the fused call on probability rows when q' is not
// asked for).  The two-pass kernels above read p twice because the row constants (theta, sum of pt) are only known
// after the whole row has been seen.  Here one workgroup of sixteen wavefronts owns one position and keeps what the
// second step needs on chip:
//   * an id j that is not kept has q'_j = (theta / S) p_j / (N + p_j), which is below p_j (theta <= 1, S >= 1/2,
//     N >= 2), so its share of the three block sums is a closed form of  P = sum p_j  and  A = sum p_j / (N + p_j)
//     over the not-kept ids of the block: sum q' = sum min(p, q') = (theta / S) A,  sum max(0, p - q') = P - (theta / S) A;
//   * a kept id needs its own p and q^: while the row streams by, the target values of the kept ids are scattered
//     into LDS, chunk by chunk in slot order (4 n bytes: one value per drafter slot; the run of every chunk starts
//     on a 16-byte boundary).
// Step A streams p, guided by the kernel's lane map (L2-resident, shared by all rows), a wavefront per chunk.  The chunk's
// run of drafter values is fetched alongside (one contiguous piece of the drafter row); the wavefront reads its own
// scattered target values back in slot order and adds up q^, q^ p and q^ / (N + p) -- the sums of the row constants cost
// no pass of their own.  Step C, once the constants are known, forms q', max(0, p - q') and min(p, q') on the kept slots.
// Its unit of work is a piece of at most 64 slots of one chunk (a table of the kernel), dealt out to groups of sixteen
// lanes in turn, so that vocabularies whose kept ids crowd into a few chunks keep every lane busy; the drafter values of
// the pieces are asked for before the constants are known, the sums of a piece take four register-speed lane exchanges,
// and the pieces of a chunk are added up in their order.  HBM traffic: p and q once.
// q' of Eq. 3 re-computed from the row constants (the finish step needs the two blocks of the crossings).
template <int PK, int QK>
struct QpTaylor {
    static constexpr bool kSpreadRows = false;
    static constexpr int kStages = 2;
    TaylorArgs a;
    typedef TaylorRow<PK, QK> Row;
    __device__ __forceinline__ Row row(int64_t b) const { return make_taylor_row<PK, QK>(a, b); }
};

constexpr int kRowThreads = 1024;
constexpr int kRowWaves = kRowThreads / kWave;
constexpr int kRowGroups = kRowThreads / 16;   // groups of sixteen lanes: one piece of kept slots each per round of step C
constexpr int kRowHeld = 10;                   // pieces per group whose drafter values are requested ahead of the row constants

struct RowLds {      // offsets in floats into the dynamic LDS block
    int pk, zero, blk_p, blk_a, blk_all, blk_aq, red, items, item_lo, isum, sum_q, sum_r, sum_a, fin, total;
};

// Where the run of chunk c (first slot lo) starts in the LDS array of kept target values: a multiple of four floats, and
// far enough from the run before it (align down costs at most 3, the 4 c make up for it).
__host__ __device__ inline int row_run_start(int lo, int c) { return (lo & ~3) + 4 * c; }

// Upper bound on the number of pieces (the size of the kernel's table): one per chunk and one per 64 slots.
__host__ __device__ inline int row_max_items(int n, int nchunks) { return nchunks + n / 64 + 1; }

__host__ __device__ inline RowLds row_lds_layout(int n, int nchunks)
{
    RowLds L;
    int off = 0;
    // target values of the kept ids: runs of slots, one per chunk, and room for the quads that a piece reads past its end
    // (their values are masked)
    L.pk = off; off += ((n + 3) & ~3) + 4 * nchunks + 4;
    L.zero = off; off += 4;                            // a quad of zeros for the lanes past the end of a piece
    L.blk_p = off; off += 4 * nchunks;                 // per chunk, in four partial sums: p over the not-kept ids
    L.blk_a = off; off += 4 * nchunks;                 //            p / (N + p) over the not-kept ids
    L.blk_all = off; off += 4 * nchunks;               //            p / (N + p) over all ids
    L.blk_aq = off; off += 4 * nchunks;                //            q^ / (N + p) over the kept ids
    L.red = off; off += kRowWaves * 9;                 // what the wavefronts hand to each other between the steps
    const int mi = (row_max_items(n, nchunks) + 1) & ~1;
    L.items = off; off += 2 * mi;                      // the kernel's table of pieces
    L.item_lo = off; off += (nchunks + 1 + 3) & ~3;    // first piece of every chunk
    L.isum = off; off += 2 * mi;                       // per piece: sums of max(0, p - q') and min(p, q')
    // per chunk: the three block sums the finish step draws from.  They are formed when the kept target values have
    // served their purpose, and take their place (4 nchunks + 8 floats are there at least).
    L.sum_q = L.pk;
    L.sum_r = L.sum_q + ((nchunks + 3) & ~3);
    L.sum_a = L.sum_r + ((nchunks + 3) & ~3);
    L.fin = off; off += kFinishFloats + 4;             // what the wavefronts of the finish step hand to each other, the uniforms
    L.total = off;
    return L;
}

// One chunk of target values (16 ids per lane, the layout of load_chunk), the lane's record of the kernel's lane map
// for that chunk, and the chunk's run of slots [lo, hi).
struct RowChunk {
    float4 p[4];
    uint64_t map;
    int lo, hi;
};

template <int PK = RDK_PROB_F32>
__device__ __forceinline__ void row_fetch(const void *pr, const uint64_t *lane_map, const int32_t *chunk_lo, int c, int N,
                                          bool vec_p, RowChunk &b)
{
    load_chunk<PK>(pr, (int64_t)c * kChunk, N, vec_p, PK == RDK_PROB_F32 ? 0.f : -INFINITY, b.p);
    b.map = lane_map[(int64_t)c * kWave + lane_id()];
    b.lo = chunk_lo[c];
    b.hi = chunk_lo[c + 1];
}

// 1 / (N + p) for 0 <= p <= 1.  For a large vocabulary the first two terms of the series in p / N are exact to fp32
// rounding (the next term is (p / N)^2 <= 2^-24 of the result for N >= 4096) and cost one multiply-add instead of a
// reciprocal, which the vector unit issues at a quarter of the rate.
template <bool SERIES>
struct RowRcp {
    float fN, invN, invN2;
    __device__ __forceinline__ float operator()(float p) const
    {
        return SERIES ? fmaf(-p, invN2, invN) : __builtin_amdgcn_rcpf(fN + p);
    }
};

// Step A for one chunk c: target values of kept ids go to their slots in LDS; sp, sa: sums of p and of p / (N + p) over
// the ids that are not kept; sall: p / (N + p) over all of them.
template <bool SERIES>
__device__ __forceinline__ void row_scatter(const RowChunk &b, int c, int lo, const RowRcp<SERIES> &rcp, float *pk, float &sp,
                                            float &sa, float &sall)
{
    const uint32_t mask = (uint32_t)b.map & 0xFFFFu;
    const int run = row_run_start(lo, c);                         // where the chunk's first slot sits in LDS
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        char *at = (char *)(pk + run + (int)((b.map >> (16 + 12 * i)) & 0xFFFu));   // slot of the lane's first kept id of this group
        const float pe[4] = {b.p[i].x, b.p[i].y, b.p[i].z, b.p[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t kept = (mask >> (4 * i + e)) & 1u;
            if (kept) *(float *)at = pe[e];
            at += 4 * kept;
            const float r = rcp(pe[e]);
            const float pn = kept ? 0.f : pe[e];
            sp += pn;
            sa = fmaf(pn, r, sa);
            sall = fmaf(pe[e], r, sall);
        }
    }
}

// The raw drafter values of four consecutive slots from s on, for the lanes whose quad starts below `end` (the others get
// the value of weight zero; n = slots in the row).  One 16-byte load when the quad lies inside the row -- four bytes of
// alignment are all a global load of that size needs; its slots from `end` on belong to the row but not to the caller --
// and single loads for the quad that crosses the end of the row.  Every load writes the one result under a one-sided
// branch, so a sequence of calls issues its loads back to back (loads merged from two code paths would each be waited
// for at the merge).
template <int QK>
__device__ __forceinline__ float4 row_raw_quad(const void *qr, int s, int end, int n)
{
    const float none = QK == RDK_PROB_F32 ? 0.f : -INFINITY;
    float4 raw = make_float4(none, none, none, none);
    if (QK == RDK_LOGIT_BF16) {
        const uint16_t *r = (const uint16_t *)qr;
        if (s < end && s + 3 < n) {
            typedef unsigned short u16x4a __attribute__((ext_vector_type(4), aligned(2)));
            const u16x4a v = *(const u16x4a *)(r + s);
            raw = make_float4(bf16_to_f32(v.x), bf16_to_f32(v.y), bf16_to_f32(v.z), bf16_to_f32(v.w));
        }
        if (s < end && s + 3 >= n) {
            raw.x = bf16_to_f32(r[s]);
            if (s + 1 < n) raw.y = bf16_to_f32(r[s + 1]);
            if (s + 2 < n) raw.z = bf16_to_f32(r[s + 2]);
        }
    } else {
        const float *r = (const float *)qr;
        if (s < end && s + 3 < n) {
            typedef float f32x4a __attribute__((ext_vector_type(4), aligned(4)));
            const f32x4a v = *(const f32x4a *)(r + s);
            raw = make_float4(v.x, v.y, v.z, v.w);
        }
        if (s < end && s + 3 >= n) {
            raw.x = r[s];
            if (s + 1 < n) raw.y = r[s + 1];
            if (s + 2 < n) raw.z = r[s + 2];
        }
    }
    return raw;
}

// The drafter weights of a raw quad (a slot that was not loaded gives zero).
template <int QK>
__device__ __forceinline__ float4 row_weights_of(const float4 raw, float qm)
{
    return make_float4(to_weight<QK>(raw.x, qm, 1.f), to_weight<QK>(raw.y, qm, 1.f), to_weight<QK>(raw.z, qm, 1.f),
                       to_weight<QK>(raw.w, qm, 1.f));
}

// The drafter values of a chunk's run of slots [lo, hi): lane l takes the quads lo + 4 l + 256 i (a run has at most
// 1024 slots).
template <int QK>
__device__ __forceinline__ void row_q_fetch(const void *qr, int lo, int hi, int n, float4 (&qv)[4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) qv[i] = row_raw_quad<QK>(qr, lo + 4 * (lane_id() + 64 * i), hi, n);
}

// Sums over the kept ids of chunk c, in slot order: the wavefront reads back the target values it has just scattered.
// A lane past the end of the run reads the run's first quad instead (its drafter weights are zero); in the one quad that
// crosses the end, the weights of the slots past it are set to zero.
template <int QK, bool SERIES>
__device__ __forceinline__ void row_kept_sums(int c, int lo, int hi, const float4 (&qv)[4], const float *pk,
                                              const RowRcp<SERIES> &rcp, float qm, float &zq, float &tn, float &aq)
{
    const float *run = pk + row_run_start(lo, c);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (lo + 256 * i < hi) {
            const int o = 4 * (lane_id() + 64 * i);
            const int left = hi - lo - o;              // slots of the run from the lane's quad on
            const float4 p4 = *(const float4 *)(run + (left > 0 ? o : 0));
            const float4 w4 = row_weights_of<QK>(qv[i], qm);
            float qe[4] = {w4.x, w4.y, w4.z, w4.w};
            const float pe[4] = {p4.x, p4.y, p4.z, p4.w};
            if (left > 0 && left < 4) {
#pragma unroll
                for (int e = 1; e < 4; ++e) qe[e] = e < left ? qe[e] : 0.f;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                zq += qe[e];
                tn = fmaf(qe[e], pe[e], tn);
                aq = fmaf(qe[e], rcp(pe[e]), aq);
            }
        }
    }
}

// q' of Eq. 3 for the finish of a row inside the one-pass kernels (finish_row_quarters): the drafter values of the kept ids
// of a quarter chunk through the lane map, the row constants nzs and ths, and 1 / (N + p) as the block sums took it.
template <int QK, class RCP>
struct Eq3Quads {
    const uint64_t *lane_map;
    const int32_t *chunk_lo, *slot_of;
    const void *qr;
    float qm, nzs, ths;
    const RCP &rcp;
    int N;
    struct Token {
        uint64_t map;
        int lo, fq;
    };
    __device__ __forceinline__ float value(float qh, float pe) const { return (nzs * qh + ths * pe) * rcp(pe); }
    __device__ __forceinline__ Token begin(int fblk, int fq, int64_t) const
    {
        return Token{lane_map[(int64_t)fblk * kWave + lane_id()], chunk_lo[fblk], fq};
    }
    __device__ __forceinline__ void end(Token &t, int64_t fidx, const float (&pv4)[4], float (&qp4)[4]) const
    {
        const uint32_t kb = (uint32_t)(t.map >> (4 * t.fq)) & 0xFu;
        int sl = t.lo + (int)((t.map >> (16 + 12 * t.fq)) & 0xFFFu);
        float qraw[4];
        bool kept_e[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            kept_e[e] = (kb >> e) & 1u;
            qraw[e] = load1<QK>(qr, kept_e[e] ? sl : 0);   // unconditional: the loads stay batched
            sl += kept_e[e] ? 1 : 0;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float qh = kept_e[e] ? to_weight<QK>(qraw[e], qm, 1.f) : 0.f;
            qp4[e] = fidx + e < N ? value(qh, pv4[e]) : 0.f;
        }
    }
    __device__ __forceinline__ float at(int dtok, float pd_w) const
    {
        const int sg = slot_of[dtok];
        return value(sg >= 0 ? to_weight<QK>(load1<QK>(qr, sg), qm, 1.f) : 0.f, pd_w);
    }
};

// The finish of a row inside the one-pass kernels, out of the three block sums per chunk in LDS and the position's
// uniforms that the kernel left behind them (all wavefronts of the workgroup have to call it).
// pm, pinv: softmax maximum and 1 / normaliser of a logit target row (0 and 1 for probabilities).
template <int PK, int QK, class RCP>
__device__ __forceinline__ void row_finish(float *lds, int l_fin, int l_sum_q, int l_sum_r, int l_sum_a,
                                           const FinalizeArgs &fin, int64_t row, int nchunks,
                                           const void *pr, float pm, float pinv, const void *qr, float qm,
                                           const uint64_t *lane_map, const int32_t *chunk_lo, const int32_t *slot_of, int N,
                                           bool vec_p, float nzs, float ths, const RCP &rcp, int wid, int lane)
{
    const uint32_t *fw = (const uint32_t *)(lds + l_fin + kFinishFloats);
    const uint32_t words[4] = {fw[0], fw[1], fw[2], fw[3]};
    const Eq3Quads<QK, RCP> quads{lane_map, chunk_lo, slot_of, qr, qm, nzs, ths, rcp, N};
    finish_row_quarters<PK>(lds + l_fin, lds + l_sum_q, lds + l_sum_r, lds + l_sum_a, nchunks, fin, row, pr, pm, pinv, N, vec_p,
                            quads, words, wid, lane);
}

template <int QK, bool SERIES>
__global__ __launch_bounds__(kRowThreads) void taylor_row_kernel(const float *p, int64_t ldp, const void *q, int64_t ldq,
                                                                 const uint64_t *lane_map, const int32_t *chunk_lo,
                                                                 const int32_t *item_lo, const int2 *row_items, int N, int n,
                                                                 bool vec_p, const SoftStat *qstat, const int32_t *slot_of,
                                                                 FinalizeArgs fin)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int nchunks = (N + kChunk - 1) / kChunk;
    const RowLds L = row_lds_layout(n, nchunks);
    float *pk = lds + L.pk;
    int2 *il = (int2 *)(lds + L.items);
    int *ilo = (int *)(lds + L.item_lo);
    float2 *isum = (float2 *)(lds + L.isum);
    const int64_t row = blockIdx.x;
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = lane_id();
    const float *pr = p + row * ldp;
    const void *qr = row_ptr<QK>(q, ldq, row);
    const float qm = QK == RDK_PROB_F32 ? 0.f : qstat[row].m;
    const float fN = (float)N;
    RowRcp<SERIES> rcp;
    rcp.fN = fN;
    rcp.invN = 1.0f / fN;
    rcp.invN2 = rcp.invN * rcp.invN;

    // ---- the kernel's table of pieces goes to LDS (entries past the last piece are never used), the array of kept target
    // values starts at zero, and the first two chunks of every wavefront are on their way meanwhile
    const int max_items = row_max_items(n, nchunks);
    const int nitems = item_lo[nchunks];
    int2 it0 = make_int2(0, 0);
    if ((int)threadIdx.x < max_items) it0 = row_items[threadIdx.x];
    RowChunk b0, b1, b2;
    int c = wid;
    if (c < nchunks) row_fetch(pr, lane_map, chunk_lo, c, N, vec_p, b0);
    if (c + kRowWaves < nchunks) row_fetch(pr, lane_map, chunk_lo, c + kRowWaves, N, vec_p, b1);
    if (threadIdx.x == 0) {                           // the position's four uniforms (Alg. 4: draft, accept, residual, bonus)
        uint32_t words[4];
        position_words(fin.d.seed, fin.d.offset + (uint64_t)row, words);
        uint32_t *fw = (uint32_t *)(lds + L.fin + kFinishFloats);
        fw[0] = words[0]; fw[1] = words[1]; fw[2] = words[2]; fw[3] = words[3];
    }
    {
        float4 *z = (float4 *)pk;
        const int quads = (L.blk_p - L.pk) / 4;
        for (int i = threadIdx.x; i < quads; i += kRowThreads) z[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if ((int)threadIdx.x < max_items) il[threadIdx.x] = it0;
        for (int k = threadIdx.x + kRowThreads; k < max_items; k += kRowThreads) il[k] = row_items[k];
        for (int cc = threadIdx.x; cc <= nchunks; cc += kRowThreads) ilo[cc] = item_lo[cc];
    }
    __syncthreads();

    // ---- step A: one pass over the row, two chunks requested ahead of the one being worked on; the drafter values of a
    // chunk's run are requested one chunk ahead, into the registers the sums of this chunk have just freed
    float zq = 0.f, tn = 0.f, an = 0.f, ball = 0.f;   // ball: sum of p / (N + p) over all ids
    float4 qv[4];
    if (c < nchunks) row_q_fetch<QK>(qr, b0.lo, b0.hi, n, qv);
#define RDK_ROW_STEP(CUR, NEXT, FREE)                                                                        \
    {                                                                                                        \
        if (c + 2 * kRowWaves < nchunks) row_fetch(pr, lane_map, chunk_lo, c + 2 * kRowWaves, N, vec_p, FREE); \
        const int lo_c = __builtin_amdgcn_readfirstlane(CUR.lo), hi_c = __builtin_amdgcn_readfirstlane(CUR.hi); \
        float sp = 0.f, sa = 0.f, sall = 0.f, aq = 0.f;                                                      \
        row_scatter<SERIES>(CUR, c, lo_c, rcp, pk, sp, sa, sall);                                            \
        row_kept_sums<QK, SERIES>(c, lo_c, hi_c, qv, pk, rcp, qm, zq, tn, aq);                               \
        ball += sall;                                                                                        \
        an += aq;                                                                                            \
        sp = row16_sum(sp);                           /* per chunk: four partial sums, one per row of sixteen lanes */ \
        sa = row16_sum(sa);                                                                                  \
        sall = row16_sum(sall);                                                                              \
        aq = row16_sum(aq);                                                                                  \
        if ((lane & 15) == 0) {                                                                              \
            const int o = 4 * c + (lane >> 4);                                                               \
            lds[L.blk_p + o] = sp;                                                                           \
            lds[L.blk_a + o] = sa;                                                                           \
            lds[L.blk_all + o] = sall;                                                                       \
            lds[L.blk_aq + o] = aq;                                                                          \
        }                                                                                                    \
        if (c + kRowWaves < nchunks)                                                                         \
            row_q_fetch<QK>(qr, __builtin_amdgcn_readfirstlane(NEXT.lo), __builtin_amdgcn_readfirstlane(NEXT.hi), n, qv); \
        c += kRowWaves;                                                                                      \
    }
    while (c < nchunks) {
        RDK_ROW_STEP(b0, b1, b2)
        if (c >= nchunks) break;
        RDK_ROW_STEP(b1, b2, b0)
        if (c >= nchunks) break;
        RDK_ROW_STEP(b2, b0, b1)
    }
#undef RDK_ROW_STEP
    zq = wave_sum(zq);
    tn = wave_sum(tn);
    an = wave_sum(an) * fN;
    ball = wave_sum(ball);
    if (lane == 0) *(float4 *)(lds + L.red + wid * 4) = make_float4(zq, tn, an, ball);

    // ---- step C works on pieces: group g of sixteen lanes takes the pieces g, g + 64, ...; lane li of the group the slots
    // 4 li .. 4 li + 3 of the piece.  The drafter values of the first rounds are asked for here, before the barrier, and
    // so is where the lane finds its target values in LDS: a lane wholly past the end of the piece is pointed at a quad of
    // zeros; the quad that crosses the end runs into the zeros that separate the runs (a piece shorter than 64 ends its
    // run).  Where the target value is zero, q' adds nothing to either sum whatever the drafter value, so nothing needs
    // masking later.
    const int grp = threadIdx.x >> 4, li = threadIdx.x & 15;
    float4 qh[kRowHeld];
    int pat[kRowHeld];
    auto piece_of = [&](int k, int &len) {            // LDS offset of the lane's quad of piece k, and the piece's length
        const int2 it = il[k];
        len = (int)((uint32_t)it.y >> 24);
        return 4 * li < len ? L.pk + it.x - ((it.y >> 22) & 3) + 4 * (it.y & 0x3FFFFF) + 4 * li : L.zero;
    };
#pragma unroll
    for (int t = 0; t < kRowHeld; ++t) {
        const int k = grp + kRowGroups * t;
        int len = 0, first = 0;
        pat[t] = L.zero;
        if (k < nitems) {
            pat[t] = piece_of(k, len);
            first = il[k].x;
        }
        qh[t] = row_raw_quad<QK>(qr, first + 4 * li, first + len, n);
    }
    __syncthreads();
    float tot[4];
    {
        float4 t = *(const float4 *)(lds + L.red);
        for (int i = 1; i < kRowWaves; ++i) {
            const float4 o = *(const float4 *)(lds + L.red + i * 4);
            t.x += o.x; t.y += o.y; t.z += o.z; t.w += o.w;
        }
        tot[0] = t.x; tot[1] = t.y; tot[2] = t.z; tot[3] = t.w;
    }
    const float inv_zq = inv_mass(tot[0]);
    const float theta = tot[1] * inv_zq;
    const float inv_S = inv_mass(tot[2] * inv_zq + theta * tot[3]);
    const float nzs = fN * inv_zq * inv_S, ths = theta * inv_S;

    // ---- step C: max(0, p - q') and min(p, q') on the kept slots, piece by piece (the sum of q' over the kept ids of a
    // chunk needs no pass: it is nzs * sum q^ / (N + p) + ths * sum p / (N + p), both known from step A)
    auto piece_sums = [&](int k, const float4 raw, int at) {
        const float4 w4 = row_weights_of<QK>(raw, qm);
        const float4 p4 = *(const float4 *)(lds + at);
        const float qe[4] = {w4.x, w4.y, w4.z, w4.w}, pe[4] = {p4.x, p4.y, p4.z, p4.w};
        float sr = 0.f, sa = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float v = (nzs * qe[e] + ths * pe[e]) * rcp(pe[e]);
            const float m = __builtin_amdgcn_fmed3f(pe[e], v, -INFINITY);   // min(p, q'): neither is a NaN
            sa += m;
            sr += pe[e] - m;
        }
        // the sixteen lanes of the group hold the piece: four lane exchanges at register speed
        sr = row16_sum(sr);
        sa = row16_sum(sa);
        if (li == 0) isum[k] = make_float2(sr, sa);
    };
#pragma unroll
    for (int t = 0; t < kRowHeld; ++t) {
        const int k = grp + kRowGroups * t;
        if (k < nitems) piece_sums(k, qh[t], pat[t]);
    }
    for (int k = grp + kRowGroups * kRowHeld; k < nitems; k += kRowGroups) {   // more pieces than the registers were given
        int len;
        const int at = piece_of(k, len);
        const int first = il[k].x;
        piece_sums(k, row_raw_quad<QK>(qr, first + 4 * li, first + len, n), at);
    }
    __syncthreads();

    // ---- the block sums of a chunk: its pieces in order (at most sixteen: one lane each), and the closed forms
    for (int cc = grp; cc < nchunks; cc += kRowGroups) {
        const int k = ilo[cc] + li;
        const float2 f = k < ilo[cc + 1] ? isum[k] : make_float2(0.f, 0.f);
        const float sr = row16_sum(f.x), sa = row16_sum(f.y);
        if (li == 0) {
            const float4 bp = *(const float4 *)(lds + L.blk_p + 4 * cc), ba = *(const float4 *)(lds + L.blk_a + 4 * cc);
            const float4 bl = *(const float4 *)(lds + L.blk_all + 4 * cc), bq = *(const float4 *)(lds + L.blk_aq + 4 * cc);
            const float ta = ths * ((ba.x + ba.y) + (ba.z + ba.w));   // sum of q' (= sum of min(p, q')) over the not-kept ids
            lds[L.sum_q + cc] = ths * ((bl.x + bl.y) + (bl.z + bl.w)) + nzs * ((bq.x + bq.y) + (bq.z + bq.w));
            lds[L.sum_a + cc] = ta + sa;
            lds[L.sum_r + cc] = (((bp.x + bp.y) + (bp.z + bp.w)) - ta) + sr;
        }
    }
    __syncthreads();

    // ---- the finish of the row (draws, accept test), spread over the wavefronts
    row_finish<RDK_PROB_F32, QK>(lds, L.fin, L.sum_q, L.sum_r, L.sum_a, fin, row, nchunks, pr, 0.f, 1.f, qr, qm, lane_map, chunk_lo, slot_of, N, vec_p, nzs, ths, rcp,
                                 wid, lane);
}

// ------------------------------------------------------------------------------------------------
// The same for LOGIT target rows.  The softmax of the row is not known while it streams, so step A works relative to the
// maximum of each chunk: e = exp(z - chunk maximum) goes to LDS for the kept ids, and instead of sums of p and p / (N + p)
// the chunk keeps the power sums of e that their series in x = p / N need (p / (N + p) = x - x^2 + x^3 and
// N / (N + p) = 1 - x + x^2 - x^3 up to x^4 <= N^-4; used from N = 1024 on): over the not-kept ids sum e, e^2, e^3, over the
// kept ids the same and sum q^ e^k, k = 0..3.  After the barrier the row maximum is the largest chunk maximum, every
// chunk's sums are brought to it (factor exp(chunk maximum - row maximum) to the power k), their totals give the softmax
// normaliser and the row constants of Eq. 3, and steps C and the finish run as for probability rows with
// p = e * factor / normaliser.  One read of the target row instead of the three of the two-pass path (statistics, sums,
// verification sums), and one exp per id instead of two.
enum { kLgMax = 0, kLgS1n, kLgS2n, kLgS3n, kLgS1k, kLgS2k, kLgS3k, kLgQ0, kLgQ1, kLgQ2, kLgQ3, kLgScale };   // chunk statistics

// sum over the 64 lanes, valid in the lanes 48..63
__device__ __forceinline__ float wave_sum_last(float v)
{
    v = row16_sum(v);
    v += dpp_move<0x142, 0xa>(v);
    v += dpp_move<0x143, 0xc>(v);
    return v;
}

// Step A of the logit variant for one chunk: statistics to `stat` (arrays of nchunks floats), e of the kept ids to LDS.
// CUBIC = false (N >= 4096): the third-order terms of the series are below 2^-24 of the first and are left out.
template <int QK, bool CUBIC>
__device__ __forceinline__ void row_logit_chunk(const RowChunk &b, int c, int lo, int hi, const float4 (&qv)[4], float *pk,
                                                const float *zero_quad, float *stat, float qm, int nchunks)
{
    const int lane = lane_id();
    float mx = fmaxf(fmaxf(fmaxf(b.p[0].x, b.p[0].y), fmaxf(b.p[0].z, b.p[0].w)), fmaxf(fmaxf(b.p[1].x, b.p[1].y), fmaxf(b.p[1].z, b.p[1].w)));
    mx = fmaxf(mx, fmaxf(fmaxf(fmaxf(b.p[2].x, b.p[2].y), fmaxf(b.p[2].z, b.p[2].w)), fmaxf(fmaxf(b.p[3].x, b.p[3].y), fmaxf(b.p[3].z, b.p[3].w))));
    mx = fmaxf(wave_max(mx), -3.0e38f);
    const uint32_t mask = (uint32_t)b.map & 0xFFFFu;
    const int run = row_run_start(lo, c);
    float s1 = 0.f, s2 = 0.f, s3 = 0.f;                // over the ids that are not kept
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        char *at = (char *)(pk + run + (int)((b.map >> (16 + 12 * i)) & 0xFFFu));
        const float ze[4] = {b.p[i].x, b.p[i].y, b.p[i].z, b.p[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t kept = (mask >> (4 * i + e)) & 1u;
            const float ev = soft_exp(ze[e] - mx);     // ids beyond N carry -inf: zero
            if (kept) *(float *)at = ev;
            at += 4 * kept;
            const float en = kept ? 0.f : ev, en2 = en * en;
            s1 += en;
            s2 += en2;
            if (CUBIC) s3 = fmaf(en2, en, s3);
        }
    }
    float k1 = 0.f, k2 = 0.f, k3 = 0.f, q0 = 0.f, q1 = 0.f, q2 = 0.f, q3 = 0.f;   // over the kept ids, in slot order
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (lo + 256 * i < hi) {
            const int o = 4 * (lane + 64 * i);
            const int left = hi - lo - o;              // slots of the run from the lane's quad on
            const float4 e4 = *(const float4 *)(left > 0 ? pk + run + o : zero_quad);   // past the run: zeros
            const float4 w4 = row_weights_of<QK>(qv[i], qm);
            float qe[4] = {w4.x, w4.y, w4.z, w4.w};
            const float ee[4] = {e4.x, e4.y, e4.z, e4.w};
            if (left > 0 && left < 4) {
#pragma unroll
                for (int e = 1; e < 4; ++e) qe[e] = e < left ? qe[e] : 0.f;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float e2 = ee[e] * ee[e];
                k1 += ee[e];
                k2 += e2;
                q0 += qe[e];
                q1 = fmaf(qe[e], ee[e], q1);
                q2 = fmaf(qe[e], e2, q2);
                if (CUBIC) {
                    k3 = fmaf(e2, ee[e], k3);
                    q3 = fmaf(qe[e] * e2, ee[e], q3);
                }
            }
        }
    }
    s1 = wave_sum_last(s1); s2 = wave_sum_last(s2);
    k1 = wave_sum_last(k1); k2 = wave_sum_last(k2);
    q0 = wave_sum_last(q0); q1 = wave_sum_last(q1); q2 = wave_sum_last(q2);
    if (CUBIC) {
        s3 = wave_sum_last(s3); k3 = wave_sum_last(k3); q3 = wave_sum_last(q3);
    }
    if (lane == kWave - 1) {
        stat[kLgMax * nchunks + c] = mx;
        stat[kLgS1n * nchunks + c] = s1; stat[kLgS2n * nchunks + c] = s2; stat[kLgS3n * nchunks + c] = s3;
        stat[kLgS1k * nchunks + c] = k1; stat[kLgS2k * nchunks + c] = k2; stat[kLgS3k * nchunks + c] = k3;
        stat[kLgQ0 * nchunks + c] = q0; stat[kLgQ1 * nchunks + c] = q1; stat[kLgQ2 * nchunks + c] = q2;
        stat[kLgQ3 * nchunks + c] = q3;
    }
}

template <int PK, int QK, bool SERIES>
__global__ __launch_bounds__(kRowThreads) void taylor_row_logit_kernel(const void *p, int64_t ldp, const void *q, int64_t ldq,
                                                                       const uint64_t *lane_map, const int32_t *chunk_lo,
                                                                       const int32_t *item_lo, const int2 *row_items, int N, int n,
                                                                       bool vec_p, const SoftStat *qstat, const int32_t *slot_of,
                                                                       FinalizeArgs fin)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int nchunks = (N + kChunk - 1) / kChunk;
    const RowLds L = row_lds_layout(n, nchunks);
    float *pk = lds + L.pk, *stat = lds + L.blk_p;
    int2 *il = (int2 *)(lds + L.items);
    int *ilo = (int *)(lds + L.item_lo);
    float2 *isum = (float2 *)(lds + L.isum);
    const int64_t row = blockIdx.x;
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = lane_id();
    const void *pr = row_ptr<PK>(p, ldp, row);
    const void *qr = row_ptr<QK>(q, ldq, row);
    const float qm = QK == RDK_PROB_F32 ? 0.f : qstat[row].m;
    const float fN = (float)N;
    RowRcp<SERIES> rcp;
    rcp.fN = fN;
    rcp.invN = 1.0f / fN;
    rcp.invN2 = rcp.invN * rcp.invN;

    // ---- prologue: as for probability rows
    const int max_items = row_max_items(n, nchunks);
    const int nitems = item_lo[nchunks];
    int2 it0 = make_int2(0, 0);
    if ((int)threadIdx.x < max_items) it0 = row_items[threadIdx.x];
    RowChunk b0, b1, b2;
    int c = wid;
    if (c < nchunks) row_fetch<PK>(pr, lane_map, chunk_lo, c, N, vec_p, b0);
    if (c + kRowWaves < nchunks) row_fetch<PK>(pr, lane_map, chunk_lo, c + kRowWaves, N, vec_p, b1);
    if (threadIdx.x == 0) {
        uint32_t words[4];
        position_words(fin.d.seed, fin.d.offset + (uint64_t)row, words);
        uint32_t *fw = (uint32_t *)(lds + L.fin + kFinishFloats);
        fw[0] = words[0]; fw[1] = words[1]; fw[2] = words[2]; fw[3] = words[3];
    }
    {
        float4 *z = (float4 *)pk;
        const int quads = (L.blk_p - L.pk) / 4;
        for (int i = threadIdx.x; i < quads; i += kRowThreads) z[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if ((int)threadIdx.x < max_items) il[threadIdx.x] = it0;
        for (int k = threadIdx.x + kRowThreads; k < max_items; k += kRowThreads) il[k] = row_items[k];
        for (int cc = threadIdx.x; cc <= nchunks; cc += kRowThreads) ilo[cc] = item_lo[cc];
    }
    __syncthreads();

    // ---- step A
    float4 qv[4];
    if (c < nchunks) row_q_fetch<QK>(qr, b0.lo, b0.hi, n, qv);
#define RDK_ROW_STEP(CUR, NEXT, FREE)                                                                        \
    {                                                                                                        \
        if (c + 2 * kRowWaves < nchunks) row_fetch<PK>(pr, lane_map, chunk_lo, c + 2 * kRowWaves, N, vec_p, FREE); \
        const int lo_c = __builtin_amdgcn_readfirstlane(CUR.lo), hi_c = __builtin_amdgcn_readfirstlane(CUR.hi); \
        row_logit_chunk<QK, !SERIES>(CUR, c, lo_c, hi_c, qv, pk, lds + L.zero, stat, qm, nchunks);           \
        if (c + kRowWaves < nchunks)                                                                         \
            row_q_fetch<QK>(qr, __builtin_amdgcn_readfirstlane(NEXT.lo), __builtin_amdgcn_readfirstlane(NEXT.hi), n, qv); \
        c += kRowWaves;                                                                                      \
    }
    while (c < nchunks) {
        RDK_ROW_STEP(b0, b1, b2)
        if (c >= nchunks) break;
        RDK_ROW_STEP(b1, b2, b0)
        if (c >= nchunks) break;
        RDK_ROW_STEP(b2, b0, b1)
    }
#undef RDK_ROW_STEP

    // ---- the pieces of step C: drafter values, LDS offsets and chunks of the first rounds, before the barrier
    const int grp = threadIdx.x >> 4, li = threadIdx.x & 15;
    float4 qh[kRowHeld];
    int pat[kRowHeld], pch[kRowHeld];
    auto piece_of = [&](int k, int &len, int &chunk) {
        const int2 it = il[k];
        len = (int)((uint32_t)it.y >> 24);
        chunk = it.y & 0x3FFFFF;
        return 4 * li < len ? L.pk + it.x - ((it.y >> 22) & 3) + 4 * chunk + 4 * li : L.zero;
    };
#pragma unroll
    for (int t = 0; t < kRowHeld; ++t) {
        const int k = grp + kRowGroups * t;
        int len = 0, first = 0;
        pat[t] = L.zero;
        pch[t] = 0;
        if (k < nitems) {
            pat[t] = piece_of(k, len, pch[t]);
            first = il[k].x;
        }
        qh[t] = row_raw_quad<QK>(qr, first + 4 * li, first + len, n);
    }
    __syncthreads();

    // ---- the row maximum, the chunk statistics relative to it, their totals
    float pm = -INFINITY;
    for (int cc = threadIdx.x; cc < nchunks; cc += kRowThreads) pm = fmaxf(pm, stat[kLgMax * nchunks + cc]);
    pm = wave_max(pm);
    if (lane == 0) lds[L.red + wid] = pm;
    __syncthreads();
    pm = lds[L.red];
    for (int i = 1; i < kRowWaves; ++i) pm = fmaxf(pm, lds[L.red + i]);
    float t7[7] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // sum e, e^2, e^3 over all ids; sum q^ e^k, k = 0..3
    for (int cc = threadIdx.x; cc < nchunks; cc += kRowThreads) {
        const float f = soft_exp_fine(stat[kLgMax * nchunks + cc] - pm), f2 = f * f, f3 = f2 * f;   // shared by 1024 ids
        const float s1n = stat[kLgS1n * nchunks + cc] * f, s2n = stat[kLgS2n * nchunks + cc] * f2, s3n = stat[kLgS3n * nchunks + cc] * f3;
        const float s1k = stat[kLgS1k * nchunks + cc] * f, s2k = stat[kLgS2k * nchunks + cc] * f2, s3k = stat[kLgS3k * nchunks + cc] * f3;
        const float q0 = stat[kLgQ0 * nchunks + cc], q1 = stat[kLgQ1 * nchunks + cc] * f, q2 = stat[kLgQ2 * nchunks + cc] * f2;
        const float q3 = stat[kLgQ3 * nchunks + cc] * f3;
        stat[kLgS1n * nchunks + cc] = s1n; stat[kLgS2n * nchunks + cc] = s2n; stat[kLgS3n * nchunks + cc] = s3n;
        stat[kLgS1k * nchunks + cc] = s1k; stat[kLgS2k * nchunks + cc] = s2k; stat[kLgS3k * nchunks + cc] = s3k;
        stat[kLgQ1 * nchunks + cc] = q1; stat[kLgQ2 * nchunks + cc] = q2; stat[kLgQ3 * nchunks + cc] = q3;
        stat[kLgScale * nchunks + cc] = f;
        t7[0] += s1n + s1k; t7[1] += s2n + s2k; t7[2] += s3n + s3k;
        t7[3] += q0; t7[4] += q1; t7[5] += q2; t7[6] += q3;
    }
#pragma unroll
    for (int j = 0; j < 7; ++j) {
        const float v = wave_sum_last(t7[j]);
        if (lane == kWave - 1) lds[L.red + kRowWaves + wid * 8 + j] = v;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 7; ++j) t7[j] = 0.f;
    for (int i = 0; i < kRowWaves; ++i) {
        const float4 a4 = *(const float4 *)(lds + L.red + kRowWaves + i * 8), b4 = *(const float4 *)(lds + L.red + kRowWaves + i * 8 + 4);
        t7[0] += a4.x; t7[1] += a4.y; t7[2] += a4.z; t7[3] += a4.w;
        t7[4] += b4.x; t7[5] += b4.y; t7[6] += b4.z;
    }
    const float pinv = 1.0f / t7[0];                   // the row maximum itself contributes e = 1: never zero
    const float c1 = pinv / fN, c2 = c1 * c1, c3 = c2 * c1;
    const float zq = t7[3], tn = t7[4] * pinv;
    const float an = t7[3] - t7[4] * c1 + t7[5] * c2 - t7[6] * c3;     // sum q^ N / (N + p)
    const float bs = t7[0] * c1 - t7[1] * c2 + t7[2] * c3;             // sum p / (N + p)
    const float inv_zq = inv_mass(zq);
    const float theta = tn * inv_zq;
    const float inv_S = inv_mass(an * inv_zq + theta * bs);
    const float nzs = fN * inv_zq * inv_S, ths = theta * inv_S;

    // ---- step C
    auto piece_sums = [&](int k, const float4 raw, int at, int chunk) {
        const float g = stat[kLgScale * nchunks + chunk] * pinv;       // e of this chunk -> p
        const float4 w4 = row_weights_of<QK>(raw, qm);
        const float4 e4 = *(const float4 *)(lds + at);
        const float qe[4] = {w4.x, w4.y, w4.z, w4.w}, pe[4] = {e4.x * g, e4.y * g, e4.z * g, e4.w * g};
        float sr = 0.f, sa = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float v = (nzs * qe[e] + ths * pe[e]) * rcp(pe[e]);
            const float m = __builtin_amdgcn_fmed3f(pe[e], v, -INFINITY);
            sa += m;
            sr += pe[e] - m;
        }
        sr = row16_sum(sr);
        sa = row16_sum(sa);
        if (li == 0) isum[k] = make_float2(sr, sa);
    };
#pragma unroll
    for (int t = 0; t < kRowHeld; ++t) {
        const int k = grp + kRowGroups * t;
        if (k < nitems) piece_sums(k, qh[t], pat[t], pch[t]);
    }
    for (int k = grp + kRowGroups * kRowHeld; k < nitems; k += kRowGroups) {
        int len, chunk;
        const int at = piece_of(k, len, chunk);
        const int first = il[k].x;
        piece_sums(k, row_raw_quad<QK>(qr, first + 4 * li, first + len, n), at, chunk);
    }
    __syncthreads();

    // ---- the block sums of a chunk: its pieces in order, and the closed forms from the chunk's power sums.  The three
    // results take the place of the kept values in LDS (no longer needed), the statistics are read before.
    for (int cc = grp; cc < nchunks; cc += kRowGroups) {
        const int k = ilo[cc] + li;
        const float2 f = k < ilo[cc + 1] ? isum[k] : make_float2(0.f, 0.f);
        const float sr = row16_sum(f.x), sa = row16_sum(f.y);
        if (li == 0) {
            const float s1n = stat[kLgS1n * nchunks + cc], s2n = stat[kLgS2n * nchunks + cc], s3n = stat[kLgS3n * nchunks + cc];
            const float s1k = stat[kLgS1k * nchunks + cc], s2k = stat[kLgS2k * nchunks + cc], s3k = stat[kLgS3k * nchunks + cc];
            const float q0 = stat[kLgQ0 * nchunks + cc], q1 = stat[kLgQ1 * nchunks + cc], q2 = stat[kLgQ2 * nchunks + cc];
            const float q3 = stat[kLgQ3 * nchunks + cc];
            const float a_nk = s1n * c1 - s2n * c2 + s3n * c3;         // sum p / (N + p), not-kept ids
            const float a_k = s1k * c1 - s2k * c2 + s3k * c3;          //                  kept ids
            const float aq = (q0 - q1 * c1 + q2 * c2 - q3 * c3) * rcp.invN;   // sum q^ / (N + p), kept ids
            const float ta = ths * a_nk;                               // sum of q' (= sum of min(p, q')) over the not-kept ids
            lds[L.sum_q + cc] = ths * (a_nk + a_k) + nzs * aq;
            lds[L.sum_a + cc] = ta + sa;
            lds[L.sum_r + cc] = (s1n * pinv - ta) + sr;
        }
    }
    __syncthreads();

    // ---- the finish of the row (draws, accept test), spread over the wavefronts
    row_finish<PK, QK>(lds, L.fin, L.sum_q, L.sum_r, L.sum_a, fin, row, nchunks, pr, pm, pinv, qr, qm, lane_map, chunk_lo, slot_of, N, vec_p, nzs, ths, rcp, wid,
                       lane);
}

constexpr int kRowSeriesMinN = 4096;   // from here on 1 / (N + p) is taken from its series in p / N (exact to fp32 rounding)
constexpr int kRowMinBatch = 64;   // below this the two-pass kernels, which split a row over workgroups, fill the chip better

// LDS a workgroup may use on the current device (asked once).
size_t row_lds_limit()
{
    static size_t limit = 0;
    if (!limit) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0)
            limit = (size_t)v;
        else
            limit = 64 * 1024;
    }
    return limit;
}

// ------------------------------------------------------------------------------------------------
// Identity kernel: q' scattered to the kept ids, zero elsewhere (token-level intersection, Eq. 1).
template <int QK>
__global__ __launch_bounds__(kThreads) void tli_scatter_kernel(const void *q, int64_t ldq, const int32_t *slot_of, int N, int B,
                                                               const SoftStat *qstat, float *out, int64_t ldo)
{
    for (int64_t row = blockIdx.y; row < B; row += gridDim.y) {   // positions beyond the grid's second dimension are looped over
        const void *qr = row_ptr<QK>(q, ldq, row);
        const float qm = qstat[row].m, inv = inv_mass(qstat[row].s);
        for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < N; j += (int64_t)gridDim.x * kThreads) {
            const int s = slot_of[j];
            out[row * ldo + j] = s >= 0 ? to_weight<QK>(load1<QK>(qr, s), qm, 1.f) * inv : 0.f;
        }
    }
}

// c == nullptr: plain Eq. 3 into `out`.  Otherwise the fused call: verification sums per block, then the finish.
template <int PK, int QK>
rdk_status_t run_taylor(const KernelHandle &h, RowInput p, RowInput q, int32_t B, float *out, int64_t ldo, void *ws,
                        const FusedCall *c, hipStream_t st)
{
    LinearWs w = carve(h, B, ws);
    rdk_status_t rc;
    {
        // the fused call without q': one pass over the target rows, one workgroup per position, when the kept target
        // values of a row fit the LDS of a compute unit and there are enough positions to fill the chip (logit rows: from
        // the vocabulary size on at which the series of their chunk sums are exact to fp32 rounding)
        const int nchunks = (h.N + kChunk - 1) / kChunk;
        const size_t lds_bytes = (size_t)row_lds_layout(h.n, nchunks).total * sizeof(float);
        const int min_N = PK == RDK_PROB_F32 ? 2 : kOnePassMinN;
        if (c && !out && h.N >= min_N && B >= kRowMinBatch && lds_bytes <= row_lds_limit()) {
            if (QK != RDK_PROB_F32) {
                rc = launch_row_stats<QK>(q, h.n, B, 1, w.qstat, st);
                if (rc != RDK_OK) return rc;
            }
            const bool vec_p = rows_vectorisable(p.ptr, p.ld, p.kind);
            if (q.kind != RDK_LOGIT_BF16 && ((uintptr_t)q.ptr % 4 != 0)) return RDK_ERR_ALIGN;
            static bool attr_set = false;     // per instantiation: dynamic LDS above the default limit has to be granted once
            if (!attr_set) {
                if constexpr (PK == RDK_PROB_F32) {
                    RDK_HIP(hipFuncSetAttribute((const void *)taylor_row_kernel<QK, true>,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)row_lds_limit()));
                    RDK_HIP(hipFuncSetAttribute((const void *)taylor_row_kernel<QK, false>,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)row_lds_limit()));
                } else {
                    RDK_HIP(hipFuncSetAttribute((const void *)taylor_row_logit_kernel<PK, QK, true>,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)row_lds_limit()));
                    RDK_HIP(hipFuncSetAttribute((const void *)taylor_row_logit_kernel<PK, QK, false>,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)row_lds_limit()));
                }
                attr_set = true;
            }
            FinalizeArgs fa{};                // the block sums stay in the workgroup's LDS
            fa.d = c->d;
            fa.p = p.ptr; fa.ldp = p.ld; fa.vec_p = vec_p;
            fa.pstat = w.pstat; fa.p_splits = w.p_splits;
            fa.nblk = nchunks;
            fa.draft_ids = c->draft_ids; fa.accept = c->accept; fa.alpha = c->alpha; fa.resid_mass = c->resid_mass;
            fa.resid_ids = c->resid_ids; fa.n_accepted = c->n_accepted; fa.out_tokens = c->out_tokens;
            const bool series = h.N >= kRowSeriesMinN;
#define RDK_ROW_LAUNCH(KERNEL, PPTR)                                                                                        \
    RDK_TIMED_LAUNCH("taylor_row_kernel", KERNEL, dim3((unsigned)B), dim3(kRowThreads), lds_bytes, st, PPTR, p.ld, q.ptr, q.ld,  \
                     h.lane_map, h.chunk_lo, h.item_lo, h.row_items, h.N, h.n, vec_p, w.qstat, h.slot_of, fa)
            if constexpr (PK == RDK_PROB_F32) {
                if (series) RDK_ROW_LAUNCH((taylor_row_kernel<QK, true>), (const float *)p.ptr);
                else RDK_ROW_LAUNCH((taylor_row_kernel<QK, false>), (const float *)p.ptr);
            } else {
                if (series) RDK_ROW_LAUNCH((taylor_row_logit_kernel<PK, QK, true>), p.ptr);
                else RDK_ROW_LAUNCH((taylor_row_logit_kernel<PK, QK, false>), p.ptr);
            }
#undef RDK_ROW_LAUNCH
            RDK_LAUNCH_CHECK("taylor_row_kernel");
            if (c->d.gamma > 0 && (fa.n_accepted || fa.out_tokens))
                return launch_sequence_scan(c->d, fa.draft_ids, fa.accept, fa.resid_ids, fa.n_accepted, fa.out_tokens, st);
            return RDK_OK;
        }
    }
    // logit target rows of a large vocabulary: the first pass of Eq. 3 also delivers the softmax statistics
    const bool onepass = PK != RDK_PROB_F32 && h.N >= kOnePassMinN;
    if (PK != RDK_PROB_F32 && !onepass) {
        rc = launch_row_stats<PK>(p, h.N, B, w.p_splits, w.pstat, st);
        if (rc != RDK_OK) return rc;
    }
    if (QK != RDK_PROB_F32) {
        rc = launch_row_stats<QK>(q, h.n, B, 1, w.qstat, st);
        if (rc != RDK_OK) return rc;
    }
    TaylorArgs a;
    a.p = p.ptr; a.q = q.ptr; a.ldp = p.ld; a.ldq = q.ld;
    a.slot_of = h.slot_of; a.kept = h.kept_ids; a.chunk_lo = h.chunk_lo; a.N = h.N; a.n = h.n; a.splits = w.t_splits;
    a.vec_p = rows_vectorisable(p.ptr, p.ld, p.kind);
    a.vec_q = rows_vectorisable(q.ptr, q.ld, q.kind);
    a.onepass = onepass;
    a.w = w;
    const bool vec_o = out ? rows_vectorisable(out, ldo, RDK_PROB_F32) : false;
    // first pass: one-pass or two-pass statistics; in the fused call (c != NULL) it leaves the target rows cacheable
    const dim3 grid((unsigned)B * w.t_splits);
#define RDK_LAUNCH_STATS(KERNEL)                                                                                         \
    RDK_TIMED_LAUNCH("taylor_stats_kernel", KERNEL, grid, dim3(kThreads), 0, st, p.ptr, p.ld, q.ptr, q.ld, h.kept_ids,  \
                     h.chunk_lo, h.N, h.n, w.t_splits, a.vec_p, a.vec_q, w)
    bool launched = false;
    if constexpr (PK != RDK_PROB_F32) {
        if (onepass) {
            if (c) RDK_LAUNCH_STATS((taylor_stats_onepass_kernel<PK, QK, true>));
            else RDK_LAUNCH_STATS((taylor_stats_onepass_kernel<PK, QK, false>));
            launched = true;
        }
    }
    if (!launched) {
        if (c) RDK_LAUNCH_STATS((taylor_stats_kernel<PK, QK, true>));
        else RDK_LAUNCH_STATS((taylor_stats_kernel<PK, QK, false>));
    }
#undef RDK_LAUNCH_STATS
    RDK_LAUNCH_CHECK("taylor_stats_kernel");
    if (!c) {
        {
            RDK_TIMED_LAUNCH("taylor_write_kernel", (taylor_write_kernel<PK, QK, false>), grid, dim3(kThreads), 0, st, a, vec_o,
                             out, ldo, (float *)nullptr, (float *)nullptr, (float *)nullptr);
        }
        RDK_LAUNCH_CHECK("taylor_write_kernel");
        return RDK_OK;
    }
    const int nchunks = (h.N + kChunk - 1) / kChunk;
    const size_t per = align_up((size_t)B * nchunks * sizeof(float), 256);
    char *pp = (char *)ws + taylor_workspace_bytes(h, B);
    float *part_q = (float *)pp, *part_r = (float *)(pp + per), *part_a = (float *)(pp + 2 * per);
    {
        RDK_TIMED_LAUNCH("taylor_write_kernel", (taylor_write_kernel<PK, QK, true>), grid, dim3(kThreads), 0, st, a, vec_o, out,
                         ldo, part_q, part_r, part_a);
    }
    RDK_LAUNCH_CHECK("taylor_write_kernel");
    FinalizeArgs fa{};
    fa.d = c->d;
    fa.p = p.ptr; fa.ldp = p.ld; fa.vec_p = a.vec_p;
    fa.pstat = w.pstat; fa.p_splits = w.p_splits;
    fa.part_q = part_q; fa.part_r = part_r; fa.part_a = part_a;
    fa.nblk = nchunks;
    fa.draft_ids = c->draft_ids; fa.accept = c->accept; fa.alpha = c->alpha; fa.resid_mass = c->resid_mass;
    fa.resid_ids = c->resid_ids; fa.n_accepted = c->n_accepted; fa.out_tokens = c->out_tokens;
    return launch_finalize<PK, 1024, true, QpTaylor<PK, QK>>(fa, QpTaylor<PK, QK>{a}, st);
}

template <int QK>
rdk_status_t run_tli(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws, hipStream_t st)
{
    LinearWs w = carve(h, B, ws);
    rdk_status_t rc = launch_row_stats<QK>(q, h.n, B, 1, w.qstat, st);
    if (rc != RDK_OK) return rc;
    const int bx = (h.N + kThreads * 4 - 1) / (kThreads * 4);
    {
        RDK_TIMED_LAUNCH("tli_scatter_kernel", (tli_scatter_kernel<QK>), dim3(bx, B < 32768 ? B : 32768), dim3(kThreads), 0, st, q.ptr,
                         q.ld, h.slot_of, h.N, B, w.qstat, out, ldo);
    }
    RDK_LAUNCH_CHECK("tli_scatter_kernel");
    return RDK_OK;
}

}  // namespace

size_t taylor_workspace_bytes(const KernelHandle &h, int32_t B)
{
    const int splits = row_splits(B, h.N, kWaves);
    return align_up((size_t)B * splits * sizeof(SoftStat), 256) + align_up((size_t)B * sizeof(SoftStat), 256) +
           align_up((size_t)B * splits * 8 * sizeof(float), 256);
}

size_t taylor_fused_workspace_bytes(const KernelHandle &h, int32_t B)
{
    const int nchunks = (h.N + kChunk - 1) / kChunk;
    return taylor_workspace_bytes(h, B) + 3 * align_up((size_t)B * nchunks * sizeof(float), 256);
}

rdk_status_t launch_taylor(const KernelHandle &h, RowInput p, RowInput q, int32_t B, float *out, int64_t ldo, void *ws,
                           const FusedCall *c, hipStream_t st)
{
#define RDK_T(PK, QK) \
    if (p.kind == PK && q.kind == QK) return run_taylor<PK, QK>(h, p, q, B, out, ldo, ws, c, st);
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

rdk_status_t launch_tli_scatter(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws, hipStream_t st)
{
    switch (q.kind) {
        case RDK_PROB_F32: return run_tli<RDK_PROB_F32>(h, q, B, out, ldo, ws, st);
        case RDK_LOGIT_F32: return run_tli<RDK_LOGIT_F32>(h, q, B, out, ldo, ws, st);
        case RDK_LOGIT_BF16: return run_tli<RDK_LOGIT_BF16>(h, q, B, out, ldo, ws, st);
    }
    return RDK_ERR_DTYPE;
}

}  // namespace rdk
