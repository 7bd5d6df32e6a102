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
#include <mutex>

#include "rdk_finalize.hpp"

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
        float4 pv[4], qv[4];
        load_chunk<KIND>(pr, (int64_t)c * kChunk, N, vec_p, pfill, pv);
        if (HAS_Q) load_chunk<RDK_PROB_F32>(qr, (int64_t)c * kChunk, N, vec_q, 0.f, qv);
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

}  // namespace

// Per-sequence scan as a launch of its own (sequences longer than one workgroup's waves).
__global__ void sequence_scan_kernel(int S, int gamma, const int32_t *draft_ids, const uint8_t *accept,
                                     const int32_t *resid_ids, int32_t *n_accepted, int32_t *out_tokens)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= S) return;
    const int64_t b0 = (int64_t)s * gamma;
    // flags are read eight at a time so that the loads of a group are in flight together (one round trip per group
    // instead of one per draft position)
    int j = gamma;
    for (int g0 = 0; g0 < gamma && j == gamma; g0 += 8) {
        uint8_t f[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) f[t] = g0 + t < gamma ? accept[b0 + g0 + t] : (uint8_t)0;
#pragma unroll
        for (int t = 7; t >= 0; --t)
            if (g0 + t < gamma && !f[t]) j = g0 + t;   // the lowest rejected position of the group wins
    }
    if (n_accepted) n_accepted[s] = j;
    if (out_tokens) {
        int32_t *o = out_tokens + (int64_t)s * (gamma + 1);
        const int32_t resid = j < gamma ? resid_ids[b0 + j] : -1;
        for (int i0 = 0; i0 <= gamma; i0 += 8) {
            int32_t d[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) d[t] = i0 + t < j ? draft_ids[b0 + i0 + t] : -1;
#pragma unroll
            for (int t = 0; t < 8; ++t)
                if (i0 + t <= gamma) o[i0 + t] = i0 + t < j ? d[t] : (i0 + t == j && j < gamma) ? resid : -1;
        }
    }
}

namespace {

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
        RDK_TIMED_LAUNCH("verify_stream_kernel", (verify_stream_kernel<KIND, HAS_Q>), dim3((unsigned)d.B * splits),
                         dim3(kStreamThreads), 0, st, p.ptr, p.ld, q, ldq, d.N, splits, vec_p, vec_q, w);
    }
    RDK_LAUNCH_CHECK("verify_stream_kernel");
    FinalizeArgs fa{};
    fa.d = d;
    fa.p = p.ptr; fa.ldp = p.ld; fa.vec_p = vec_p;
    fa.pstat = w.pstat; fa.p_splits = w.stat_splits;
    fa.part_q = w.part_q; fa.part_r = w.part_r; fa.part_a = w.part_a;
    fa.nblk = w.nchunks;
    fa.draft_ids = draft_ids; fa.accept = accept; fa.alpha = alpha; fa.resid_mass = resid_mass;
    fa.resid_ids = resid_ids; fa.n_accepted = n_accepted; fa.out_tokens = out_tokens;
    QpMemory qp{q, ldq, vec_q, d.N};
    return launch_finalize<KIND, 1024, HAS_Q, QpMemory>(fa, qp, st);
}

// Sums of each 1024-id block of materialised rows (the draft draw from a q' that sits in memory).
__global__ __launch_bounds__(kStreamThreads) void row_block_sums_kernel(const float *q, int64_t ldq, int N, int nchunks, int splits,
                                                                        bool vec_q, float *part_q)
{
    const int64_t row = blockIdx.x / splits;
    const int split = blockIdx.x % splits;
    const int cpw = (nchunks + splits - 1) / splits;
    const int c_begin = split * cpw, c_end = min(nchunks, c_begin + cpw);
    const float *qr = q + row * ldq;
    const int wid = threadIdx.x / kWave, lane = lane_id();
    for (int c = c_begin + wid; c < c_end; c += kWavesPerBlock) {
        float4 qv[4];
        load_chunk<RDK_PROB_F32>(qr, (int64_t)c * kChunk, N, vec_q, 0.f, qv);
        float sq = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) sq += (qv[i].x + qv[i].y) + (qv[i].z + qv[i].w);
        sq = wave_sum(sq);
        if (lane == 0) part_q[row * nchunks + c] = sq;
    }
}

}  // namespace

size_t draft_rows_workspace_bytes(int32_t B, int32_t N) { return align_up((size_t)B * chunks_of(N) * sizeof(float), 256); }

rdk_status_t launch_draft_from_rows(const float *q_prime, int64_t ldq, int32_t B, int32_t N, uint64_t seed, uint64_t offset,
                                    int32_t *draft_ids, float *q_draft, void *ws, hipStream_t st)
{
    const int nchunks = chunks_of(N);
    const int splits = row_splits(B, N, kWavesPerBlock);
    const bool vec_q = rows_vectorisable(q_prime, ldq, RDK_PROB_F32);
    float *part_q = (float *)ws;
    RDK_TIMED_LAUNCH("row_block_sums_kernel", row_block_sums_kernel, dim3((unsigned)B * splits), dim3(kStreamThreads), 0, st,
                     q_prime, ldq, N, nchunks, splits, vec_q, part_q);
    RDK_LAUNCH_CHECK("row_block_sums_kernel");
    DraftArgs a{B, N, seed, offset, part_q, nchunks, draft_ids, q_draft};
    return launch_draft_finalize<1024, QpMemory>(a, QpMemory{q_prime, ldq, vec_q, N}, st);
}

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

// ---- verification without a caller workspace: the scratch of the two kernels lives in a device array of this
// library, one copy per GPU, held until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

size_t verify_static_scratch_limit() { return kStaticScratchBytes; }

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up once per GPU
}  // namespace

rdk_status_t launch_verify_static(const rdk_verify_desc_t &d, RowInput p, const float *q_prime, int64_t ldq, int32_t *draft_ids,
                                  uint8_t *accept, float *alpha, float *resid_mass, int32_t *resid_ids, int32_t *n_accepted,
                                  int32_t *out_tokens, hipStream_t st)
{
    if (verify_workspace_bytes(d) > kStaticScratchBytes) return RDK_ERR_WORKSPACE;
    int dev = -1;
    RDK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return RDK_ERR_UNSUPPORTED;
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            // the array's name is a host-side handle, not a device address: every use below goes through `ptr`
            void *sym = nullptr;
            RDK_HIP(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
            if (!sym) return RDK_ERR_HIP;
            g_scratch_ptr[dev] = sym;
        }
        ptr = g_scratch_ptr[dev];
    }
    // nothing in the scratch has to start at zero: the streaming pass writes every block sum the finish step reads
    return launch_verify(d, p, q_prime, ldq, draft_ids, accept, alpha, resid_mass, resid_ids, n_accepted, out_tokens, ptr, st);
}

rdk_status_t launch_sequence_scan(const rdk_verify_desc_t &d, const int32_t *draft_ids, const uint8_t *accept,
                                  const int32_t *resid_ids, int32_t *n_accepted, int32_t *out_tokens, hipStream_t st)
{
    const int S = d.B / d.gamma;
    {
        RDK_TIMED_LAUNCH("sequence_scan_kernel", sequence_scan_kernel, dim3((S + 63) / 64), dim3(64), 0, st, S, d.gamma,
                         draft_ids, accept, resid_ids, n_accepted, out_tokens);
    }
    RDK_LAUNCH_CHECK("sequence_scan_kernel");
    return RDK_OK;
}

rdk_status_t launch_philox_words(uint64_t seed, uint64_t offset, int32_t count, uint32_t *words, hipStream_t st)
{
    hipLaunchKernelGGL(philox_words_kernel, dim3((count + 255) / 256), dim3(256), 0, st, seed, offset, count, words);
    RDK_LAUNCH_CHECK("philox_words_kernel");
    return RDK_OK;
}

}  // namespace rdk
