// Verification of several candidates per position.  The paper's introduction names multi-candidate (tree)
// verification among the related work only; the steps are those of the method cited there (multi-step speculative
// sampling, Miao et al., "SpecInfer", 2024) with the redistributed drafter q' in the drafter's place:
//   r <- p;  for i = 0 .. C-1:  x_i ~ q' (or the caller's);  keep x_i with probability min(1, r(x_i) / q'(x_i)) and stop,
//   else  r <- normalize(max(0, r - q'));  nothing kept: t ~ r.
// With C = 1 these are steps 2 and 6-8 of Alg. 4.  A position may hold fewer than C candidates (a negative id ends its
// list; none at all: t ~ p), which is what the nodes of a token tree need: verifying every node with its children as
// candidates and then following the kept children from the root (tree_walk_kernel) verifies the tree.
//
// The residual is never stored.  Because q' >= 0,  max(0, max(0, x) - q') = max(0, x - q'),  so after i rejections
//   r_i(j) = max(0, ca * p(j) - cb * q'(j))   with  (ca, cb) = (1, 0)  and  (ca, cb) <- (ca, cb + 1) / Z,
// Z = sum_j max(0, ca * p(j) - (cb + 1) * q'(j)) being the mass that the rejection leaves.  One workgroup owns one
// position: every rejection costs one pass over the two rows (HBM-bound: 8 bytes per id), whose 1024-id block sums
// stay in LDS; they give Z (added in fp64) and, after the last rejection, the block of the final draw, which is then
// re-read and scanned in fp64.  The candidates are drawn the same way from the block sums of q'.
#include "rdk_finalize.hpp"

namespace rdk {

namespace {

constexpr int kMultiThreads = 1024;
constexpr int kMultiWaves = kMultiThreads / kWave;
constexpr int kMultiMaxBlocks = 2048;      // 1024-id blocks of a row held in LDS
constexpr int kMultiMaxCandidates = 16;

struct MultiArgs {
    rdk_multi_desc_t d;
    const void *p;
    int64_t ldp;
    bool vec_p;
    const float *q;
    int64_t ldq;
    bool vec_q;
    const SoftStat *pstat;   // [B, p_splits] (logit p only)
    int p_splits;
    int32_t *cand_ids, *accepted, *token;
    float *resid_mass;       // [B, C] or NULL
};

// The m-th uniform of a position: word m % 4 of the Philox block with counter (index, m / 4, 0).
__device__ __forceinline__ double multi_unit(uint64_t seed, uint64_t index, int m)
{
    uint32_t w[4];
    philox4x32_10((uint32_t)index, (uint32_t)(index >> 32), (uint32_t)(m / 4), 0u, (uint32_t)seed, (uint32_t)(seed >> 32), w);
    const uint32_t pick = (m % 4) == 0 ? w[0] : (m % 4) == 1 ? w[1] : (m % 4) == 2 ? w[2] : w[3];
    return word_to_unit(pick);
}

// Weight of one id in the pass with coefficients (ca, cb): the drafter row itself (RESID = false) or the residual.
template <bool RESID>
__device__ __forceinline__ float multi_weight(float pe, float qe, float ca, float cb)
{
    return RESID ? fmaxf(pe * ca - qe * cb, 0.f) : qe;
}

template <int KIND>
struct MultiRow {
    const void *pr;
    const float *qr;
    int N;
    bool vec_p, vec_q;
    float m, inv, pfill;

    // block sums of the weights into LDS (all wavefronts), ends with a barrier
    // (WITH_Q = false: the drafter row is not read and counts as zero -- the pass over p alone of a leaf)
    template <bool RESID, bool WITH_Q = true>
    __device__ __forceinline__ void pass(float *blk, int nblk, float ca, float cb) const
    {
        const int wid = threadIdx.x / kWave, lane = lane_id();
        for (int c = wid; c < nblk; c += kMultiWaves) {
            float4 pv[4], qv[4];
            if (RESID) load_chunk<KIND, false>(pr, (int64_t)c * kChunk, N, vec_p, pfill, pv);
            if (WITH_Q) {
                load_chunk<RDK_PROB_F32, false>(qr, (int64_t)c * kChunk, N, vec_q, 0.f, qv);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) qv[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float qe[4] = {qv[i].x, qv[i].y, qv[i].z, qv[i].w};
                float pe[4] = {0.f, 0.f, 0.f, 0.f};
                if (RESID) {
                    pe[0] = to_weight<KIND>(pv[i].x, m, inv); pe[1] = to_weight<KIND>(pv[i].y, m, inv);
                    pe[2] = to_weight<KIND>(pv[i].z, m, inv); pe[3] = to_weight<KIND>(pv[i].w, m, inv);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) s += multi_weight<RESID>(pe[e], qe[e], ca, cb);
            }
            s = wave_sum(s);
            if (lane == 0) blk[c] = s;
        }
        __syncthreads();
    }

    // one wavefront: inverse-CDF draw from the weights whose block sums are in blk; `total` = their fp64 sum
    template <bool RESID>
    __device__ __forceinline__ int draw(const float *blk, int nblk, int per_lane, double lane_sum, double total, double u,
                                        float ca, float cb) const
    {
        if (!(total > 0.0)) return -1;
        const double thr = u * total;
        double before = 0.0;
        const int b = locate_block(blk, nblk, per_lane, lane_sum, thr, before);
        if (b < 0) return -1;
        const int lane = lane_id();
        float4 w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t idx = (int64_t)b * kChunk + i * 256 + lane * 4;
            const float4 q4 = load4<RDK_PROB_F32>(qr, idx, N, vec_q, 0.f);
            float4 p4 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (RESID) {
                const float4 raw = load4<KIND>(pr, idx, N, vec_p, pfill);
                p4 = make_float4(to_weight<KIND>(raw.x, m, inv), to_weight<KIND>(raw.y, m, inv), to_weight<KIND>(raw.z, m, inv),
                                 to_weight<KIND>(raw.w, m, inv));
            }
            w[i] = make_float4(multi_weight<RESID>(p4.x, q4.x, ca, cb), multi_weight<RESID>(p4.y, q4.y, ca, cb),
                               multi_weight<RESID>(p4.z, q4.z, ca, cb), multi_weight<RESID>(p4.w, q4.w, ca, cb));
        }
        return search_block<4>(w, b * kChunk, thr - before);
    }
};

template <int KIND>
__global__ __launch_bounds__(kMultiThreads) void verify_multi_kernel(MultiArgs a)
{
    __shared__ float blk[kMultiMaxBlocks];
    __shared__ int32_t sh_cand[kMultiMaxCandidates];
    __shared__ float sh_px[kMultiMaxCandidates], sh_qx[kMultiMaxCandidates];
    __shared__ double sh_u[kMultiMaxCandidates];
    __shared__ double sh_total;
    const int64_t row = blockIdx.x;
    const int wid = threadIdx.x / kWave, lane = lane_id();
    const int N = a.d.N, C = a.d.C;
    const int nblk = (N + kChunk - 1) / kChunk;
    const int per_lane = ((nblk + kWave - 1) / kWave + 3) & ~3;
    const uint64_t index = a.d.offset + (uint64_t)row;
    MultiRow<KIND> r;
    r.pr = row_ptr<KIND>(a.p, a.ldp, row);
    r.qr = a.q + row * a.ldq;
    r.N = N;
    r.vec_p = a.vec_p;
    r.vec_q = a.vec_q;
    r.m = 0.f;
    r.inv = 1.f;
    if (KIND != RDK_PROB_F32) {
        const SoftStat rs = merged_row_stat<KIND>(a.pstat, a.p_splits, row);
        r.m = rs.m;
        r.inv = 1.0f / rs.s;
    }
    r.pfill = KIND == RDK_PROB_F32 ? 0.f : -INFINITY;
    if (a.resid_mass && threadIdx.x < C) a.resid_mass[row * C + threadIdx.x] = 0.f;

    // the candidates: drawn from q' (uniforms 0 .. C-1), or the caller's
    if (a.d.sample_candidates) {
        r.template pass<false>(blk, nblk, 0.f, 0.f);
        if (wid == 0) {
            const double lane_sum = lane_partial_sum(blk, nblk, per_lane);
            const double total = wave_sum(lane_sum);
            for (int i = 0; i < C; ++i) {
                const int x = r.template draw<false>(blk, nblk, per_lane, lane_sum, total, multi_unit(a.d.seed, index, i), 0.f, 0.f);
                if (lane == 0) {
                    sh_cand[i] = x;
                    a.cand_ids[row * C + i] = x;
                }
            }
        }
    } else if (threadIdx.x < C) {
        sh_cand[threadIdx.x] = a.cand_ids[row * C + threadIdx.x];
    }
    __syncthreads();
    // both rows at every candidate and the uniforms of the tests, fetched together (one round trip instead of one per
    // round); a candidate beyond the vocabulary gets zero weights and is never kept (u * 0 < 0 is false); a negative
    // id ends the list of the position
    if (threadIdx.x < C) {
        const int x = sh_cand[threadIdx.x];
        const bool valid = x >= 0 && x < N;
        sh_px[threadIdx.x] = valid ? to_weight<KIND>(load1<KIND>(r.pr, valid ? x : 0), r.m, r.inv) : 0.f;
        sh_qx[threadIdx.x] = valid ? r.qr[x] : 0.f;
        sh_u[threadIdx.x] = multi_unit(a.d.seed, index, C + threadIdx.x);
    }
    __syncthreads();

    float ca = 1.f, cb = 0.f;   // r_i = max(0, ca p - cb q')
    float wa = 1.f, wb = 1.f;   // coefficients of the last pass
    int accepted = C, token = -1;
    double Z = 0.0;
    bool any_pass = false;
    for (int i = 0; i < C; ++i) {
        if (sh_cand[i] < 0) break;   // end of the list: the same for every thread
        const float rho = fmaxf(sh_px[i] * ca - sh_qx[i] * cb, 0.f);
        if (sh_u[i] * (double)sh_qx[i] < (double)rho) {   // the same for every thread
            accepted = i;
            token = sh_cand[i];
            break;
        }
        wa = ca;
        wb = cb + 1.f;
        r.template pass<true>(blk, nblk, wa, wb);
        any_pass = true;
        if (wid == 0) {
            const double total = wave_sum(lane_partial_sum(blk, nblk, per_lane));
            if (lane == 0) {
                sh_total = total;
                if (a.resid_mass) a.resid_mass[row * C + i] = (float)total;
            }
        }
        __syncthreads();
        Z = sh_total;
        if (Z > 0.0) {
            ca = (float)((double)wa / Z);
            cb = (float)((double)wb / Z);
        } else {   // nothing is left of the target row: no later candidate can be kept
            ca = 0.f;
            cb = 0.f;
        }
        __syncthreads();   // sh_total is written again in the next round
    }
    if (accepted == C && !any_pass) {
        // a position without candidates (a leaf of a token tree): t ~ p, the residual with nothing taken off
        wa = 1.f;
        wb = 0.f;
        r.template pass<true, false>(blk, nblk, wa, wb);
    }
    if (accepted == C && wid == 0) {
        // every candidate was rejected: t ~ r, whose un-normalised weights are those of the last pass
        const double lane_sum = lane_partial_sum(blk, nblk, per_lane);
        const double total = any_pass ? Z : wave_sum(lane_sum);
        token = r.template draw<true>(blk, nblk, per_lane, lane_sum, total, multi_unit(a.d.seed, index, 2 * C), wa, wb);
    }
    if (threadIdx.x == 0) {
        a.accepted[row] = accepted;
        a.token[row] = token;
    }
}

// Walk through verified token trees: one thread per tree follows, from the root, the candidate that the verification
// of each node kept, and emits that node's token; it stops at the first node that kept none (integer work only).
__global__ void tree_walk_kernel(int S, int nodes, int C, const int32_t *child_node, const int32_t *accepted,
                                 const int32_t *token, int32_t *n_accepted, int32_t *out_tokens)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= S) return;
    int32_t *out = out_tokens + (int64_t)s * nodes;
    int v = 0, len = 0;
    while (len < nodes) {
        const int64_t pos = (int64_t)s * nodes + v;
        out[len++] = token[pos];
        const int kept = accepted[pos];
        if (kept < 0 || kept >= C) break;
        const int next = child_node[pos * C + kept];
        if (next <= v || next >= nodes) break;   // not a tree: stop rather than loop
        v = next;
    }
    n_accepted[s] = len - 1;
    for (int i = len; i < nodes; ++i) out[i] = -1;
}

template <int KIND>
rdk_status_t run_multi(MultiArgs a, RowInput p, void *ws, hipStream_t st)
{
    if (KIND != RDK_PROB_F32) {
        a.p_splits = row_splits(a.d.B, a.d.N, kStatThreads / kWave);
        a.pstat = (SoftStat *)ws;
        rdk_status_t rc = launch_row_stats<KIND>(p, a.d.N, a.d.B, a.p_splits, (SoftStat *)ws, st);
        if (rc != RDK_OK) return rc;
    }
    {
        RDK_TIMED_LAUNCH("verify_multi_kernel", (verify_multi_kernel<KIND>), dim3((unsigned)a.d.B), dim3(kMultiThreads), 0, st, a);
    }
    RDK_LAUNCH_CHECK("verify_multi_kernel");
    return RDK_OK;
}

}  // namespace

int multi_max_ids() { return kMultiMaxBlocks * kChunk; }
int multi_max_candidates() { return kMultiMaxCandidates; }

size_t multi_workspace_bytes(const rdk_multi_desc_t &d, rdk_input_kind_t p_kind)
{
    if (p_kind == RDK_PROB_F32) return 256;
    return align_up((size_t)d.B * row_splits(d.B, d.N, kStatThreads / kWave) * sizeof(SoftStat), 256);
}

rdk_status_t launch_tree_walk(int32_t S, int32_t nodes, int32_t C, const int32_t *child_node, const int32_t *accepted,
                              const int32_t *token, int32_t *n_accepted, int32_t *out_tokens, hipStream_t st)
{
    {
        RDK_TIMED_LAUNCH("tree_walk_kernel", tree_walk_kernel, dim3((S + 63) / 64), dim3(64), 0, st, S, nodes, C, child_node,
                         accepted, token, n_accepted, out_tokens);
    }
    RDK_LAUNCH_CHECK("tree_walk_kernel");
    return RDK_OK;
}

rdk_status_t launch_verify_multi(const rdk_multi_desc_t &d, RowInput p, const float *q_prime, int64_t ldq, int32_t *cand_ids,
                                 int32_t *accepted, int32_t *token, float *resid_mass, void *ws, hipStream_t st)
{
    MultiArgs a{};
    a.d = d;
    a.p = p.ptr; a.ldp = p.ld; a.vec_p = rows_vectorisable(p.ptr, p.ld, p.kind);
    a.q = q_prime; a.ldq = ldq; a.vec_q = rows_vectorisable(q_prime, ldq, RDK_PROB_F32);
    a.cand_ids = cand_ids; a.accepted = accepted; a.token = token; a.resid_mass = resid_mass;
    switch (p.kind) {
        case RDK_PROB_F32: return run_multi<RDK_PROB_F32>(a, p, ws, st);
        case RDK_LOGIT_F32: return run_multi<RDK_LOGIT_F32>(a, p, ws, st);
        case RDK_LOGIT_BF16: return run_multi<RDK_LOGIT_BF16>(a, p, ws, st);
    }
    return RDK_ERR_DTYPE;
}

}  // namespace rdk
