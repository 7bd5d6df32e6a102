// Per-row finish of the verification step (Alg. 4, steps 2 and 4-10), shared by the stand-alone
// verify call and by the fused redistribute+verify calls.
//
// Input: for every row three partial sums per block of BLOCK ids (sum q', sum max(0, p - q'),
// sum min(p, q')), written by a streaming pass.  One wavefront per row (small batches; large ones spread the same
// steps over four or eight wavefronts, see verify_finalize_wide_kernel and finish_row_quarters) then
//   1. adds the partials in fp64 (alpha, residual mass, sum q'), draws the Philox uniforms,
//   2. finds the blocks in which the two inverse-CDF thresholds are crossed,
//   3. re-reads (or re-computes) those blocks and scans them in fp64 for the exact ids,
//   4. decides acceptance in fp64, and, when a workgroup holds one whole sequence, runs the
//      first-rejection scan.
// Where q' comes from is the `QP` policy: memory (a materialised q' row) or a formula.  A policy hands out q' of
// four consecutive ids in kStages steps on a `Pending` record, each step issuing the loads whose addresses the
// step before produced; the kernel runs step k for ALL blocks it needs before step k + 1, so a chain of dependent
// loads costs kStages round trips in total rather than per block.
#pragma once
#include "rdk_rowstats.hpp"

namespace rdk {

struct FinalizeArgs {
    rdk_verify_desc_t d;
    const void *p;
    int64_t ldp;
    bool vec_p;
    const SoftStat *pstat;   // [B, p_splits] (logit p only)
    int p_splits;
    const float *part_q, *part_r, *part_a;   // [B, nblk]
    int nblk;
    int rows_per_block;
    bool scan_here;
    int32_t *draft_ids;
    uint8_t *accept;
    float *alpha, *resid_mass;
    int32_t *resid_ids, *n_accepted, *out_tokens;
};

// q' read back from memory.
struct QpMemory {
    static constexpr bool kSpreadRows = false;
    static constexpr int kStages = 1;
    const float *q;
    int64_t ldq;
    bool vec;
    int N;
    struct Row {
        const float *qr;
        bool vec;
        int N;
        struct Pending {
            float4 v;
        };
        template <int K>
        __device__ __forceinline__ void stage(Pending &t, int64_t idx) const
        {
            t.v = rdk::load4<RDK_PROB_F32>(qr, idx, N, vec, 0.f);
        }
        __device__ __forceinline__ float4 result(Pending &t, int64_t) const { return t.v; }
        __device__ __forceinline__ float load1(int j) const { return qr[j]; }
    };
    __device__ __forceinline__ Row row(int64_t b) const { return Row{q + b * ldq, vec, N}; }
};

// Runs step K of the policy on the SUB records of one block (nothing when the block is not wanted).
template <int K, int SUB, class Row>
__device__ __forceinline__ void stage_block(const Row &r, typename Row::Pending (&t)[SUB], int base, bool wanted)
{
    if (!wanted) return;   // also false for the lanes beyond a block shorter than 256 ids
#pragma unroll
    for (int i = 0; i < SUB; ++i) r.template stage<K>(t[i], (int64_t)base + i * 256 + lane_id() * 4);
}

__device__ __forceinline__ double lane_partial_sum(const float *part, int nblk, int per_lane)
{
    const int c0 = lane_id() * per_lane;
    double s = 0.0;
    for (int t = 0; t < per_lane; t += 4) {   // four loads in flight at a time
        float v[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) v[x] = (t + x < per_lane && c0 + t + x < nblk) ? part[c0 + t + x] : 0.f;
#pragma unroll
        for (int x = 0; x < 4; ++x) s += (double)v[x];
    }
    return s;
}

// Block in which the inclusive prefix of `part` first exceeds thr (-1 if none) and the prefix before it.
// Lane l owns the per_lane consecutive blocks from l * per_lane.
__device__ __forceinline__ int locate_block(const float *part, int nblk, int per_lane, double lane_sum, double thr,
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
        for (int t = 0; t < per_lane && c0 + t < nblk; ++t) {
            const double v = (double)part[c0 + t];
            if (pre + v > thr) {
                blk = c0 + t;
                break;
            }
            pre += v;
        }
    }
    blk = lane_value(blk, src);
    prefix_before = lane_value(pre, src);
    return blk;
}

// The same on partials that the lanes already hold in registers (at most kRegBlocks per lane): saves the
// dependent re-read.  v[t] = partial of block lane * per_lane + t (0 beyond nblk); R = blocks a lane can hold.
// A lane's blocks are consecutive in memory, so the lanes of one load are per_lane words apart and every load
// instruction touches up to 64 cache lines.  When the row, the blocks per lane and the block count all are multiples
// of four words, groups of four blocks are read by one unconditional 16-byte load each (a group is then wholly inside
// or wholly outside the row; the address of an outside group is clamped and its values dropped): a quarter of the
// line requests and no branch around any load.
template <int R>
__device__ __forceinline__ void load_partials(const float *part, int nblk, int per_lane, float (&v)[R])
{
    static_assert(R % 4 == 0, "a lane holds whole groups of four block sums");
    const int c0 = lane_id() * per_lane;
    if (((uintptr_t)part & 15) == 0 && per_lane % 4 == 0 && nblk % 4 == 0 && nblk >= 4) {   // the same for all lanes
#pragma unroll
        for (int t = 0; t < R; t += 4) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (t < per_lane) {
                const float4 y = *(const float4 *)(part + min(c0 + t, nblk - 4));
                if (c0 + t < nblk) x = y;
            }
            v[t] = x.x; v[t + 1] = x.y; v[t + 2] = x.z; v[t + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int t = 0; t < R; ++t) v[t] = (t < per_lane && c0 + t < nblk) ? part[c0 + t] : 0.f;
    }
}

template <int R>
__device__ __forceinline__ double sum_partials(const float (&v)[R])
{
    double s = 0.0;
#pragma unroll
    for (int t = 0; t < R; ++t) s += (double)v[t];
    return s;
}

template <int R>
__device__ __forceinline__ int locate_block_regs(const float (&v)[R], int nblk, int per_lane, double lane_sum, double thr,
                                                 double &prefix_before)
{
    const double incl = wave_inclusive_scan(lane_sum);
    const unsigned long long hits = __ballot(incl > thr);
    if (hits == 0ull) return -1;
    const int src = __ffsll(hits) - 1;
    const int c0 = lane_id() * per_lane;
    int blk = -1;
    double pre = incl - lane_sum;
#pragma unroll
    for (int t = 0; t < R; ++t) {
        const double x = (double)v[t];
        const bool here = blk < 0 && t < per_lane && c0 + t < nblk && pre + x > thr;
        if (here) blk = c0 + t;
        if (blk < 0) pre += x;
    }
    blk = lane_value(blk, src);
    prefix_before = lane_value(pre, src);
    return blk;
}

// Element (i, e) of a lane's block registers: sub-block i, component e, both run-time values.
template <int SUB>
__device__ __forceinline__ float pick(const float4 (&w)[SUB], int i, int e)
{
    float r = 0.f;
#pragma unroll
    for (int ii = 0; ii < SUB; ++ii) {
        const float t = e == 0 ? w[ii].x : e == 1 ? w[ii].y : e == 2 ? w[ii].z : w[ii].w;
        r = ii == i ? t : r;
    }
    return r;
}

// Smallest id of the block whose inclusive prefix of weights exceeds thr_local; if rounding leaves none,
// the last id of the block with a positive weight.  wv[i] = weights of ids base + i*256 + lane*4 .. +3.
template <int SUB>
__device__ __forceinline__ int search_block(const float4 (&wv)[SUB], int base, double thr_local)
{
    const int lane = lane_id();
    double carried = 0.0;
    int last_positive = -1;
#pragma unroll
    for (int i = 0; i < SUB; ++i) {
        const int idx = base + i * 256 + lane * 4;
        const double l0 = (double)wv[i].x, l1 = l0 + (double)wv[i].y, l2 = l1 + (double)wv[i].z, l3 = l2 + (double)wv[i].w;
        const double incl = wave_inclusive_scan(l3);
        const double excl = carried + (incl - l3);
        const unsigned long long hits = __ballot(excl + l3 > thr_local);
        if (hits != 0ull) {
            const int src = __ffsll(hits) - 1;
            const int e = (excl + l0 > thr_local) ? 0 : (excl + l1 > thr_local) ? 1 : (excl + l2 > thr_local) ? 2 : 3;
            return lane_value(idx + e, src);
        }
        const int mine = wv[i].w > 0.f ? 3 : wv[i].z > 0.f ? 2 : wv[i].y > 0.f ? 1 : wv[i].x > 0.f ? 0 : -1;
        const unsigned long long pos = __ballot(mine >= 0);
        if (pos != 0ull) {
            const int src = 63 - __clzll(pos);
            last_positive = lane_value(idx + mine, src);
        }
        carried += lane_value(incl, kWave - 1);
    }
    return last_positive;
}

// The same for a block of 64 ids held one per lane (w = weight of id base + lane).
__device__ __forceinline__ int search_block1(float w, int base, double thr_local)
{
    const double incl = wave_inclusive_scan((double)w);
    const unsigned long long hits = __ballot(incl > thr_local);
    if (hits != 0ull) return base + (__ffsll(hits) - 1);
    const unsigned long long pos = __ballot(w > 0.f);
    return pos != 0ull ? base + (63 - __clzll(pos)) : -1;
}

constexpr int kFinalizeRows = 8;   // rows (wavefronts) per workgroup at most: leaves 256 VGPRs per lane

// Which row a one-row workgroup takes when the policy re-computes q' from tables that the kernel before it left in the
// L2 of one XCD (the sparse product sweeps the rows of a 32-position block on one XCD when there are 8 k such blocks):
// consecutive workgroup ids go to consecutive XCDs, so workgroup i takes a row of the blocks that XCD i % 8 has swept.
// Any other batch shape keeps the identity; the mapping only decides which cache a row's lookups find warm.
__device__ __forceinline__ int64_t xcd_row(int64_t i, int B)
{
    if (B % 256 != 0) return i;
    const int64_t per_xcd = B / 8;
    return (i % 8) * per_xcd + i / 8;
}
constexpr int kSpreadMinRows = 128;   // from this many rows on every row gets a workgroup of its own

// The finish of one row by one wavefront: pq, prr, pa = the row's block sums of q', max(0, p - q') and min(p, q').
// Writes the row's outputs and hands back the drafted id, the residual id and the accept flag (for a scan by the caller).
// BLOCK = ids per block of partial sums: a multiple of 256, or 64 (then one id per lane).
template <int KIND, int BLOCK, bool HAS_Q, class QP>
__device__ __forceinline__ void finalize_row(const FinalizeArgs &a, const QP &qp, int64_t row, const float *pq, const float *prr,
                                             const float *pa, int32_t &dtok_out, int32_t &rtok_out, uint8_t &acc_out)
{
    constexpr int SUB = BLOCK >= 256 ? BLOCK / 256 : 1;
    constexpr int kLanes = BLOCK >= 256 ? kWave : BLOCK / 4;      // lanes that hold ids of a block
    constexpr int kRegBlocks = QP::kSpreadRows ? 32 : 8;          // block partials a lane keeps in registers
    const rdk_verify_desc_t &d = a.d;
    const int lane = lane_id();
    const int N = d.N;
    const void *pr = row_ptr<KIND>(a.p, a.ldp, row);
    float m = 0.f, inv = 1.f;
    if (KIND != RDK_PROB_F32) {
        const SoftStat rs = merged_row_stat<KIND>(a.pstat, a.p_splits, row);
        m = rs.m;
        inv = 1.0f / rs.s;
    }
    const float pfill = KIND == RDK_PROB_F32 ? 0.f : -INFINITY;
    const int per_lane = ((a.nblk + kWave - 1) / kWave + 3) & ~3;   // blocks per lane, in whole groups of four
    const bool draw_draft = HAS_Q && d.sample_draft;

    // 1. block partials (one round trip; kept in registers when they fit), the row's own constants and the
    //    uniforms meanwhile
    const bool in_regs = per_lane <= kRegBlocks;
    float vq[kRegBlocks], vr[kRegBlocks], va[kRegBlocks];
    double lane_r, lane_q = 0.0, lane_a = 0.0;
    if (in_regs) {
        load_partials(prr, a.nblk, per_lane, vr);
        if (draw_draft) load_partials(pq, a.nblk, per_lane, vq);
        if (HAS_Q) load_partials(pa, a.nblk, per_lane, va);
    }
    const typename QP::Row qrow = qp.row(row);
    if (in_regs) {
        lane_r = sum_partials(vr);
        if (draw_draft) lane_q = sum_partials(vq);
        if (HAS_Q) lane_a = sum_partials(va);
    } else {
        lane_r = lane_partial_sum(prr, a.nblk, per_lane);
        if (draw_draft) lane_q = lane_partial_sum(pq, a.nblk, per_lane);
        if (HAS_Q) lane_a = lane_partial_sum(pa, a.nblk, per_lane);
    }
    int32_t dtok = (HAS_Q && !d.sample_draft) ? a.draft_ids[row] : -1;
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
        blk_d = in_regs ? locate_block_regs(vq, a.nblk, per_lane, lane_q, thr_d, before_d)
                        : locate_block(pq, a.nblk, per_lane, lane_q, thr_d, before_d);
    }
    if (R > 0.0) {
        thr_r = word_to_unit(words[HAS_Q ? 2 : 3]) * R;
        blk_r = in_regs ? locate_block_regs(vr, a.nblk, per_lane, lane_r, thr_r, before_r)
                        : locate_block(prr, a.nblk, per_lane, lane_r, thr_r, before_r);
    }

    // 3. both blocks are fetched together (q' and the target weights of each), then scanned.  A draft token
    //    that the caller supplied may lie anywhere: its two values are requested in the same round trip.
    const int base_d = max(blk_d, 0) * BLOCK, base_r = max(blk_r, 0) * BLOCK;
    const bool same = draw_draft && blk_r == blk_d;
    float pd_w = 0.f, qd = 0.f;
    const bool given = HAS_Q && !d.sample_draft && dtok >= 0 && dtok < N;
    if (given) {
        pd_w = to_weight<KIND>(load1<KIND>(pr, dtok), m, inv);
        qd = qrow.load1(dtok);
    }
    const bool want_r = HAS_Q && !same;
    int32_t rtok = -1;
    if constexpr (BLOCK == 64) {
        // blocks of 64 ids, one id per lane: the policy's chain of dependent loads is as short as it gets (one
        // slot, one table row, its gathers) and all 64 lanes share it
        typename QP::Row::Pending1 td, tr;
        const int id_d = base_d + lane, id_r = base_r + lane;
        if (draw_draft) qrow.template stage1<0>(td, id_d);
        if (want_r) qrow.template stage1<0>(tr, id_r);
        float pdv = pfill, wpv = pfill;
        if (draw_draft && id_d < N) pdv = load1<KIND>(pr, id_d);
        if (!same && id_r < N) wpv = load1<KIND>(pr, id_r);
        if (draw_draft) qrow.template stage1<1>(td, id_d);
        if (want_r) qrow.template stage1<1>(tr, id_r);
        if (draw_draft) qrow.template stage1<2>(td, id_d);
        if (want_r) qrow.template stage1<2>(tr, id_r);
        const float wdv = draw_draft ? qrow.result1(td, id_d) : 0.f;
        float wqv = want_r ? qrow.result1(tr, id_r) : 0.f;
        if (same) {
            wpv = pdv;
            wqv = wdv;
        }
        if (blk_d >= 0) {
            dtok = search_block1(wdv, base_d, thr_d - before_d);
            if (dtok >= 0) {
                qd = lane_value(wdv, dtok - base_d);
                pd_w = to_weight<KIND>(lane_value(pdv, dtok - base_d), m, inv);
            }
        }
        if (blk_r >= 0) {
            wpv = to_weight<KIND>(wpv, m, inv);
            if (HAS_Q) wpv = fmaxf(wpv - wqv, 0.f);
            rtok = search_block1(wpv, base_r, thr_r - before_r);
        }
    } else {
        float4 wd[SUB], pd[SUB], wp[SUB], wq[SUB];
        const bool holds = lane < kLanes;
        typename QP::Row::Pending td[SUB], tr[SUB];
        const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f), fill4 = make_float4(pfill, pfill, pfill, pfill);
        stage_block<0, SUB>(qrow, td, base_d, draw_draft && holds);
        stage_block<0, SUB>(qrow, tr, base_r, want_r && holds);
#pragma unroll
        for (int i = 0; i < SUB; ++i) {
            if (draw_draft) pd[i] = holds ? load4<KIND>(pr, base_d + i * 256 + lane * 4, N, a.vec_p, pfill) : fill4;
            if (!same) wp[i] = holds ? load4<KIND>(pr, base_r + i * 256 + lane * 4, N, a.vec_p, pfill) : fill4;
        }
        if (QP::kStages > 1) {
            stage_block<1, SUB>(qrow, td, base_d, draw_draft && holds);
            stage_block<1, SUB>(qrow, tr, base_r, want_r && holds);
        }
        if (QP::kStages > 2) {
            stage_block<2, SUB>(qrow, td, base_d, draw_draft && holds);
            stage_block<2, SUB>(qrow, tr, base_r, want_r && holds);
        }
#pragma unroll
        for (int i = 0; i < SUB; ++i) {
            if (draw_draft) wd[i] = holds ? qrow.result(td[i], (int64_t)base_d + i * 256 + lane * 4) : zero4;
            if (want_r) wq[i] = holds ? qrow.result(tr[i], (int64_t)base_r + i * 256 + lane * 4) : zero4;
            if (same) {
                wp[i] = pd[i];
                wq[i] = wd[i];
            }
        }
        if (blk_d >= 0) {
            dtok = search_block<SUB>(wd, base_d, thr_d - before_d);
            // 4. the accept test needs p and q' at the draft token: both sit in the registers of one lane
            if (dtok >= 0) {
                const int off = dtok - base_d, i = off / 256, src = (off % 256) / 4, e = off % 4;
                qd = lane_value(pick<SUB>(wd, i, e), src);
                pd_w = to_weight<KIND>(lane_value(pick<SUB>(pd, i, e), src), m, inv);
            }
        }
        if (blk_r >= 0) {
#pragma unroll
            for (int i = 0; i < SUB; ++i) {
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
            rtok = search_block<SUB>(wp, base_r, thr_r - before_r);
        }
    }
    const bool d_ok = HAS_Q && dtok >= 0 && dtok < N;
    uint8_t acc = 0;
    if (d_ok) acc = (word_to_unit(words[1]) * (double)qd < (double)pd_w) ? 1 : 0;
    if (lane == 0) {
        if (draw_draft) a.draft_ids[row] = dtok;
        a.accept[row] = acc;
        if (a.alpha) a.alpha[row] = (float)A;
        if (a.resid_mass) a.resid_mass[row] = (float)R;
        a.resid_ids[row] = rtok;
    }
    dtok_out = dtok;
    rtok_out = rtok;
    acc_out = acc;
}

template <int KIND, int BLOCK, bool HAS_Q, class QP>
__global__ __launch_bounds__(QP::kSpreadRows ? kWave : kFinalizeRows * kWave) void verify_finalize_kernel(FinalizeArgs a, QP qp)
{
    __shared__ int32_t sh_draft[kFinalizeRows], sh_resid[kFinalizeRows];
    __shared__ uint8_t sh_acc[kFinalizeRows];
    const rdk_verify_desc_t &d = a.d;
    const int wid = threadIdx.x / kWave, lane = lane_id();
    const int64_t row = QP::kSpreadRows ? xcd_row(blockIdx.x, d.B) : (int64_t)blockIdx.x * a.rows_per_block + wid;
    if (row < d.B) {
        int32_t dtok, rtok;
        uint8_t acc;
        finalize_row<KIND, BLOCK, HAS_Q, QP>(a, qp, row, a.part_q + row * a.nblk, a.part_r + row * a.nblk, a.part_a + row * a.nblk,
                                             dtok, rtok, acc);
        if (a.scan_here && lane == 0) {
            sh_draft[wid] = dtok;
            sh_resid[wid] = rtok;
            sh_acc[wid] = acc;
        }
    }
    if (a.scan_here) {  // the workgroup holds exactly one sequence: steps 4-10 of Alg. 4
        __syncthreads();
        if (threadIdx.x == 0) {
            const int g = d.gamma;
            int j = 0;
            while (j < g && sh_acc[j]) ++j;
            if (a.n_accepted) a.n_accepted[blockIdx.x] = j;
            if (a.out_tokens) {
                int32_t *o = a.out_tokens + (int64_t)blockIdx.x * (g + 1);
                for (int i = 0; i <= g; ++i) o[i] = i < j ? sh_draft[i] : (i == j && j < g) ? sh_resid[i] : -1;
            }
        }
    }
}

// The finish of one row by a workgroup of four wavefronts, for the policies that re-compute q' one id per lane (blocks
// of 64 ids).  A lone wavefront pays the full latency of every dependent instruction, and half of its time went into
// adding up and searching the three kinds of block sums one after the other; here wavefront 0 takes the sums of q' and
// the draft's block, wavefront 1 the residual sums and the residual's block, wavefront 2 alpha (and the two values of a
// draft the caller supplied), each with the routines of finalize_row, so the results are the same bits.
template <int KIND, class QP>
__global__ __launch_bounds__(4 * kWave) void verify_finalize_wide_kernel(FinalizeArgs a, QP qp)
{
    constexpr int kRegBlocks = 64;   // block sums a lane keeps in registers: one kind per wavefront, so 4096 blocks (N = 262144) fit
    __shared__ double sh_d[2];   // alpha, residual mass
    __shared__ int sh_i[2];      // the drafted id, the residual id
    __shared__ float sh_f[2];    // q' and p at the draft
    const rdk_verify_desc_t &d = a.d;
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = lane_id();
    const int64_t row = xcd_row(blockIdx.x, d.B);
    const int N = d.N;
    const void *pr = row_ptr<KIND>(a.p, a.ldp, row);
    float m = 0.f, inv = 1.f;
    if (KIND != RDK_PROB_F32) {
        const SoftStat rs = merged_row_stat<KIND>(a.pstat, a.p_splits, row);
        m = rs.m;
        inv = 1.0f / rs.s;
    }
    const float pfill = KIND == RDK_PROB_F32 ? 0.f : -INFINITY;
    const bool draw_draft = d.sample_draft;
    const int per_lane = ((a.nblk + kWave - 1) / kWave + 3) & ~3;   // blocks per lane, in whole groups of four
    const bool in_regs = per_lane <= kRegBlocks;
    uint32_t words[4] = {0u, 0u, 0u, 0u};
    int blk = -1;                // the block of this wavefront's draw (-1: nothing to draw) and the threshold inside it
    double thr_local = 0.0;
    // 1. one kind of block sums per wavefront
    if (wid < 3) {
        const float *part = (wid == 0 ? a.part_q : wid == 1 ? a.part_r : a.part_a) + row * a.nblk;
        const bool wanted = wid == 0 ? draw_draft : true;
        float v[kRegBlocks];
        double lane_s = 0.0;
        if (wanted && in_regs) load_partials(part, a.nblk, per_lane, v);
        position_words(d.seed, d.offset + (uint64_t)row, words);   // while the sums are on their way
        if (wanted) lane_s = in_regs ? sum_partials(v) : lane_partial_sum(part, a.nblk, per_lane);
        const double T = wanted ? wave_sum(lane_s) : 0.0;
        if (wid < 2 && wanted && T > 0.0) {
            const double thr = word_to_unit(words[wid == 0 ? 0 : 2]) * T;
            double before = 0.0;
            blk = in_regs ? locate_block_regs(v, a.nblk, per_lane, lane_s, thr, before)
                          : locate_block(part, a.nblk, per_lane, lane_s, thr, before);
            thr_local = thr - before;
        }
        if (lane == 0 && wid >= 1) sh_d[2 - wid] = T;   // wavefront 1: residual mass -> [1], wavefront 2: alpha -> [0]
    }
    // 2. the block of the draft (wavefront 0) and of the residual draw (wavefront 1), one id per lane; the two values of
    //    a caller's draft (wavefront 2)
    const typename QP::Row qrow = qp.row(row);
    if (wid < 2) {
        int tok = -1;
        if (blk >= 0) {
            const int base = blk * 64, id = base + lane;
            typename QP::Row::Pending1 t;
            qrow.template stage1<0>(t, id);
            float pv = pfill;
            if (id < N) pv = load1<KIND>(pr, id);
            qrow.template stage1<1>(t, id);
            qrow.template stage1<2>(t, id);
            const float wq = qrow.result1(t, id);
            const float pw = to_weight<KIND>(pv, m, inv);
            tok = search_block1(wid == 0 ? wq : fmaxf(pw - wq, 0.f), base, thr_local);
            if (wid == 0 && tok >= 0) {
                const float qd = lane_value(wq, tok - base), pd = lane_value(pw, tok - base);
                if (lane == 0) {
                    sh_f[0] = qd;
                    sh_f[1] = pd;
                }
            }
        }
        if (lane == 0) sh_i[wid] = tok;
    } else if (wid == 2 && !draw_draft) {
        const int32_t dtok = a.draft_ids[row];
        if (dtok >= 0 && dtok < N) {
            const float pd = to_weight<KIND>(load1<KIND>(pr, dtok), m, inv), qd = qrow.load1(dtok);
            if (lane == 0) {
                sh_f[0] = qd;
                sh_f[1] = pd;
            }
        }
    }
    __syncthreads();
    // 3. the accept test and the row's outputs
    if (threadIdx.x == 0) {
        const int32_t dtok = draw_draft ? sh_i[0] : a.draft_ids[row];
        const bool d_ok = dtok >= 0 && dtok < N;
        uint8_t acc = 0;
        if (d_ok) acc = (word_to_unit(words[1]) * (double)sh_f[0] < (double)sh_f[1]) ? 1 : 0;
        if (draw_draft) a.draft_ids[row] = dtok;
        a.accept[row] = acc;
        if (a.alpha) a.alpha[row] = (float)sh_d[0];
        if (a.resid_mass) a.resid_mass[row] = (float)sh_d[1];
        a.resid_ids[row] = sh_i[1];
    }
}

// ---- The finish of one row by eight wavefronts, for block sums over 1024 ids (Alg. 4, steps 2 and 4-6 for one position).
// A lone wavefront pays the full latency of every dependent step; here
//   1. three wavefronts add up one kind of block sum each in fp64 (sum q', residual mass, alpha) and find the block
//      in which the inverse-CDF threshold of the draft / of the residual draw is crossed;
//   2. eight wavefronts take a quarter of one of the two blocks each (256 ids, four per lane: the target values from
//      memory, q' from the policy) and scan it in fp64;
//   3. with the totals of the quarters before its own, each finds the crossing in its quarter (or its last id with
//      a positive weight, the answer when rounding leaves no crossing);
//   4. the first wavefront picks the first crossing, tests acceptance in fp64 and writes the row's outputs.
// The arithmetic, its order and the conventions are those of the one-wavefront finish (finalize_row, search_block).
// Every wavefront of the workgroup calls it (more than eight may; the others only meet the barriers).
//   scratch        kFinishFloats floats of LDS
//   sq, sr, sa     the row's nblk block sums of q', max(0, p - q') and min(p, q') (LDS or memory)
//   pm, pinv       softmax maximum and 1 / normaliser of a logit target row (0 and 1 for probabilities)
//   words          the position's four uniforms (Alg. 4: draft, accept, residual, bonus)
//   quads          where q' comes from: begin() issues the loads that need no target value, end() hands out q' of four
//                  ids given their target weights, at() q' of one id
constexpr int kFinishFloats = 64;

template <int KIND, class Quads>
__device__ __forceinline__ void finish_row_quarters(float *scratch, const float *sq, const float *sr, const float *sa, int nblk,
                                                    const FinalizeArgs &fin, int64_t row, const void *pr, float pm, float pinv,
                                                    int N, bool vec_p, const Quads &quads, const uint32_t (&words)[4], int wid,
                                                    int lane)
{
    constexpr int kBlock = 1024;
    double *fd = (double *)scratch;                   // [0..1] local thresholds, [2] alpha, [3] residual mass, [4..11] quarter totals
    int *fi = (int *)(scratch + 24);                  // [0..1] the two blocks (-1: nothing to draw)
    float4 *fc = (float4 *)(scratch + 32);            // per quarter: crossing id, last positive id, q' and p at the candidate
    const rdk_verify_desc_t &d = fin.d;
    const bool draw_draft = d.sample_draft;
    if (wid < 3) {
        const float *part = wid == 0 ? sq : wid == 1 ? sr : sa;
        const bool wanted = wid == 0 ? draw_draft : true;
        constexpr int kRegBlocks = 8;
        const int per_lane = ((nblk + kWave - 1) / kWave + 3) & ~3;
        const bool in_regs = per_lane <= kRegBlocks;
        float v[kRegBlocks];
        double lane_s = 0.0;
        if (wanted) {
            if (in_regs) {
                load_partials(part, nblk, per_lane, v);
                lane_s = sum_partials(v);
            } else {
                lane_s = lane_partial_sum(part, nblk, per_lane);
            }
        }
        const double T = wanted ? wave_sum(lane_s) : 0.0;
        int blk = -1;
        double thr = 0.0, before = 0.0;
        if (wid < 2 && wanted && T > 0.0) {
            thr = word_to_unit(words[wid == 0 ? 0 : 2]) * T;
            blk = in_regs ? locate_block_regs(v, nblk, per_lane, lane_s, thr, before)
                          : locate_block(part, nblk, per_lane, lane_s, thr, before);
        }
        if (lane == 0) {
            if (wid < 2) {
                fi[wid] = blk;
                fd[wid] = thr - before;
            }
            if (wid >= 1) fd[4 - wid] = T;            // wavefront 1: residual mass -> [3], wavefront 2: alpha -> [2]
        }
    }
    __syncthreads();
    const int fb = wid >> 2, fq = wid & 3;            // which of the two blocks, which quarter of it
    const int fblk = wid < 8 ? fi[fb] : -1;
    const bool factive = fblk >= 0;
    const int64_t fidx = (int64_t)max(fblk, 0) * kBlock + fq * 256 + lane * 4;
    float qp4[4] = {0.f, 0.f, 0.f, 0.f}, pv4[4] = {0.f, 0.f, 0.f, 0.f}, wv4[4] = {0.f, 0.f, 0.f, 0.f};
    double l0 = 0.0, l1 = 0.0, l2 = 0.0, l3 = 0.0, incl = 0.0;
    int last_pos = -1;
    if (factive) {
        typename Quads::Token t = quads.begin(fblk, fq, fidx);
        const float4 pl = load4<KIND>(pr, fidx, N, vec_p, KIND == RDK_PROB_F32 ? 0.f : -INFINITY);
        pv4[0] = to_weight<KIND>(pl.x, pm, pinv); pv4[1] = to_weight<KIND>(pl.y, pm, pinv);
        pv4[2] = to_weight<KIND>(pl.z, pm, pinv); pv4[3] = to_weight<KIND>(pl.w, pm, pinv);
        quads.end(t, fidx, pv4, qp4);
#pragma unroll
        for (int e = 0; e < 4; ++e) wv4[e] = fb == 0 ? qp4[e] : fmaxf(pv4[e] - qp4[e], 0.f);
        l0 = (double)wv4[0]; l1 = l0 + (double)wv4[1]; l2 = l1 + (double)wv4[2]; l3 = l2 + (double)wv4[3];
        incl = wave_inclusive_scan(l3);
        if (lane == kWave - 1) fd[4 + wid] = incl;
        const int mine = wv4[3] > 0.f ? 3 : wv4[2] > 0.f ? 2 : wv4[1] > 0.f ? 1 : wv4[0] > 0.f ? 0 : -1;
        const unsigned long long pos = __ballot(mine >= 0);
        if (pos != 0ull) last_pos = lane_value((int)fidx + mine, 63 - __clzll(pos));
    }
    __syncthreads();
    if (factive) {
        double carried = 0.0;
        for (int i = 0; i < fq; ++i) carried += fd[4 + 4 * fb + i];
        const double thr_local = fd[fb];
        const double excl = carried + (incl - l3);
        const unsigned long long hits = __ballot(excl + l3 > thr_local);
        int hit = -1;
        if (hits != 0ull) {
            const int e = (excl + l0 > thr_local) ? 0 : (excl + l1 > thr_local) ? 1 : (excl + l2 > thr_local) ? 2 : 3;
            hit = lane_value((int)fidx + e, __ffsll(hits) - 1);
        }
        const int cand = hit >= 0 ? hit : last_pos;
        float qc = 0.f, pc = 0.f;
        if (cand >= 0) {
            const int off = cand - (fblk * kBlock + fq * 256), src = off / 4, e = off % 4;
            qc = lane_value(e == 0 ? qp4[0] : e == 1 ? qp4[1] : e == 2 ? qp4[2] : qp4[3], src);
            pc = lane_value(e == 0 ? pv4[0] : e == 1 ? pv4[1] : e == 2 ? pv4[2] : pv4[3], src);
        }
        if (lane == 0) fc[wid] = make_float4(__int_as_float(hit), __int_as_float(last_pos), qc, pc);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int tok[2] = {-1, -1};
        float qd = 0.f, pd_w = 0.f;
        for (int b = 0; b < 2; ++b) {
            if (fi[b] < 0) continue;
            int chosen = -1;
            for (int i = 0; i < 4 && chosen < 0; ++i)
                if (__float_as_int(fc[4 * b + i].x) >= 0) chosen = i;
            if (chosen < 0)
                for (int i = 3; i >= 0 && chosen < 0; --i)
                    if (__float_as_int(fc[4 * b + i].y) >= 0) chosen = i;
            if (chosen >= 0) {
                const float4 c4 = fc[4 * b + chosen];
                tok[b] = __float_as_int(c4.x) >= 0 ? __float_as_int(c4.x) : __float_as_int(c4.y);
                if (b == 0) {
                    qd = c4.z;
                    pd_w = c4.w;
                }
            }
        }
        int32_t dtok = tok[0];
        if (!draw_draft) {                            // the caller's draft: its two values are fetched here
            dtok = fin.draft_ids[row];
            if (dtok >= 0 && dtok < N) {
                pd_w = to_weight<KIND>(load1<KIND>(pr, dtok), pm, pinv);
                qd = quads.at(dtok, pd_w);
            }
        }
        const bool d_ok = dtok >= 0 && dtok < N;
        uint8_t acc = 0;
        if (d_ok) acc = (word_to_unit(words[1]) * (double)qd < (double)pd_w) ? 1 : 0;
        if (draw_draft) fin.draft_ids[row] = dtok;
        fin.accept[row] = acc;
        if (fin.alpha) fin.alpha[row] = (float)fd[2];
        if (fin.resid_mass) fin.resid_mass[row] = (float)fd[3];
        fin.resid_ids[row] = tok[1];
    }
}

// q' of four ids from a policy's row (its steps run back to back: one quarter of a block per wavefront).
template <class Row, int STAGES>
struct PolicyQuads {
    const Row &r;
    typedef typename Row::Pending Token;
    __device__ __forceinline__ Token begin(int, int, int64_t fidx) const
    {
        Token t;
        r.template stage<0>(t, fidx);
        return t;
    }
    __device__ __forceinline__ void end(Token &t, int64_t fidx, const float (&)[4], float (&qp4)[4]) const
    {
        if (STAGES > 1) r.template stage<1>(t, fidx);
        if (STAGES > 2) r.template stage<2>(t, fidx);
        const float4 v = r.result(t, fidx);
        qp4[0] = v.x; qp4[1] = v.y; qp4[2] = v.z; qp4[3] = v.w;
    }
    __device__ __forceinline__ float at(int dtok, float) const { return r.load1(dtok); }
};

// One row per workgroup of eight wavefronts, block sums over 1024 ids in memory.
template <int KIND, class QP>
__global__ __launch_bounds__(8 * kWave) void verify_finalize_quarters_kernel(FinalizeArgs a, QP qp)
{
    __shared__ __attribute__((aligned(16))) float scratch[kFinishFloats];
    const rdk_verify_desc_t &d = a.d;
    const int wid = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = lane_id();
    const int64_t row = blockIdx.x;
    const void *pr = row_ptr<KIND>(a.p, a.ldp, row);
    float m = 0.f, inv = 1.f;
    if (KIND != RDK_PROB_F32) {
        const SoftStat rs = merged_row_stat<KIND>(a.pstat, a.p_splits, row);
        m = rs.m;
        inv = 1.0f / rs.s;
    }
    uint32_t words[4];
    position_words(d.seed, d.offset + (uint64_t)row, words);
    const typename QP::Row qrow = qp.row(row);
    const PolicyQuads<typename QP::Row, QP::kStages> quads{qrow};
    finish_row_quarters<KIND>(scratch, a.part_q + row * a.nblk, a.part_r + row * a.nblk, a.part_a + row * a.nblk, a.nblk, a, row, pr,
                              m, inv, d.N, a.vec_p, quads, words, wid, lane);
}

// ---- Draft draw alone (Alg. 4 step 2 on the drafter's side, before a target row exists): one wavefront per row,
// block sums of q' in, the drafted id and q' at that id out.
struct DraftArgs {
    int32_t B, N;
    uint64_t seed, offset;
    const float *part_q;   // [B, nblk]
    int nblk;
    int32_t *draft_ids;
    float *q_draft;        // may be NULL
};

template <int BLOCK, class QP>
__global__ __launch_bounds__(kWave) void draft_finalize_kernel(DraftArgs a, QP qp)
{
    constexpr int SUB = BLOCK >= 256 ? BLOCK / 256 : 1;
    constexpr int kLanes = BLOCK >= 256 ? kWave : BLOCK / 4;
    constexpr int kRegBlocks = 32;
    const int64_t row = QP::kSpreadRows ? xcd_row(blockIdx.x, a.B) : (int64_t)blockIdx.x;
    const int lane = lane_id();
    const int per_lane = ((a.nblk + kWave - 1) / kWave + 3) & ~3;   // blocks per lane, in whole groups of four
    const float *pq = a.part_q + row * a.nblk;
    const bool in_regs = per_lane <= kRegBlocks;
    float vq[kRegBlocks];
    double lane_q;
    if (in_regs) load_partials(pq, a.nblk, per_lane, vq);
    const typename QP::Row qrow = qp.row(row);
    lane_q = in_regs ? sum_partials(vq) : lane_partial_sum(pq, a.nblk, per_lane);
    uint32_t words[4];
    position_words(a.seed, a.offset + (uint64_t)row, words);
    const double Q = wave_sum(lane_q);
    int blk = -1;
    double thr = 0.0, before = 0.0;
    if (Q > 0.0) {
        thr = word_to_unit(words[0]) * Q;
        blk = in_regs ? locate_block_regs(vq, a.nblk, per_lane, lane_q, thr, before)
                      : locate_block(pq, a.nblk, per_lane, lane_q, thr, before);
    }
    int32_t dtok = -1;
    float qd = 0.f;
    if (blk >= 0) {
        const int base = blk * BLOCK;
        if constexpr (BLOCK == 64) {
            typename QP::Row::Pending1 td;
            const int id = base + lane;
            qrow.template stage1<0>(td, id);
            qrow.template stage1<1>(td, id);
            qrow.template stage1<2>(td, id);
            const float wdv = qrow.result1(td, id);
            dtok = search_block1(wdv, base, thr - before);
            if (dtok >= 0) qd = lane_value(wdv, dtok - base);
        } else {
            const bool holds = lane < kLanes;
            typename QP::Row::Pending td[SUB];
            float4 wd[SUB];
            stage_block<0, SUB>(qrow, td, base, holds);
            if (QP::kStages > 1) stage_block<1, SUB>(qrow, td, base, holds);
            if (QP::kStages > 2) stage_block<2, SUB>(qrow, td, base, holds);
#pragma unroll
            for (int i = 0; i < SUB; ++i)
                wd[i] = holds ? qrow.result(td[i], (int64_t)base + i * 256 + lane * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
            dtok = search_block<SUB>(wd, base, thr - before);
            if (dtok >= 0) {
                const int off = dtok - base;
                qd = lane_value(pick<SUB>(wd, off / 256, off % 4), (off % 256) / 4);
            }
        }
    }
    if (lane == 0) {
        a.draft_ids[row] = dtok;
        if (a.q_draft) a.q_draft[row] = qd;
    }
}

template <int BLOCK, class QP>
rdk_status_t launch_draft_finalize(const DraftArgs &a, QP qp, hipStream_t st)
{
    RDK_TIMED_LAUNCH("draft_finalize_kernel", (draft_finalize_kernel<BLOCK, QP>), dim3((unsigned)a.B), dim3(kWave), 0, st, a,
                     qp);
    RDK_LAUNCH_CHECK("draft_finalize_kernel");
    return RDK_OK;
}

// Per-sequence scan as a launch of its own (sequences longer than one workgroup's wavefronts).
__global__ void sequence_scan_kernel(int S, int gamma, const int32_t *draft_ids, const uint8_t *accept,
                                     const int32_t *resid_ids, int32_t *n_accepted, int32_t *out_tokens);

rdk_status_t launch_sequence_scan(const rdk_verify_desc_t &d, const int32_t *draft_ids, const uint8_t *accept,
                                  const int32_t *resid_ids, int32_t *n_accepted, int32_t *out_tokens, hipStream_t st);

template <int KIND, int BLOCK, bool HAS_Q, class QP>
rdk_status_t launch_finalize(FinalizeArgs a, QP qp, hipStream_t st)
{
    const rdk_verify_desc_t &d = a.d;
    // One wavefront per row is bound by its own chain of dependent steps, and eight of them on one compute unit share
    // its four vector units: a large batch gets a workgroup per row (and the per-sequence scan a launch of its own),
    // a small one keeps a sequence together and scans it in place.  A policy that re-computes q' is heavy on the vector
    // memory pipe of its compute unit and always gets one per row.
    const bool spread = QP::kSpreadRows || d.B >= kSpreadMinRows;
    a.scan_here = d.gamma >= 1 && d.gamma <= kFinalizeRows && !spread;
    a.rows_per_block = a.scan_here ? d.gamma : (spread ? 1 : 4);
    const int blocks = (d.B + a.rows_per_block - 1) / a.rows_per_block;
    constexpr bool kWide = QP::kSpreadRows && BLOCK == 64 && HAS_Q;   // four wavefronts per row, one id per lane
    constexpr bool kQuarters = BLOCK == 1024 && HAS_Q;                // eight wavefronts per row when rows are spread
    bool launched = false;
    if constexpr (kWide) {
        RDK_TIMED_LAUNCH("verify_finalize_kernel", (verify_finalize_wide_kernel<KIND, QP>), dim3((unsigned)d.B), dim3(4 * kWave), 0,
                         st, a, qp);
        launched = true;
    } else if constexpr (kQuarters) {
        if (spread) {
            RDK_TIMED_LAUNCH("verify_finalize_kernel", (verify_finalize_quarters_kernel<KIND, QP>), dim3((unsigned)d.B),
                             dim3(8 * kWave), 0, st, a, qp);
            launched = true;
        }
    }
    if (!launched) {
        RDK_TIMED_LAUNCH("verify_finalize_kernel", (verify_finalize_kernel<KIND, BLOCK, HAS_Q, QP>), dim3(blocks),
                         dim3(a.rows_per_block * kWave), 0, st, a, qp);
    }
    RDK_LAUNCH_CHECK("verify_finalize_kernel");
    if (d.gamma > 0 && !a.scan_here && (a.n_accepted || a.out_tokens))
        return launch_sequence_scan(d, a.draft_ids, a.accept, a.resid_ids, a.n_accepted, a.out_tokens, st);
    return RDK_OK;
}

}  // namespace rdk
