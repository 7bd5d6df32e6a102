// Alg. 1, step 2 with the top-k sparse kernel:  q'[b, j] = sum_t w[j, t] * TLI(q)[b, slot[j, t]]  for a
// pruned id j,  q'[b, j] = self_w[s] * TLI(q)[b, s]  for a kept id j (slot s).
//
// The product costs (N - n) * k gathered multiply-adds per position, an order of magnitude more
// cache traffic than its compulsory HBM bytes, so everything here is arranged around the gather:
//   * the drafter rows are first laid out position-minor, 32 positions side by side
//     (qT[pb][slot][32]); one neighbour of one id is then ONE 128-byte cache line that serves 32
//     positions (the vector L1 of a CU spends about 2.4 clocks per distinct line, whatever part of the
//     line is used);
//   * a workgroup owns 256 consecutive target ids x 32 positions; its pruned ids and kept ids are
//     contiguous runs of pruned slots / kept slots, handled separately (16 gathers vs one coalesced read);
//   * workgroups are numbered so that each XCD sweeps all id tiles of one position block before moving
//     on: the 4 MB slab of that block stays in the XCD's own L2;
//   * results are staged in LDS and leave as full 1 KB row segments.
#include "rdk_finalize.hpp"

namespace rdk {

namespace {

constexpr int kThreads = 512;     // product kernel: 8 wavefronts share one staged tile
constexpr int kWaves = kThreads / kWave;
constexpr int kPrepThreads = 256; // transposition kernel
constexpr int kTSlots = 64;       // slots per LDS tile of the transposition kernel (128 and 256 were slower)
constexpr int kTGroup = 8;        // tiles per workgroup of the transposition kernel: one partial row sum per 512 slots
constexpr int kPosBlock = 32;    // positions per gather: 32 fp32 = one 128-byte line
constexpr int kTileIds = 256;    // target ids per workgroup
constexpr int kStageLd = kTileIds + 4;   // rows stay 16-byte aligned for the float4 read-out
constexpr int kSubIds = 64;       // ids per block of verification sums in the fused form: 16 lanes x 4 ids

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

struct SparseWs {
    SoftStat *qpart;   // [B, q_splits]  drafter row statistics, a few partials per row
    float *zpart;      // [B, zt]  partial sums of the drafter weights, one per 512 slots (Eq. 1 divides by their sum)
    int zt;
    float *qT;         // [ceil(B/32), n, 32]
    int q_splits;
};

SparseWs carve(const KernelHandle &h, int32_t B, void *ws)
{
    SparseWs w;
    w.q_splits = row_splits(B, h.n, kPrepThreads / kWave);
    char *p = (char *)ws;
    w.qpart = (SoftStat *)p; p += align_up((size_t)B * kMaxSplits * sizeof(SoftStat), 256);
    w.zt = (h.n + kTSlots * kTGroup - 1) / (kTSlots * kTGroup);
    w.zpart = (float *)p; p += align_up((size_t)B * w.zt * sizeof(float), 256);
    w.qT = (float *)p;
    return w;
}

// Sum over the 8 lanes of an aligned group.
__device__ __forceinline__ float oct_sum(float v)
{
    v += __shfl_xor(v, 1, kWave);
    v += __shfl_xor(v, 2, kWave);
    v += __shfl_xor(v, 4, kWave);
    return v;
}

// ------------------------------------------------------------------------------------------------
// qT[(pb * n + s) * 32 + r] = weight(q[pb*32 + r, s]); zero for positions beyond B.  weight = the raw
// probability, or exp(z - row max) for logits; the division by the row sum (Eq. 1) happens in the product, from the
// partial sums this kernel leaves: zpart[b, x] = sum of the weights of row b over the 512 slots of workgroup x (eight
// threads per row, eight tiles of 64 slots each, all loads of a workgroup requested before the first is used).
template <int QK>
__global__ __launch_bounds__(kPrepThreads) void q_transpose_kernel(const void *q, int64_t ldq, int n, int B,
                                                                   const SoftStat *qpart, int q_splits, bool vec, float *zpart,
                                                                   int zt, float *qT, const SoftStat *pstat, int p_splits,
                                                                   SoftStat *pmerged)
{
    __shared__ float tile[2][kTSlots][kPosBlock + 1];
    const int pb = blockIdx.y;
    const int g0 = blockIdx.x * kTSlots * kTGroup;
    const int r = threadIdx.x / 8, part = threadIdx.x % 8;     // 8 threads per position: slots 4 part .. + 3 and 32 + 4 part .. + 3 of a tile
    const int64_t b = (int64_t)pb * kPosBlock + r;
    if (pstat != nullptr && blockIdx.x == 0) {
        // softmax statistics of the logit TARGET rows of this position block, merged once here so that the product
        // kernel and the finish kernel read one (max, sum) pair per row instead of merging the partials in every tile
        SoftStat v;
        v.m = -INFINITY;
        v.s = 0.f;
        if (b < B)
            for (int i = part; i < p_splits; i += 8) v = soft_merge(v, pstat[b * p_splits + i]);
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) {
            SoftStat o;
            o.m = __shfl_xor(v.m, off, kWave);
            o.s = __shfl_xor(v.s, off, kWave);
            v = soft_merge(v, o);
        }
        if (part == 0 && b < B) pmerged[b] = v;
    }
    float qm = 0.f;
    if (QK != RDK_PROB_F32) {
        // row maximum of the logit rows, from the partials of the statistics pass
        float m = -INFINITY;
        if (b < B)
            for (int i = part; i < q_splits; i += 8) m = fmaxf(m, qpart[b * q_splits + i].m);
        m = fmaxf(m, __shfl_xor(m, 1, kWave));
        m = fmaxf(m, __shfl_xor(m, 2, kWave));
        m = fmaxf(m, __shfl_xor(m, 4, kWave));
        qm = m;
    }
    // the row's 512 slots of this workgroup: 8 slots per thread and tile
    float v[kTGroup][8];
    {
        const float fill = QK == RDK_PROB_F32 ? 0.f : -INFINITY;
        float4 raw[kTGroup][2];
#pragma unroll
        for (int t = 0; t < kTGroup; ++t) {
            raw[t][0] = raw[t][1] = make_float4(fill, fill, fill, fill);
            if (b < B) {
                const void *qr = row_ptr<QK>(q, ldq, b);
                const int s = g0 + t * kTSlots + part * 4;   // the eight threads of a row read 128 contiguous bytes per load
                raw[t][0] = load4<QK>(qr, s, n, vec, fill);
                raw[t][1] = load4<QK>(qr, s + 32, n, vec, fill);
            }
        }
        float z = 0.f;
#pragma unroll
        for (int t = 0; t < kTGroup; ++t) {
            const float x[8] = {raw[t][0].x, raw[t][0].y, raw[t][0].z, raw[t][0].w, raw[t][1].x, raw[t][1].y, raw[t][1].z, raw[t][1].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[t][e] = b < B ? to_weight<QK>(x[e], qm, 1.f) : 0.f;
                z += v[t][e];
            }
        }
        z = oct_sum(z);
        if (part == 0 && b < B) zpart[b * zt + blockIdx.x] = z;
    }
    // tile by tile through LDS: 8 threads per slot write 4 positions each (one 128-byte line per slot and store), 32 slots
    // per pass; two tiles alternate, so one barrier per tile
    const int pq = (threadIdx.x % 8) * 4, sl = threadIdx.x / 8;
#pragma unroll
    for (int t = 0; t < kTGroup; ++t) {
        float (*tl)[kPosBlock + 1] = tile[t & 1];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            tl[part * 4 + e][r] = v[t][e];
            tl[32 + part * 4 + e][r] = v[t][4 + e];
        }
        __syncthreads();
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int s = g0 + t * kTSlots + half * 32 + sl;
            if (s < n)
                *(float4 *)(qT + ((int64_t)pb * n + s) * kPosBlock + pq) =
                    make_float4(tl[half * 32 + sl][pq], tl[half * 32 + sl][pq + 1], tl[half * 32 + sl][pq + 2], tl[half * 32 + sl][pq + 3]);
        }
    }
}

// 1 / (sum of the drafter weights of row b) from the partial sums of the transposition (0 for a row without mass), by
// a whole wavefront: lane l adds the partials l, l + 64, ..., then the lanes are added up; the same bits wherever it is
// called.  `first` = partial number lane_id() when the caller fetched it ahead of time.
__device__ __forceinline__ float row_mass_rest(const float *zpart, int zt, int64_t b, float first)
{
    float z = first;
    for (int i = lane_id() + kWave; i < zt; i += kWave) z += zpart[b * zt + i];
    return inv_mass(wave_sum(z));
}

__device__ __forceinline__ float row_mass_inv(const float *zpart, int zt, int64_t b)
{
    return row_mass_rest(zpart, zt, b, lane_id() < zt ? zpart[b * zt + lane_id()] : 0.f);
}

// Broadcast within each group of four lanes: every lane receives the value held by lane `SRC` of its group.
template <int SRC>
__device__ __forceinline__ int quad_bcast(int v)
{
    return __builtin_amdgcn_mov_dpp(v, SRC * 0x55, 0xf, 0xf, true);
}

struct SparseArgs {
    const int32_t *slot_of, *pruned_ids, *kept_ids;
    const int2 *nbr;
    const float *self_w;
    int kk;
    const float *qT;
    const float *zpart;
    int zt;
    int N, n, B;
    int tiles, per_xcd, total_work;
    float *out;
    int64_t ldo;
    bool vec_o;
};

// Number of pruned ids below target id j (j may be N).
__device__ __forceinline__ int pruned_below(const int32_t *slot_of, int j, int N, int n)
{
    if (j >= N) return N - n;
    const int s = slot_of[j];
    return s < 0 ? -s - 1 : j - s;
}

// The product for one workgroup tile, left in `stage[position][id - j0]` (not yet divided by the row
// sums).  Lane layout of a wavefront: lane = 8 * i + o; i = id within a group of 8, o = which four of
// the 32 positions.  One 128-byte line holds the 16 (slot, weight) pairs of a round: lane o of an id's
// group fetches pairs 2o and 2o+1, and the pairs go round the group through the swizzle crossbar.
// The lines of pairs are requested two rounds ahead of the gathers that use them.  The kernel runs at the throughput
// of the CU's vector memory pipe (address and data-return units about 80 % busy); occupancy beyond two workgroups
// per CU does not change its time.
template <int kEllAhead>
__device__ __forceinline__ void sparse_tile(const SparseArgs &a, int pb, int j0, float (*stage)[kStageLd])
{
    const int wid = threadIdx.x / kWave, lane = lane_id();
    const int o = lane & 7, i = lane >> 3;
    const int j1 = min(a.N, j0 + kTileIds);
    const int u_lo = pruned_below(a.slot_of, j0, a.N, a.n), u_hi = pruned_below(a.slot_of, j1, a.N, a.n);
    const int s_lo = j0 - u_lo, s_hi = j1 - u_hi;
    const float *qslab = a.qT + (int64_t)pb * a.n * kPosBlock + o * 4;
    const int rounds = a.kk / 16;
    const int2 *nbr_lane = a.nbr + 2 * o;

    // pruned ids of the tile: pruned slots [u_lo, u_hi), 8 per wavefront step
    int u0 = u_lo + wid * 8;
    // the lines of pairs are requested kEllAhead rounds ahead (a round = 16 neighbours of 8 ids)
    int pf_u = u0, pf_rd = 0;   // where the next request points
    i32x4 evq[kEllAhead];
#pragma unroll
    for (int t = 0; t < kEllAhead; ++t) {
        evq[t] = i32x4{0, 0, 0, 0};
        if (pf_u < u_hi) evq[t] = *((const i32x4 *)(nbr_lane + (int64_t)min(pf_u + i, u_hi - 1) * a.kk + pf_rd * 16));
        if (++pf_rd == rounds) { pf_rd = 0; pf_u += 8 * kWaves; }
    }
    for (; u0 < u_hi; u0 += 8 * kWaves) {
        const int u = u0 + i;
        const bool valid = u < u_hi;
        const int pid = a.pruned_ids[min(u, u_hi - 1)];   // asked for now, needed after the gathers of this step
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int rd = 0; rd < rounds; ++rd) {
            const i32x4 ev = evq[0];
#pragma unroll
            for (int t = 0; t + 1 < kEllAhead; ++t) evq[t] = evq[t + 1];
            if (pf_u < u_hi)
                evq[kEllAhead - 1] = *((const i32x4 *)(nbr_lane + (int64_t)min(pf_u + i, u_hi - 1) * a.kk + pf_rd * 16));
            if (++pf_rd == rounds) { pf_rd = 0; pf_u += 8 * kWaves; }
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float4 g[8];
                float wt[8];
#define RDK_GATHER(T)                                                                                                       \
    {                                                                                                                       \
        const int s_ = half ? __builtin_amdgcn_ds_swizzle(ev[2 * ((T) & 1)], ((4 + ((T) >> 1)) << 5) | 0x18)                \
                            : __builtin_amdgcn_ds_swizzle(ev[2 * ((T) & 1)], (((T) >> 1) << 5) | 0x18);                     \
        wt[T] = __int_as_float(half ? __builtin_amdgcn_ds_swizzle(ev[2 * ((T) & 1) + 1], ((4 + ((T) >> 1)) << 5) | 0x18)    \
                                    : __builtin_amdgcn_ds_swizzle(ev[2 * ((T) & 1) + 1], (((T) >> 1) << 5) | 0x18));        \
        g[T] = *(const float4 *)(qslab + (int64_t)s_ * kPosBlock);                                                          \
    }
                RDK_GATHER(0) RDK_GATHER(1) RDK_GATHER(2) RDK_GATHER(3) RDK_GATHER(4) RDK_GATHER(5) RDK_GATHER(6) RDK_GATHER(7)
#undef RDK_GATHER
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    acc.x += wt[t] * g[t].x; acc.y += wt[t] * g[t].y; acc.z += wt[t] * g[t].z; acc.w += wt[t] * g[t].w;
                }
            }
        }
        if (valid) {
            const int c = pid - j0;
            stage[o * 4 + 0][c] = acc.x;
            stage[o * 4 + 1][c] = acc.y;
            stage[o * 4 + 2][c] = acc.z;
            stage[o * 4 + 3][c] = acc.w;
        }
    }
    // kept ids of the tile: kept slots [s_lo, s_hi) are consecutive rows of the slab
    for (int sb = s_lo + wid * 8; sb < s_hi; sb += 8 * kWaves) {
        const int s = sb + i;
        if (s < s_hi) {
            const float sw = a.self_w[s];
            const float4 g = *(const float4 *)(qslab + (int64_t)s * kPosBlock);
            const int c = a.kept_ids[s] - j0;
            stage[o * 4 + 0][c] = sw * g.x;
            stage[o * 4 + 1][c] = sw * g.y;
            stage[o * 4 + 2][c] = sw * g.z;
            stage[o * 4 + 3][c] = sw * g.w;
        }
    }
    __syncthreads();
}

// Consecutive workgroup ids go to consecutive XCDs; give each XCD one contiguous share of the
// (position block major, id tile minor) work list.
__device__ __forceinline__ bool xcd_work(const SparseArgs &a, int &pb, int &tile)
{
    const int xcd = blockIdx.x % 8, rank = blockIdx.x / 8;
    const int work = xcd * a.per_xcd + rank;
    if (rank >= a.per_xcd || work >= a.total_work) return false;
    pb = work / a.tiles;
    tile = work % a.tiles;
    return true;
}

// What the fused form adds to the product: the target rows, and where the per-block sums go.
struct FuseArgs {
    const void *p;
    int64_t ldp;
    bool vec_p;
    const SoftStat *pstat;             // [B] softmax statistics of the logit target rows, one merged pair per row
    int p_splits;                      // = 1 (the layout the finish kernel expects: partials per row)
    float *part_q, *part_r, *part_a;   // [B, tiles * 4]: one entry per 64-id block
};

// PK = -1: plain product (q' is written).  PK = -2: also the sum of q' per 64-id block (draft draw without a
// target row; q' written only if WRITE_Q).  PK >= 0: fused with the verification sums against the target
// rows of kind PK -- per (position, 64-id block) the sums of q', max(0, p - q') and min(p, q') --
// and q' is written only if WRITE_Q.
template <int PK, bool WRITE_Q>
__global__ __launch_bounds__(kThreads) void sparse_product_kernel(SparseArgs a, FuseArgs f)
{
    constexpr bool FUSE = PK >= 0, SUMS = PK != -1;
    constexpr int PKIND = FUSE ? PK : RDK_PROB_F32;
    __shared__ __attribute__((aligned(16))) float stage[kPosBlock][kStageLd];
    int pb, tile;
    if (!xcd_work(a, pb, tile)) return;
    const int j0 = tile * kTileIds;
    // each wavefront finishes 4 of the 32 rows; a lane holds the ids j0 + 4 lane .. + 3 (one 16-byte access per row
    // for the target values, for the staged q' and for the store).  The target values are requested before the
    // gathers start.
    const int wid = threadIdx.x / kWave, lane = lane_id();
    constexpr int kRowsPerWave = kPosBlock / kWaves;
    const float pfill = PKIND == RDK_PROB_F32 ? 0.f : -INFINITY;
    const int jl = j0 + 4 * lane;
    float4 praw[kRowsPerWave];
    // every lane's four ids exist (all tiles but the last): decided for the whole workgroup, so that the loads and
    // stores of the common case sit behind no per-lane branch
    const bool whole_tile = j0 + kTileIds <= a.N;
    if (FUSE) {
#pragma unroll
        for (int rr = 0; rr < kRowsPerWave; ++rr) {
            const int64_t b = (int64_t)pb * kPosBlock + wid * kRowsPerWave + rr;
            // streamed past the caches' replacement order: the L2 of this XCD should keep the drafter slab instead
            if (b >= a.B)
                praw[rr] = make_float4(pfill, pfill, pfill, pfill);
            else if (f.vec_p && whole_tile)
                praw[rr] = load4_full<PKIND, true>(row_ptr<PKIND>(f.p, f.ldp, b), jl);
            else
                praw[rr] = load4<PKIND>(row_ptr<PKIND>(f.p, f.ldp, b), jl, a.N, f.vec_p, pfill);
        }
    }
    // Eq. 1: the row sums of the four rows this wavefront finishes, from the partials of the transposition (asked for now)
    float zfirst[kRowsPerWave];
#pragma unroll
    for (int rr = 0; rr < kRowsPerWave; ++rr) {
        const int64_t b = (int64_t)pb * kPosBlock + wid * kRowsPerWave + rr;
        zfirst[rr] = (b < a.B && lane < a.zt) ? a.zpart[b * a.zt + lane] : 0.f;
    }
    // rounds of neighbour pairs requested ahead of their gathers: two when the target rows stream through the same
    // memory pipe (105 against 108 us per launch), one otherwise (92 against 99 us)
    sparse_tile<(PK >= 0 ? 2 : 1)>(a, pb, j0, stage);
#pragma unroll
    for (int rr = 0; rr < kRowsPerWave; ++rr) {
        const int r = wid * kRowsPerWave + rr;
        const int64_t b = (int64_t)pb * kPosBlock + r;
        if (b >= a.B) break;
        const float inv_z = row_mass_rest(a.zpart, a.zt, b, zfirst[rr]);
        const float4 sv = *(const float4 *)&stage[r][4 * lane];
        const float qv[4] = {jl + 0 < a.N ? sv.x * inv_z : 0.f, jl + 1 < a.N ? sv.y * inv_z : 0.f,
                             jl + 2 < a.N ? sv.z * inv_z : 0.f, jl + 3 < a.N ? sv.w * inv_z : 0.f};
        if (WRITE_Q) {
            float *o = a.out + b * a.ldo + jl;
            if (a.vec_o && whole_tile) {
                const f32x4 v = {qv[0], qv[1], qv[2], qv[3]};
                __builtin_nontemporal_store(v, (f32x4 *)o);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (jl + e < a.N) o[e] = qv[e];
            }
        }
        if (SUMS) {
            float m = 0.f, inv = 1.f;
            if (FUSE && PKIND != RDK_PROB_F32) {
                const SoftStat rs = f.pstat[b];   // merged by the transposition kernel
                m = rs.m;
                inv = 1.0f / rs.s;
            }
            float sq = 0.f, sr = 0.f, sa = 0.f;
            if (FUSE) {
                const float pr4[4] = {praw[rr].x, praw[rr].y, praw[rr].z, praw[rr].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float pe = to_weight<PKIND>(pr4[e], m, inv);
                    sq += qv[e];
                    sr += fmaxf(pe - qv[e], 0.f);
                    sa += fminf(pe, qv[e]);
                }
            } else {
                sq = ((qv[0] + qv[1]) + qv[2]) + qv[3];   // the order of the fused form: same block sums, same drafts
            }
            // one block of sums per 16 lanes (64 ids): reduce inside each row of the wavefront only
            sq = row16_sum(sq);
            if (FUSE) {
                sr = row16_sum(sr);
                sa = row16_sum(sa);
            }
            if ((lane & 15) == 0) {
                const int64_t o = b * ((int64_t)a.tiles * (kTileIds / kSubIds)) + tile * (kTileIds / kSubIds) + (lane >> 4);
                f.part_q[o] = sq;
                if (FUSE) {
                    f.part_r[o] = sr;
                    f.part_a[o] = sa;
                }
            }
        }
    }
}

// q' of one position recomputed from the sparse kernel (the finalize step needs two 64-id blocks of it).
struct QpSparse {
    static constexpr bool kSpreadRows = true;
    static constexpr int kStages = 3;
    SparseArgs a;
    struct Row {
        const int32_t *slot_of;
        const int2 *nbr;
        const float *self_w;
        int kk, N;
        const float *qcol;   // qT + (pb * n) * 32 + r : element of slot s is qcol[s * 32]
        float inv_z;
        __device__ __forceinline__ float value(int j) const
        {
            if (j >= N) return 0.f;
            const int s = slot_of[j];
            if (s >= 0) return self_w[s] * qcol[(int64_t)s * kPosBlock] * inv_z;
            const int64_t u = -s - 1;
            float acc = 0.f;
            for (int t0 = 0; t0 < kk; t0 += 2) {   // same order of additions as the product kernel
                const int4 ev = *(const int4 *)(nbr + u * kk + t0);
                acc += __int_as_float(ev.y) * qcol[(int64_t)ev.x * kPosBlock];
                acc += __int_as_float(ev.w) * qcol[(int64_t)ev.z * kPosBlock];
            }
            return acc * inv_z;
        }
        // Four consecutive ids in three steps: slots; the first sixteen table entries of each id (a kept id is
        // treated as a row whose entries all point at its own slot, the first with the diagonal weight); the
        // gathers.  Rows longer than sixteen entries are finished round by round in result().
        struct Pending {
            int se[4];
            int ii[4][16];
            float ww[4][16], gg[4][16];
        };
        template <int K>
        __device__ __forceinline__ void stage(Pending &t, int64_t idx) const
        {
            if (K == 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e) t.se[e] = idx + e < N ? slot_of[idx + e] : 0;   // beyond N: computed, discarded
            } else if (K == 1) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int s = t.se[e];
                    const bool kept = s >= 0;
                    const int64_t u = kept ? 0 : -s - 1;
#pragma unroll
                    for (int x = 0; x < 16; x += 2) {
                        const int4 ev = *(const int4 *)(nbr + u * kk + x);
                        t.ii[e][x] = ev.x; t.ww[e][x] = __int_as_float(ev.y);
                        t.ii[e][x + 1] = ev.z; t.ww[e][x + 1] = __int_as_float(ev.w);
                    }
                    const float sw = self_w[max(s, 0)];
                    if (kept) {
#pragma unroll
                        for (int x = 0; x < 16; ++x) {
                            t.ii[e][x] = s;
                            t.ww[e][x] = x == 0 ? sw : 0.f;
                        }
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int x = 0; x < 16; ++x) t.gg[e][x] = qcol[(int64_t)t.ii[e][x] * kPosBlock];
            }
        }
        // The record is reused for the rounds beyond the first: all pairs of a round for the four ids, then all their
        // gathers, then the sums -- two round trips per round, whatever the number of ids.  A kept id takes its own
        // slot with zero weights there (its row has the diagonal only).
        __device__ __forceinline__ float4 result(Pending &t, int64_t idx) const
        {
            float acc[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[e] = 0.f;
#pragma unroll
                for (int x = 0; x < 16; ++x) acc[e] += t.ww[e][x] * t.gg[e][x];   // same order of additions as the product kernel
            }
            for (int x0 = 16; x0 < kk; x0 += 16) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool kept = t.se[e] >= 0;
                    const int64_t u = kept ? 0 : -t.se[e] - 1;
#pragma unroll
                    for (int x = 0; x < 16; x += 2) {
                        const int4 ev = *(const int4 *)(nbr + u * kk + x0 + x);
                        t.ii[e][x] = kept ? t.se[e] : ev.x; t.ww[e][x] = kept ? 0.f : __int_as_float(ev.y);
                        t.ii[e][x + 1] = kept ? t.se[e] : ev.z; t.ww[e][x + 1] = kept ? 0.f : __int_as_float(ev.w);
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int x = 0; x < 16; ++x) t.gg[e][x] = qcol[(int64_t)t.ii[e][x] * kPosBlock];
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int x = 0; x < 16; ++x) acc[e] += t.ww[e][x] * t.gg[e][x];
            }
            float out[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = idx + e < N ? acc[e] * inv_z : 0.f;
            return make_float4(out[0], out[1], out[2], out[3]);
        }
        // One id per lane (blocks of 64 ids): the slot, then the first sixteen table entries, then their gathers; a kept
        // id is a row whose entries all point at its own slot, the first with the diagonal weight.
        struct Pending1 {
            int se;
            int ii[16];
            float ww[16], gg[16];
        };
        template <int K>
        __device__ __forceinline__ void stage1(Pending1 &t, int64_t idx) const
        {
            if (K == 0) {
                t.se = idx < N ? slot_of[idx] : 0;   // beyond N: computed, discarded
            } else if (K == 1) {
                const int s = t.se;
                const bool kept = s >= 0;
                const int64_t u = kept ? 0 : -s - 1;
#pragma unroll
                for (int x = 0; x < 16; x += 2) {
                    const int4 ev = *(const int4 *)(nbr + u * kk + x);
                    t.ii[x] = ev.x; t.ww[x] = __int_as_float(ev.y);
                    t.ii[x + 1] = ev.z; t.ww[x + 1] = __int_as_float(ev.w);
                }
                const float sw = self_w[max(s, 0)];
                if (kept) {
#pragma unroll
                    for (int x = 0; x < 16; ++x) {
                        t.ii[x] = s;
                        t.ww[x] = x == 0 ? sw : 0.f;
                    }
                }
            } else {
#pragma unroll
                for (int x = 0; x < 16; ++x) t.gg[x] = qcol[(int64_t)t.ii[x] * kPosBlock];
            }
        }
        __device__ __forceinline__ float result1(Pending1 &t, int64_t idx) const
        {
            float acc = 0.f;
#pragma unroll
            for (int x = 0; x < 16; ++x) acc += t.ww[x] * t.gg[x];   // same order of additions as the product kernel
            const bool kept = t.se >= 0;
            const int64_t u = kept ? 0 : -t.se - 1;
            for (int x0 = 16; x0 < kk; x0 += 16) {
#pragma unroll
                for (int x = 0; x < 16; x += 2) {
                    const int4 ev = *(const int4 *)(nbr + u * kk + x0 + x);
                    t.ii[x] = kept ? t.se : ev.x; t.ww[x] = kept ? 0.f : __int_as_float(ev.y);
                    t.ii[x + 1] = kept ? t.se : ev.z; t.ww[x + 1] = kept ? 0.f : __int_as_float(ev.w);
                }
#pragma unroll
                for (int x = 0; x < 16; ++x) t.gg[x] = qcol[(int64_t)t.ii[x] * kPosBlock];
#pragma unroll
                for (int x = 0; x < 16; ++x) acc += t.ww[x] * t.gg[x];
            }
            return idx < N ? acc * inv_z : 0.f;
        }
        __device__ __forceinline__ float load1(int j) const { return value(j); }
    };
    __device__ __forceinline__ Row row(int64_t b) const
    {
        const int pb = (int)(b / kPosBlock), r = (int)(b % kPosBlock);
        return Row{a.slot_of, a.nbr, a.self_w, a.kk, a.N, a.qT + (int64_t)pb * a.n * kPosBlock + r, row_mass_inv(a.zpart, a.zt, b)};
    }
};

struct SparseFusedWs {
    SparseWs base;
    SoftStat *pstat;
    float *part_q, *part_r, *part_a;
    int p_splits;
};

size_t fused_extra_bytes(const KernelHandle &h, int32_t B)
{
    const size_t blocks = (size_t)((h.N + kTileIds - 1) / kTileIds) * (kTileIds / kSubIds);
    return align_up((size_t)B * kMaxSplits * sizeof(SoftStat), 256) + align_up((size_t)B * sizeof(SoftStat), 256) +
           3 * align_up((size_t)B * blocks * sizeof(float), 256);
}

SparseArgs make_args(const KernelHandle &h, const SparseWs &w, int32_t B, float *out, int64_t ldo)
{
    SparseArgs a;
    a.slot_of = h.slot_of; a.pruned_ids = h.pruned_ids; a.kept_ids = h.kept_ids; a.nbr = h.nbr;
    a.self_w = h.self_w; a.kk = h.kk;
    a.qT = w.qT; a.zpart = w.zpart; a.zt = w.zt;
    a.N = h.N; a.n = h.n; a.B = B;
    const int pbs = (B + kPosBlock - 1) / kPosBlock;
    a.tiles = (h.N + kTileIds - 1) / kTileIds;
    a.total_work = pbs * a.tiles;
    a.per_xcd = (a.total_work + 7) / 8;
    a.out = out; a.ldo = ldo; a.vec_o = out ? rows_vectorisable(out, ldo, RDK_PROB_F32) : false;
    return a;
}

template <int QK>
rdk_status_t prepare_q(const KernelHandle &h, RowInput q, int32_t B, const SparseWs &w, hipStream_t st,
                       const SoftStat *pstat = nullptr, int p_splits = 0, SoftStat *pmerged = nullptr)
{
    if (QK != RDK_PROB_F32) {   // logit rows: the row maxima first; probability rows are summed by the transposition itself
        const rdk_status_t rc = launch_row_stats<QK>(q, h.n, B, w.q_splits, w.qpart, st);
        if (rc != RDK_OK) return rc;
    }
    const int pbs = (B + kPosBlock - 1) / kPosBlock;
    {
        RDK_TIMED_LAUNCH("q_transpose_kernel", (q_transpose_kernel<QK>), dim3(w.zt, pbs), dim3(kPrepThreads), 0, st,
                         q.ptr, q.ld, h.n, B, w.qpart, w.q_splits, rows_vectorisable(q.ptr, q.ld, q.kind), w.zpart, w.zt, w.qT, pstat, p_splits,
                         pmerged);
    }
    RDK_LAUNCH_CHECK("q_transpose_kernel");
    return RDK_OK;
}

template <int QK>
rdk_status_t run_sparse(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws, hipStream_t st)
{
    SparseWs w = carve(h, B, ws);
    rdk_status_t rc = prepare_q<QK>(h, q, B, w, st);
    if (rc != RDK_OK) return rc;
    const SparseArgs a = make_args(h, w, B, out, ldo);
    {
        RDK_TIMED_LAUNCH("sparse_product_kernel", (sparse_product_kernel<-1, true>), dim3(8 * a.per_xcd), dim3(kThreads), 0, st,
                         a, FuseArgs{});
    }
    RDK_LAUNCH_CHECK("sparse_product_kernel");
    return RDK_OK;
}

template <int PK, int QK>
rdk_status_t run_sparse_fused(const KernelHandle &h, const FusedCall &c, void *ws, hipStream_t st)
{
    const int32_t B = c.d.B;
    SparseWs w = carve(h, B, ws);
    char *p = (char *)ws + sparse_workspace_bytes(h, B);
    FuseArgs f{};
    f.p = c.p.ptr; f.ldp = c.p.ld; f.vec_p = rows_vectorisable(c.p.ptr, c.p.ld, c.p.kind);
    const int p_splits = row_splits(B, h.N, kStatThreads / kWave);
    SoftStat *ppart = (SoftStat *)p; p += align_up((size_t)B * kMaxSplits * sizeof(SoftStat), 256);   // partials per split
    SoftStat *pmerged = (SoftStat *)p; p += align_up((size_t)B * sizeof(SoftStat), 256);              // one per row
    f.pstat = pmerged;
    f.p_splits = 1;
    const size_t blocks = (size_t)((h.N + kTileIds - 1) / kTileIds) * (kTileIds / kSubIds);
    const size_t per = align_up((size_t)B * blocks * sizeof(float), 256);
    f.part_q = (float *)p; p += per;
    f.part_r = (float *)p; p += per;
    f.part_a = (float *)p;
    rdk_status_t rc;
    if (PK != RDK_PROB_F32) {
        rc = launch_row_stats<PK>(c.p, h.N, B, p_splits, ppart, st);
        if (rc != RDK_OK) return rc;
    }
    rc = PK != RDK_PROB_F32 ? prepare_q<QK>(h, c.q, B, w, st, ppart, p_splits, pmerged) : prepare_q<QK>(h, c.q, B, w, st);
    if (rc != RDK_OK) return rc;
    const SparseArgs a = make_args(h, w, B, c.q_prime, c.ldo);
    {
        if (c.q_prime)
            RDK_TIMED_LAUNCH("sparse_product_kernel", (sparse_product_kernel<PK, true>), dim3(8 * a.per_xcd), dim3(kThreads), 0,
                             st, a, f);
        else
            RDK_TIMED_LAUNCH("sparse_product_kernel", (sparse_product_kernel<PK, false>), dim3(8 * a.per_xcd), dim3(kThreads),
                             0, st, a, f);
    }
    RDK_LAUNCH_CHECK("sparse_product_kernel");
    FinalizeArgs fa{};
    fa.d = c.d;
    fa.p = c.p.ptr; fa.ldp = c.p.ld; fa.vec_p = f.vec_p;
    fa.pstat = f.pstat; fa.p_splits = f.p_splits;
    fa.part_q = f.part_q; fa.part_r = f.part_r; fa.part_a = f.part_a;
    fa.nblk = (int)blocks;
    fa.draft_ids = c.draft_ids; fa.accept = c.accept; fa.alpha = c.alpha; fa.resid_mass = c.resid_mass;
    fa.resid_ids = c.resid_ids; fa.n_accepted = c.n_accepted; fa.out_tokens = c.out_tokens;
    return launch_finalize<PK, kSubIds, true, QpSparse>(fa, QpSparse{a}, st);
}

template <int QK>
rdk_status_t run_sparse_draft(const KernelHandle &h, RowInput q, int32_t B, uint64_t seed, uint64_t offset, int32_t *draft_ids,
                              float *q_draft, float *q_prime, int64_t ldo, void *ws, hipStream_t st)
{
    SparseWs w = carve(h, B, ws);
    FuseArgs f{};
    f.part_q = (float *)((char *)ws + sparse_workspace_bytes(h, B));
    rdk_status_t rc = prepare_q<QK>(h, q, B, w, st);
    if (rc != RDK_OK) return rc;
    const SparseArgs a = make_args(h, w, B, q_prime, ldo);
    if (q_prime)
        RDK_TIMED_LAUNCH("sparse_product_kernel", (sparse_product_kernel<-2, true>), dim3(8 * a.per_xcd), dim3(kThreads), 0, st,
                         a, f);
    else
        RDK_TIMED_LAUNCH("sparse_product_kernel", (sparse_product_kernel<-2, false>), dim3(8 * a.per_xcd), dim3(kThreads), 0,
                         st, a, f);
    RDK_LAUNCH_CHECK("sparse_product_kernel");
    const int blocks = a.tiles * (kTileIds / kSubIds);
    DraftArgs da{B, h.N, seed, offset, f.part_q, blocks, draft_ids, q_draft};
    return launch_draft_finalize<kSubIds, QpSparse>(da, QpSparse{a}, st);
}

}  // namespace

size_t sparse_draft_workspace_bytes(const KernelHandle &h, int32_t B)
{
    const size_t blocks = (size_t)((h.N + kTileIds - 1) / kTileIds) * (kTileIds / kSubIds);
    return sparse_workspace_bytes(h, B) + align_up((size_t)B * blocks * sizeof(float), 256);
}

rdk_status_t launch_sparse_draft(const KernelHandle &h, RowInput q, int32_t B, uint64_t seed, uint64_t offset, int32_t *draft_ids,
                                 float *q_draft, float *q_prime, int64_t ldo, void *ws, hipStream_t st)
{
    switch (q.kind) {
        case RDK_PROB_F32: return run_sparse_draft<RDK_PROB_F32>(h, q, B, seed, offset, draft_ids, q_draft, q_prime, ldo, ws, st);
        case RDK_LOGIT_F32: return run_sparse_draft<RDK_LOGIT_F32>(h, q, B, seed, offset, draft_ids, q_draft, q_prime, ldo, ws, st);
        case RDK_LOGIT_BF16: return run_sparse_draft<RDK_LOGIT_BF16>(h, q, B, seed, offset, draft_ids, q_draft, q_prime, ldo, ws, st);
    }
    return RDK_ERR_DTYPE;
}

size_t sparse_workspace_bytes(const KernelHandle &h, int32_t B)
{
    const size_t pbs = (B + kPosBlock - 1) / kPosBlock;
    const size_t zt = (h.n + kTSlots * kTGroup - 1) / (kTSlots * kTGroup);
    return align_up((size_t)B * kMaxSplits * sizeof(SoftStat), 256) + align_up((size_t)B * zt * sizeof(float), 256) +
           align_up(pbs * h.n * kPosBlock * sizeof(float), 256);
}

size_t sparse_fused_workspace_bytes(const KernelHandle &h, int32_t B) { return sparse_workspace_bytes(h, B) + fused_extra_bytes(h, B); }

rdk_status_t launch_sparse(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws, hipStream_t st)
{
    switch (q.kind) {
        case RDK_PROB_F32: return run_sparse<RDK_PROB_F32>(h, q, B, out, ldo, ws, st);
        case RDK_LOGIT_F32: return run_sparse<RDK_LOGIT_F32>(h, q, B, out, ldo, ws, st);
        case RDK_LOGIT_BF16: return run_sparse<RDK_LOGIT_BF16>(h, q, B, out, ldo, ws, st);
    }
    return RDK_ERR_DTYPE;
}

rdk_status_t launch_sparse_fused(const KernelHandle &h, const FusedCall &c, void *ws, hipStream_t st)
{
#define RDK_F(PK, QK) \
    if (c.p.kind == PK && c.q.kind == QK) return run_sparse_fused<PK, QK>(h, c, ws, st);
    RDK_F(RDK_PROB_F32, RDK_PROB_F32)
    RDK_F(RDK_PROB_F32, RDK_LOGIT_F32)
    RDK_F(RDK_PROB_F32, RDK_LOGIT_BF16)
    RDK_F(RDK_LOGIT_F32, RDK_PROB_F32)
    RDK_F(RDK_LOGIT_F32, RDK_LOGIT_F32)
    RDK_F(RDK_LOGIT_F32, RDK_LOGIT_BF16)
    RDK_F(RDK_LOGIT_BF16, RDK_PROB_F32)
    RDK_F(RDK_LOGIT_BF16, RDK_LOGIT_F32)
    RDK_F(RDK_LOGIT_BF16, RDK_LOGIT_BF16)
#undef RDK_F
    return RDK_ERR_DTYPE;
}

}  // namespace rdk
