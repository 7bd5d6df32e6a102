// Exact redistribution (Alg. 1, step 2):  P'[b, j] = sum_s Q'[b, s] M[s, j]  with a dense kernel M.
//   fp32 kernel:  LDS-tiled fp32 FMA product, split over the kept slots, fixed-order reduction.
//   bf16 kernel:  both operands rounded to bf16, fp32 accumulation on the matrix cores
//                 (v_mfma_f32_32x32x16_bf16), rows rescaled so that they sum to one.
// Step 1 (Eq. 1) is folded in: rows of Q' are the drafter rows divided by their sums.
#include "rdk_rowstats.hpp"

namespace rdk {

namespace {

// ------------------------------------------------------------------------------------------------ fp32
constexpr int kColsF = 128;   // columns (target ids) per workgroup
constexpr int kRowsF = 64;    // positions per workgroup
constexpr int kDepthF = 32;   // kept slots per LDS stage

template <int QK>
__global__ __launch_bounds__(256) void exact_f32_kernel(const void *q, int64_t ldq, const SoftStat *qstat, const float *M,
                                                        int64_t ldm, int n, int N, int B, int slots_per_split,
                                                        float *dst, int64_t ldd, int64_t split_stride, bool scale_here)
{
    __shared__ float Qs[kDepthF][kRowsF + 4];
    __shared__ float Ms[kDepthF][kColsF + 4];
    const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;
    const int j0 = blockIdx.x * kColsF, b0 = blockIdx.y * kRowsF;
    const int s_begin = blockIdx.z * slots_per_split, s_end = min(n, s_begin + slots_per_split);
    float acc[8][4];
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;

    // loader roles
    const int q_row = threadIdx.x / 4, q_k0 = (threadIdx.x % 4) * 8;   // 64 rows x 32 slots: 8 slots per thread
    const void *qr = (b0 + q_row < B) ? row_ptr<QK>(q, ldq, b0 + q_row) : nullptr;
    const float qm = (qr && QK != RDK_PROB_F32) ? qstat[b0 + q_row].m : 0.f;

    for (int s0 = s_begin; s0 < s_end; s0 += kDepthF) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int s = s0 + q_k0 + e;
            Qs[q_k0 + e][q_row] = (qr && s < s_end) ? to_weight<QK>(load1<QK>(qr, s), qm, 1.f) : 0.f;
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int f = it * 256 + threadIdx.x;           // float4 index in the 32 x 128 tile
            const int kr = f / (kColsF / 4), c4 = (f % (kColsF / 4)) * 4;
            const int s = s0 + kr;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (s < s_end) {
                const float *src = M + (int64_t)s * ldm + j0 + c4;
                if (j0 + c4 + 3 < N && (ldm % 4 == 0)) {
                    v = *(const float4 *)src;
                } else {
                    if (j0 + c4 + 0 < N) v.x = src[0];
                    if (j0 + c4 + 1 < N) v.y = src[1];
                    if (j0 + c4 + 2 < N) v.z = src[2];
                    if (j0 + c4 + 3 < N) v.w = src[3];
                }
            }
            *(float4 *)&Ms[kr][c4] = v;
        }
        __syncthreads();
#pragma unroll 8
        for (int kq = 0; kq < kDepthF; ++kq) {
            const float4 mv = *(const float4 *)&Ms[kq][tx * 4];
            const float4 qa = *(const float4 *)&Qs[kq][ty * 8];
            const float4 qb = *(const float4 *)&Qs[kq][ty * 8 + 4];
            const float qv[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                acc[r][0] += qv[r] * mv.x;
                acc[r][1] += qv[r] * mv.y;
                acc[r][2] += qv[r] * mv.z;
                acc[r][3] += qv[r] * mv.w;
            }
        }
    }
    float *base = dst + (int64_t)blockIdx.z * split_stride;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int b = b0 + ty * 8 + r;
        if (b >= B) continue;
        const float sc = scale_here ? 1.0f / qstat[b].s : 1.f;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int j = j0 + tx * 4 + c;
            if (j < N) base[(int64_t)b * ldd + j] = acc[r][c] * sc;
        }
    }
}

// Sum of the split partials in split order, divided by the drafter row sum (Eq. 1).
__global__ void exact_reduce_kernel(const float *part, int64_t ldd, int64_t split_stride, int splits, const SoftStat *qstat,
                                    int N, float *out, int64_t ldo)
{
    const int b = blockIdx.y;
    const float sc = 1.0f / qstat[b].s;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < N; j += (int64_t)gridDim.x * blockDim.x) {
        float s = 0.f;
        for (int z = 0; z < splits; ++z) s += part[(int64_t)z * split_stride + (int64_t)b * ldd + j];
        out[(int64_t)b * ldo + j] = s * sc;
    }
}

// ------------------------------------------------------------------------------------------------ bf16
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kKStep = 16;          // kept slots per MFMA (32x32x16)
constexpr int kColBlock = 32;       // target ids per MFMA tile
constexpr int kColBlocksPerWg = 4;  // 128 target ids per workgroup

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)(u >> 16);   // inf / nan pass through
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Packed layout of the bf16 kernel: for column block jb (32 ids) and slot block kb (16 slots) one
// contiguous 1 KB record holding, for lane l = 32 * g + c (g = 0..1, c = 0..31), the eight values
// M[kb*16 + g*8 + e, jb*32 + c], e = 0..7 -- exactly the B operand of one 32x32x16 MFMA, so that a
// wavefront fetches it with a single 16-byte-per-lane load.  Records of one jb are consecutive in kb.
__global__ void pack_bf16_kernel(const float *M, int64_t ldm, int n, int N, int KB, uint16_t *packed)
{
    const int jb = blockIdx.x, lane = threadIdx.x;
    const int g = lane / 32, c = lane % 32;
    const int j = jb * kColBlock + c;
    for (int kb = blockIdx.y; kb < KB; kb += gridDim.y) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const int s = kb * kKStep + g * 8 + e;
            const float v0 = (s < n && j < N) ? M[(int64_t)s * ldm + j] : 0.f;
            const float v1 = (s + 1 < n && j < N) ? M[(int64_t)(s + 1) * ldm + j] : 0.f;
            w[e / 2] = (uint32_t)f32_to_bf16_rne(v0) | ((uint32_t)f32_to_bf16_rne(v1) << 16);
        }
        *(uint4 *)(packed + (((int64_t)jb * KB + kb) * 64 + lane) * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// fp32 sums of the bf16-rounded rows of M (needed to rescale output rows to unit mass).
__global__ void rounded_row_sum_kernel(const float *M, int64_t ldm, int N, float *row_sum)
{
    const int s = blockIdx.x;
    double sum = 0.0;
    for (int j = threadIdx.x; j < N; j += blockDim.x)
        sum += (double)bf16_to_f32(f32_to_bf16_rne(M[(int64_t)s * ldm + j]));
    sum = wave_sum(sum);
    __shared__ double sh[4];
    if (lane_id() == 0) sh[threadIdx.x / kWave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) row_sum[s] = (float)((sh[0] + sh[1]) + (sh[2] + sh[3]));
}

__global__ void unpack_bf16_kernel(const uint16_t *packed, int n, int N, int KB, float *M, int64_t ldm)
{
    const int jb = blockIdx.x, lane = threadIdx.x;
    const int g = lane / 32, c = lane % 32;
    const int j = jb * kColBlock + c;
    if (j >= N) return;
    for (int kb = blockIdx.y; kb < KB; kb += gridDim.y) {
        const uint16_t *rec = packed + (((int64_t)jb * KB + kb) * 64 + lane) * 8;
        for (int e = 0; e < 8; ++e) {
            const int s = kb * kKStep + g * 8 + e;
            if (s < n) M[(int64_t)s * ldm + j] = bf16_to_f32(rec[e]);
        }
    }
}

// A operand: TLI-normalised drafter rows rounded to bf16, packed like M: for row block rb (32 positions) and
// slot block kb (16 slots) one 1 KB record holding, for lane l = 32 * g + r, the eight values
// q'[rb*32 + r, kb*16 + g*8 + e], e = 0..7 -- the A operand of one 32x32x16 MFMA.  Also per row the factor
// 1 / sum_s bf16(q'_s) * row_sum[s], which makes the output row sum to one.  One workgroup per position.
template <int QK>
__global__ __launch_bounds__(256) void prep_a_bf16_kernel(const void *q, int64_t ldq, const SoftStat *qstat, const float *row_sum,
                                                          int n, int KB, int B, uint16_t *Ap, float *out_scale)
{
    const int b = blockIdx.x;
    const int rb = b / 32, r = b % 32;
    double mass = 0.0;
    const void *qr = b < B ? row_ptr<QK>(q, ldq, b) : nullptr;
    const float qm = b < B ? qstat[b].m : 0.f, inv = b < B ? 1.0f / qstat[b].s : 0.f;
    for (int c = threadIdx.x; c < KB * 2; c += blockDim.x) {   // chunk of 8 consecutive slots
        const int kb = c / 2, g = c % 2;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (qr) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int s = c * 8 + e;
                uint16_t h = 0;
                if (s < n) {
                    h = f32_to_bf16_rne(to_weight<QK>(load1<QK>(qr, s), qm, 1.f) * inv);
                    mass += (double)bf16_to_f32(h) * (double)row_sum[s];
                }
                w[e / 2] |= (uint32_t)h << (16 * (e % 2));
            }
        }
        *(uint4 *)(Ap + (((int64_t)rb * KB + kb) * 64 + g * 32 + r) * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    mass = wave_sum(mass);
    __shared__ double sh[4];
    if (lane_id() == 0) sh[threadIdx.x / kWave] = mass;
    __syncthreads();
    if (threadIdx.x == 0 && b < B) out_scale[b] = (float)(1.0 / ((sh[0] + sh[1]) + (sh[2] + sh[3])));
}

// P'[512 x 128] per workgroup: W wavefronts, wavefront w owns RB row blocks (32 positions each) and all four
// column blocks (32 target ids each) of the workgroup's column group, i.e. RB x 4 accumulator tiles of
// 32 x 32 fp32.  The kept slots are walked in stages of 64 (four MFMA steps):
//   * A records come straight from global memory (L2-resident: every workgroup walks the slots at the same pace),
//   * the 16 B records of a stage are fetched once per workgroup, parked in LDS (double buffered) and read by all
//     wavefronts: the vector memory pipe of a CU could not feed every wavefront its own copy;
//   * requests run two (A) and three (B) stages ahead of the MFMAs; large batches use one wavefront per SIMD with
//     the whole register file (accumulators in the AGPR half), which halves the LDS reads per MFMA.
// M is streamed from HBM exactly once when all positions fit one row of workgroups (B <= 512).
template <int W, int RB>
__global__ __launch_bounds__(W * 64) void exact_bf16_kernel(const uint16_t *Ap, const uint16_t *Mp, int KB, int N, int B,
                                                            const float *out_scale, float *out, int64_t ldo)
{
    constexpr int RPW = 16 / W;   // B records a wavefront fetches per stage
    __shared__ bf16x8 bbuf[2][16][64];
    const int wid = threadIdx.x / kWave, lane = lane_id();
    const int jb0 = blockIdx.x * kColBlocksPerWg;
    const int rb0 = (blockIdx.y * W + wid) * RB;
    const int n_jb = (N + kColBlock - 1) / kColBlock;
    const int stages = KB / 4;
    f32x16 acc[RB][kColBlocksPerWg];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int c = 0; c < kColBlocksPerWg; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;

    const bf16x8 *a_ptr[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) a_ptr[r] = (const bf16x8 *)Ap + ((int64_t)(rb0 + r) * KB) * 64 + lane;
    const bf16x8 *b_src[RPW];
    int b_rec[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        b_rec[i] = wid * RPW + i;                               // record = jb * 4 + kb within the stage
        const int jb = min(jb0 + b_rec[i] / 4, n_jb - 1);       // surplus column blocks recompute the last one
        b_src[i] = (const bf16x8 *)Mp + ((int64_t)jb * KB + b_rec[i] % 4) * 64 + lane;
    }
    // Loads return to a wavefront in issue order, so every load inherits the latency of the slowest one before
    // it.  The B records come from HBM: they are requested three stages ahead and kept in a ring of registers.
    // The A records (L2) are requested two stages ahead, block by block as their registers fall free; the only
    // B request older than an A record at the time it is needed is then two whole stages old.
    bf16x8 a_even[RB][4], a_odd[RB][4], b_ring[3][RPW];
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
        for (int i = 0; i < RPW; ++i) b_ring[t][i] = b_src[i][(int64_t)min(t, stages - 1) * 4 * 64];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            a_even[r][kb] = a_ptr[r][kb * 64];
            a_odd[r][kb] = a_ptr[r][((int64_t)min(1, stages - 1) * 4 + kb) * 64];
        }
#pragma unroll
    for (int i = 0; i < RPW; ++i) bbuf[0][b_rec[i]][lane] = b_ring[0][i];
    __syncthreads();

    // One stage.  SLOT = s % 3 is the ring entry free for the B request three stages ahead.  ACUR holds the A
    // records of this stage; as soon as the MFMAs of one slot block are issued, its registers take the request
    // for the same block TWO stages ahead (even and odd stages own one register set each), so twice as many A
    // bytes are in flight as with whole-stage double buffering.  All indices are clamped: no branches.
#define RDK_STAGE(SLOT, ACUR)                                                                                        \
    {                                                                                                                \
        const int cur = s & 1;                                                                                       \
        const int64_t sa = min(s + 2, stages - 1), sb = min(s + 3, stages - 1);                                      \
        _Pragma("unroll") for (int i = 0; i < RPW; ++i) b_ring[SLOT][i] = b_src[i][sb * 4 * 64];                     \
        __builtin_amdgcn_sched_barrier(0);                                                                           \
        bf16x8 bq[3];                        /* B fragments are read from LDS two MFMA groups ahead */               \
        bq[0] = bbuf[cur][0][lane];                                                                                  \
        bq[1] = bbuf[cur][4][lane];                                                                                  \
        _Pragma("unroll") for (int f = 0; f < 16; ++f) {     /* f = kb * 4 + c */                                    \
            const int kb = f / 4, c = f % 4;                                                                         \
            if (f + 2 < 16) bq[(f + 2) % 3] = bbuf[cur][((f + 2) % 4) * 4 + (f + 2) / 4][lane];                      \
            _Pragma("unroll") for (int r = 0; r < RB; ++r)                                                           \
                acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ACUR[r][kb], bq[f % 3], acc[r][c], 0, 0, 0);     \
            if (c == 3) {                                                                                            \
                __builtin_amdgcn_sched_barrier(0);                                                                   \
                _Pragma("unroll") for (int r = 0; r < RB; ++r) ACUR[r][kb] = a_ptr[r][(sa * 4 + kb) * 64];           \
                __builtin_amdgcn_sched_barrier(0);                                                                   \
            }                                                                                                        \
        }                                                                                                            \
        _Pragma("unroll") for (int i = 0; i < RPW; ++i) bbuf[cur ^ 1][b_rec[i]][lane] = b_ring[(SLOT + 1) % 3][i];   \
        __syncthreads();                                                                                             \
        ++s;                                                                                                         \
    }
    // the number of stages is a multiple of six (the slot count is padded for it): six stages of straight-line code
    for (int s = 0; s < stages;) {
        RDK_STAGE(0, a_even)
        RDK_STAGE(1, a_odd)
        RDK_STAGE(2, a_even)
        RDK_STAGE(0, a_odd)
        RDK_STAGE(1, a_even)
        RDK_STAGE(2, a_odd)
    }
#undef RDK_STAGE
    // D layout of the 32x32 tile: lane l holds column l % 32 and rows 8 * (v / 4) + 4 * (l / 32) + v % 4, v = 0..15
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int c = 0; c < kColBlocksPerWg; ++c) {
            const int j = (jb0 + c) * kColBlock + (lane % 32);
            if (jb0 + c >= n_jb || j >= N) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int b = (rb0 + r) * 32 + 8 * (v / 4) + 4 * (lane / 32) + (v % 4);
                if (b < B) out[(int64_t)b * ldo + j] = acc[r][c][v] * out_scale[b];
            }
        }
}

// wavefronts per workgroup and row blocks per wavefront for a batch of B positions
inline void bf16_shape(int B, int &W, int &RB)
{
    if (B <= 128) { W = 4; RB = 1; }
    else if (B <= 256) { W = 8; RB = 1; }
    else { W = 4; RB = 4; }   // one wavefront per SIMD with all 512 registers: half the LDS reads per MFMA
}

struct ExactWs {
    SoftStat *qstat;   // [B]
    float *part;       // fp32 path: [splits, B, N_ld]
    uint16_t *A;       // bf16 path: [B_pad, n_pad]
    float *out_scale;  // bf16 path: [B]
};

int f32_splits(const KernelHandle &h, int B)
{
    const int tiles = ((h.N + kColsF - 1) / kColsF) * ((B + kRowsF - 1) / kRowsF);
    int want = (1024 + tiles - 1) / tiles;
    const int maxs = (h.n + 8 * kDepthF - 1) / (8 * kDepthF);    // at least 256 slots per split
    if (want > maxs) want = maxs;
    if (want > 32) want = 32;
    return want < 1 ? 1 : want;
}

template <int QK>
rdk_status_t run_exact(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws, hipStream_t st)
{
    char *p = (char *)ws;
    ExactWs w;
    w.qstat = (SoftStat *)p; p += align_up((size_t)B * sizeof(SoftStat), 256);
    rdk_status_t rc = launch_row_stats<QK>(q, h.n, B, 1, w.qstat, st);
    if (rc != RDK_OK) return rc;
    if (h.format == RDK_DENSE_F32) {
        w.part = (float *)p;
        const int splits = f32_splits(h, B);
        const int per = (((h.n + splits - 1) / splits) + kDepthF - 1) / kDepthF * kDepthF;
        const int64_t ldd = (h.N + 3) / 4 * 4;
        dim3 grid((h.N + kColsF - 1) / kColsF, (B + kRowsF - 1) / kRowsF, splits);
        if (splits == 1) {
            {
                RDK_TIMED_LAUNCH("exact_f32_kernel", (exact_f32_kernel<QK>), grid, dim3(256), 0, st, q.ptr, q.ld, w.qstat, h.dense, h.ldm, h.n, h.N,
                                   B, per, out, ldo, (int64_t)0, true);
            }
            RDK_LAUNCH_CHECK("exact_f32_kernel");
        } else {
            {
                RDK_TIMED_LAUNCH("exact_f32_kernel", (exact_f32_kernel<QK>), grid, dim3(256), 0, st, q.ptr, q.ld, w.qstat, h.dense, h.ldm, h.n, h.N,
                                   B, per, w.part, ldd, (int64_t)B * ldd, false);
            }
            RDK_LAUNCH_CHECK("exact_f32_kernel");
            {
                RDK_TIMED_LAUNCH("exact_reduce_kernel", exact_reduce_kernel, dim3((h.N + 1023) / 1024, B), dim3(256), 0, st, w.part, ldd,
                                   (int64_t)B * ldd, splits, w.qstat, h.N, out, ldo);
            }
            RDK_LAUNCH_CHECK("exact_reduce_kernel");
        }
        return RDK_OK;
    }
    // bf16
    int W, RB;
    bf16_shape(B, W, RB);
    const int rows_per_wg = W * RB * 32;
    const int B_pad = (B + rows_per_wg - 1) / rows_per_wg * rows_per_wg;
    const int KB = h.n_pad / kKStep;
    w.A = (uint16_t *)p; p += align_up((size_t)B_pad * h.n_pad * 2, 256);
    w.out_scale = (float *)p;
    {
        RDK_TIMED_LAUNCH("prep_a_bf16_kernel", (prep_a_bf16_kernel<QK>), dim3(B_pad), dim3(256), 0, st, q.ptr, q.ld, w.qstat, h.row_sum, h.n, KB, B,
                           w.A, w.out_scale);
    }
    RDK_LAUNCH_CHECK("prep_a_bf16_kernel");
    const int n_jb = (h.N + kColBlock - 1) / kColBlock;
    dim3 grid((n_jb + kColBlocksPerWg - 1) / kColBlocksPerWg, B_pad / rows_per_wg);
    {
        if (W == 4 && RB == 1)
            RDK_TIMED_LAUNCH("exact_bf16_kernel", (exact_bf16_kernel<4, 1>), grid, dim3(256), 0, st, w.A, h.packed, KB, h.N, B, w.out_scale, out, ldo);
        else if (W == 8)
            RDK_TIMED_LAUNCH("exact_bf16_kernel", (exact_bf16_kernel<8, 1>), grid, dim3(512), 0, st, w.A, h.packed, KB, h.N, B, w.out_scale, out, ldo);
        else
            RDK_TIMED_LAUNCH("exact_bf16_kernel", (exact_bf16_kernel<4, 4>), grid, dim3(256), 0, st, w.A, h.packed, KB, h.N, B, w.out_scale, out, ldo);
    }
    RDK_LAUNCH_CHECK("exact_bf16_kernel");
    return RDK_OK;
}

}  // namespace

size_t packed_bf16_bytes(int32_t n, int32_t N, int32_t *n_pad, int32_t *N_pad)
{
    const int32_t np = (n + 24 * kKStep - 1) / (24 * kKStep) * (24 * kKStep);   // six whole stages of four MFMA steps
    const int32_t Np = (N + kColBlock - 1) / kColBlock * kColBlock;
    if (n_pad) *n_pad = np;
    if (N_pad) *N_pad = Np;
    return (size_t)np * Np * 2;
}

size_t exact_workspace_bytes(const KernelHandle &h, int32_t B)
{
    size_t bytes = align_up((size_t)B * sizeof(SoftStat), 256);
    if (h.format == RDK_DENSE_F32) {
        const int splits = f32_splits(h, B);
        if (splits > 1) bytes += align_up((size_t)splits * B * ((h.N + 3) / 4 * 4) * sizeof(float), 256);
    } else if (h.format == RDK_DENSE_BF16) {
        int W, RB;
        bf16_shape(B, W, RB);
        const int rows_per_wg = W * RB * 32;
        const size_t B_pad = (size_t)(B + rows_per_wg - 1) / rows_per_wg * rows_per_wg;
        bytes += align_up(B_pad * h.n_pad * 2, 256) + align_up((size_t)B * sizeof(float), 256);
    }
    return bytes;
}

rdk_status_t launch_pack_bf16(const float *M, int64_t ldm, int32_t n, int32_t N, uint16_t *packed, float *row_sum,
                              hipStream_t st)
{
    int32_t n_pad, N_pad;
    packed_bf16_bytes(n, N, &n_pad, &N_pad);
    const int KB = n_pad / kKStep;
    hipLaunchKernelGGL(pack_bf16_kernel, dim3(N_pad / kColBlock, KB < 64 ? KB : 64), dim3(64), 0, st, M, ldm, n, N, KB, packed);
    RDK_LAUNCH_CHECK("pack_bf16_kernel");
    hipLaunchKernelGGL(rounded_row_sum_kernel, dim3(n), dim3(256), 0, st, M, ldm, N, row_sum);
    RDK_LAUNCH_CHECK("rounded_row_sum_kernel");
    return RDK_OK;
}

rdk_status_t launch_unpack_bf16(const KernelHandle &h, float *M, int64_t ldm, hipStream_t st)
{
    const int KB = h.n_pad / kKStep;
    hipLaunchKernelGGL(unpack_bf16_kernel, dim3(h.N_pad / kColBlock, KB < 64 ? KB : 64), dim3(64), 0, st, h.packed, h.n, h.N,
                       KB, M, ldm);
    RDK_LAUNCH_CHECK("unpack_bf16_kernel");
    return RDK_OK;
}

rdk_status_t launch_exact(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws, hipStream_t st)
{
    switch (q.kind) {
        case RDK_PROB_F32: return run_exact<RDK_PROB_F32>(h, q, B, out, ldo, ws, st);
        case RDK_LOGIT_F32: return run_exact<RDK_LOGIT_F32>(h, q, B, out, ldo, ws, st);
        case RDK_LOGIT_BF16: return run_exact<RDK_LOGIT_BF16>(h, q, B, out, ldo, ws, st);
    }
    return RDK_ERR_DTYPE;
}

}  // namespace rdk
