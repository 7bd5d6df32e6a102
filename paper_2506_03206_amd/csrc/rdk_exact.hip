// Exact redistribution (Alg. 1, step 2):  P'[b, j] = sum_s Q'[b, s] M[s, j]  with a dense kernel M.
//   fp32 kernel:  both operands split into three bf16 parts each, six part products per term on the bf16 matrix
//                 cores (v_mfma_f32_32x32x16_bf16) with fp32 accumulation; M read straight from its row-major
//                 rows, split over the kept slots, fixed-order reduction.
//   bf16 kernel:  M rounded to bf16, the drafter rows to eleven significant bits; both held as scaled fp16 numbers,
//                 fp32 accumulation on the matrix cores (v_mfma_f32_32x32x16_f16), rows rescaled so that they sum to one.
// Step 1 (Eq. 1) is folded in: rows of Q' are the drafter rows divided by their sums.
#include "rdk_rowstats.hpp"

namespace rdk {

namespace {

// ------------------------------------------------------------------------------------------------ fp32
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kRowGroup = 64;    // positions per wavefront tile: two 32-row MFMA blocks
constexpr int kColSet = 128;     // target ids per wavefront tile

// At 64 positions the product needs 2 n N flop against 4 n N bytes of M: 32 flop per byte, more than the fp32 matrix
// unit delivers per HBM byte (157 TFLOP/s : 8 TB/s = 20).  The bf16 matrix instruction is sixteen times as fast, and
// an fp32 number is the exact sum of three bf16 numbers (its leading, middle and trailing eight significant bits), so
// the product of two fp32 numbers is taken from the six largest products of their parts, all accumulated in fp32 by
// the MFMA:
//   x y = xh yh + (xh ym + xm yh) + (xh yl + xl yh + xm ym) + terms below 2^-24 |x y|.
// Every part product is exact in fp32, so the result carries the rounding of an fp32 dot product.  With six bf16
// MFMAs in place of sixteen fp32 ones per sixteen slots the path is bound by reading M, not by the matrix rate.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSplitStep = 16;   // kept slots per bf16 MFMA
constexpr int kSplitRing = 3;     // slot blocks in the load ring (all but one ahead of the MFMAs; deeper rings gain nothing)

// Upper halves of h, m, l hold the three bf16 parts of x (x = h + m + l exactly, for normal numbers).
__device__ __forceinline__ void split3(float x, uint32_t &h, uint32_t &m, uint32_t &l)
{
    h = __float_as_uint(x) & 0xFFFF0000u;
    const float r = x - __uint_as_float(h);      // exact: at most sixteen significant bits are left
    m = __float_as_uint(r) & 0xFFFF0000u;
    l = __float_as_uint(r - __uint_as_float(m)); // exact, at most eight significant bits: already a bf16 number
}

// two bf16 numbers given in the upper halves of a and b, packed as (a, b) = (low half, high half)
__device__ __forceinline__ uint32_t pack_upper(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xFFFF0000u); }

// A records of this form: for row block rb (32 positions) and slot block kb (16 slots) three consecutive 1 KB
// records, part p = 0 (leading), 1, 2; lane l = 32 g + r holds part p of the unnormalised drafter weights of
// position 32 rb + r at slots 16 kb + 8 g + e, e = 0..7 -- the A operand of one 32x32x16 MFMA.  Zero beyond B and n.
template <int QK>
__global__ void prep_a_split_kernel(const void *q, int64_t ldq, const SoftStat *qstat, int n, int B, int KB, int64_t records,
                                    uint16_t *Ap)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= records * kWave) return;
    const int l = (int)(idx % kWave);
    const int64_t rec = idx / kWave;
    const int kb = (int)(rec % KB);
    const int b = (int)(rec / KB) * 32 + l % 32, g = l / 32;
    uint32_t h[8], m[8], lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = m[e] = lo[e] = 0u;
    if (b < B) {
        const void *qr = row_ptr<QK>(q, ldq, b);
        const float qm = QK == RDK_PROB_F32 ? 0.f : qstat[b].m;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int s = kb * kSplitStep + g * 8 + e;
            if (s < n) split3(to_weight<QK>(load1<QK>(qr, s), qm, 1.f), h[e], m[e], lo[e]);
        }
    }
    uint4 *dst = (uint4 *)(Ap + ((rec * 3) * kWave + l) * 8);
    dst[0] = make_uint4(pack_upper(h[0], h[1]), pack_upper(h[2], h[3]), pack_upper(h[4], h[5]), pack_upper(h[6], h[7]));
    dst[kWave] = make_uint4(pack_upper(m[0], m[1]), pack_upper(m[2], m[3]), pack_upper(m[4], m[5]), pack_upper(m[6], m[7]));
    dst[2 * kWave] = make_uint4(pack_upper(lo[0], lo[1]), pack_upper(lo[2], lo[3]), pack_upper(lo[4], lo[5]), pack_upper(lo[6], lo[7]));
}

// One wavefront per (128 target ids, 64 positions, one split of the slot blocks), one wavefront per SIMD.  The B
// operand of the 32x32x16 MFMA wants from lane l = 32 g + c the eight slots 8 g .. 8 g + 7 of column c.  Column c of
// MFMA e (e = 0..3) is given the target id j0 + 4 c + e, so the lane reads M[s][j0 + 4c .. + 3] for its eight slots
// s = 16 kb + 8 g + i with eight 16-byte loads of the row-major M -- no packing of M, no LDS -- splits the 32 values
// in registers and feeds four MFMA columns; the four results of a lane are again four consecutive ids.  Loads run
// two slot blocks ahead through a ring of three register sets; the split length is a multiple of three blocks (A is
// zero beyond n, rows of M are clamped to the last one).  Tiles of 64 ids at two wavefronts per SIMD were slower
// (0.26 ms against 0.22 ms): every wavefront reads all drafter records of its split.
constexpr int kSplitWaves = 4;   // wavefronts per workgroup: neighbouring id tiles, walked in step

__global__ __launch_bounds__(kSplitWaves * kWave) __attribute__((amdgpu_waves_per_eu(1, 1))) void exact_f32_split_kernel(
    const uint16_t *Ap, const float *M, int64_t ldm, int n, int N, int B, int KB, int blocks_per_split, const SoftStat *qstat,
    float *dst, int64_t ldd, int64_t split_stride, bool scale_here, bool vec_d)
{
    const int lane = lane_id(), c = lane % 32, g = lane / 32;
    const int tile = blockIdx.x * kSplitWaves + threadIdx.x / kWave;
    if (tile * kColSet >= N) return;   // a whole wavefront; the kernel has no barrier
    const int j0 = tile * kColSet, col = j0 + 4 * c;
    const int rg = blockIdx.y;
    const int kb0 = blockIdx.z * blocks_per_split, kb_last = kb0 + blocks_per_split - 1;
    const bool full = col + 3 < N;
    const int lcol = col < N ? col : 0;   // lanes beyond N read column 0 (never stored): no branch around the loads
    f32x16 acc[2][4];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rb][e][v] = 0.f;
    const bf16x8 *a_rec[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) a_rec[rb] = (const bf16x8 *)Ap + ((int64_t)(rg * 2 + rb) * KB) * 3 * kWave + lane;

    bf16x8 a_ring[kSplitRing][2][3];
    float4 b_ring[kSplitRing][8];
#define RDK_LOAD_BLOCK(SLOT, KBI)                                                                                    \
    {                                                                                                                \
        const int kb_ = min((KBI), kb_last);                                                                         \
        _Pragma("unroll") for (int rb = 0; rb < 2; ++rb)                                                             \
            _Pragma("unroll") for (int pt = 0; pt < 3; ++pt)                                                         \
                a_ring[SLOT][rb][pt] = a_rec[rb][((int64_t)kb_ * 3 + pt) * kWave];                                   \
        _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                              \
            const int s_ = min(kb_ * kSplitStep + 8 * g + i, n - 1);                                                 \
            b_ring[SLOT][i] = *(const float4 *)(M + (int64_t)s_ * ldm + lcol);                                       \
        }                                                                                                            \
        __builtin_amdgcn_sched_barrier(0);                                                                           \
    }
    // the four MFMA columns of a block, two at a time: split the eight values of each, then the six part products
    // smallest first, alternating between the four accumulators involved
#define RDK_MFMA_BLOCK(SLOT)                                                                                         \
    {                                                                                                                \
        _Pragma("unroll") for (int ep = 0; ep < 4; ep += 2) {                                                        \
            bf16x8 bh_[2], bm_[2], bl_[2];                                                                           \
            _Pragma("unroll") for (int ee = 0; ee < 2; ++ee) {                                                       \
                uint32_t h_[8], m_[8], l_[8];                                                                        \
                _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                      \
                    const float4 bv_ = b_ring[SLOT][i];                                                              \
                    const float x_ = (ep + ee) == 0 ? bv_.x : (ep + ee) == 1 ? bv_.y : (ep + ee) == 2 ? bv_.z : bv_.w; \
                    split3(x_, h_[i], m_[i], l_[i]);                                                                 \
                }                                                                                                    \
                const u32x4 hv_ = {pack_upper(h_[0], h_[1]), pack_upper(h_[2], h_[3]), pack_upper(h_[4], h_[5]), pack_upper(h_[6], h_[7])}; \
                const u32x4 mv_ = {pack_upper(m_[0], m_[1]), pack_upper(m_[2], m_[3]), pack_upper(m_[4], m_[5]), pack_upper(m_[6], m_[7])}; \
                const u32x4 lv_ = {pack_upper(l_[0], l_[1]), pack_upper(l_[2], l_[3]), pack_upper(l_[4], l_[5]), pack_upper(l_[6], l_[7])}; \
                bh_[ee] = __builtin_bit_cast(bf16x8, hv_);                                                           \
                bm_[ee] = __builtin_bit_cast(bf16x8, mv_);                                                           \
                bl_[ee] = __builtin_bit_cast(bf16x8, lv_);                                                           \
            }                                                                                                        \
            RDK_PART_PRODUCT(SLOT, ep, 1, bm_)                                                                       \
            RDK_PART_PRODUCT(SLOT, ep, 2, bh_)                                                                       \
            RDK_PART_PRODUCT(SLOT, ep, 0, bl_)                                                                       \
            RDK_PART_PRODUCT(SLOT, ep, 1, bh_)                                                                       \
            RDK_PART_PRODUCT(SLOT, ep, 0, bm_)                                                                       \
            RDK_PART_PRODUCT(SLOT, ep, 0, bh_)                                                                       \
        }                                                                                                            \
    }
#define RDK_PART_PRODUCT(SLOT, EP, APART, BPART)                                                                     \
    _Pragma("unroll") for (int ee = 0; ee < 2; ++ee)                                                                 \
        _Pragma("unroll") for (int rb = 0; rb < 2; ++rb)                                                             \
            acc[rb][(EP) + ee] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_ring[SLOT][rb][APART], BPART[ee],         \
                                                                         acc[rb][(EP) + ee], 0, 0, 0);
#pragma unroll
    for (int t = 0; t < kSplitRing - 1; ++t) RDK_LOAD_BLOCK(t, kb0 + t)
    for (int kb = kb0; kb <= kb_last; kb += kSplitRing) {
#pragma unroll
        for (int t = 0; t < kSplitRing; ++t) {   // ring entries are compile-time constants after unrolling
            RDK_LOAD_BLOCK((t + kSplitRing - 1) % kSplitRing, kb + t + kSplitRing - 1)
            RDK_MFMA_BLOCK(t)
        }
    }
#undef RDK_LOAD_BLOCK
#undef RDK_MFMA_BLOCK
#undef RDK_PART_PRODUCT
    // D layout of a 32x32 tile: lane l holds column l % 32 and rows 8 * (v / 4) + 4 * (l / 32) + v % 4, v = 0..15
    float *base = dst + (int64_t)blockIdx.z * split_stride;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int b = rg * kRowGroup + rb * 32 + 8 * (v / 4) + 4 * g + (v % 4);
            if (b >= B) continue;
            const float sc = scale_here ? inv_mass(qstat[b].s) : 1.f;
            const float o[4] = {acc[rb][0][v] * sc, acc[rb][1][v] * sc, acc[rb][2][v] * sc, acc[rb][3][v] * sc};
            float *drow = base + (int64_t)b * ldd + col;
            if (full && vec_d) {
                *(float4 *)drow = make_float4(o[0], o[1], o[2], o[3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < N) drow[e] = o[e];
            }
        }
}

// Sum of the split partials in split order, divided by the drafter row sum (Eq. 1).
__global__ void exact_reduce_kernel(const float *part, int64_t ldd, int64_t split_stride, int splits, const SoftStat *qstat,
                                    int N, int B, float *out, int64_t ldo)
{
    for (int b = blockIdx.y; b < B; b += gridDim.y) {   // positions beyond the grid's second dimension are looped over
        const float sc = inv_mass(qstat[b].s);
        for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < N; j += (int64_t)gridDim.x * blockDim.x) {
            float s = 0.f;
            for (int z = 0; z < splits; ++z) s += part[(int64_t)z * split_stride + (int64_t)b * ldd + j];
            out[(int64_t)b * ldo + j] = s * sc;
        }
    }
}

// ------------------------------------------------------------------------------------------------ bf16

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

// The 16-bit operands of the dense product.  A bf16 number keeps eight significant bits: rounding a peaked drafter row
// to it moves single outputs by up to 2^-8, twice the tolerance this path states (2e-3).  The matrix cores run fp16
// at the same rate, and fp16 keeps eleven bits, so both operands are held as fp16 numbers scaled by 2^15:
//   * an entry of M is first rounded to bf16 (the format the kernel is specified in) and that value, times 2^15, is
//     an fp16 number exactly as long as it is at least 2^-29;
//   * an entry of a normalised drafter row is rounded to eleven significant bits (relative error at most 2^-12).
// Values whose scaled magnitude is below the smallest normal fp16 number (2^-14, i.e. below 2^-29 = 1.9e-9 unscaled)
// are stored as zero, whatever the denormal mode of the hardware; the products carry the factor 2^30, taken out
// again by the row scale.
constexpr float kOperandScale = 32768.0f;                 // 2^15
constexpr float kOperandUnscale = 1.0f / 32768.0f;
constexpr float kHalfMinNormal = 6.103515625e-05f;        // 2^-14

__device__ __forceinline__ uint16_t f32_to_operand(float x)   // x >= 0, at most 1
{
    const float y = x * kOperandScale;
    if (!(y >= kHalfMinNormal)) return 0;
    return __builtin_bit_cast(uint16_t, (_Float16)y);   // round to nearest even
}

__device__ __forceinline__ float operand_to_f32(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h) * kOperandUnscale; }

// an entry of M as stored: rounded to bf16, then held as a scaled fp16 number
__device__ __forceinline__ uint16_t kernel_entry(float m) { return f32_to_operand(bf16_to_f32(f32_to_bf16_rne(m))); }

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
            w[e / 2] = (uint32_t)kernel_entry(v0) | ((uint32_t)kernel_entry(v1) << 16);
        }
        *(uint4 *)(packed + (((int64_t)jb * KB + kb) * 64 + lane) * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// fp32 sums of the rows of M as stored (needed to rescale output rows to unit mass).
__global__ void rounded_row_sum_kernel(const float *M, int64_t ldm, int N, float *row_sum)
{
    const int s = blockIdx.x;
    double sum = 0.0;
    for (int j = threadIdx.x; j < N; j += blockDim.x)
        sum += (double)operand_to_f32(kernel_entry(M[(int64_t)s * ldm + j]));
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
            if (s < n) M[(int64_t)s * ldm + j] = operand_to_f32(rec[e]);
        }
    }
}

// A operand: TLI-normalised drafter rows as 16-bit operands (see f32_to_operand), packed like M: for row block rb (32 positions) and
// slot block kb (16 slots) one 1 KB record holding, for lane l = 32 * g + r, the eight values
// q'[rb*32 + r, kb*16 + g*8 + e], e = 0..7 -- the A operand of one 32x32x16 MFMA.  Also per row the factor
// 2^-30 / sum_s rounded(q'_s) * row_sum[s]: it takes the operand scales out and makes the output row sum to one.
// One workgroup per position.
template <int QK>
__global__ __launch_bounds__(256) void prep_a_bf16_kernel(const void *q, int64_t ldq, const SoftStat *qstat, const float *row_sum,
                                                          int n, int KB, int B, uint16_t *Ap, float *out_scale)
{
    const int b = blockIdx.x;
    const int rb = b / 32, r = b % 32;
    double mass = 0.0;
    const void *qr = b < B ? row_ptr<QK>(q, ldq, b) : nullptr;
    const float qm = b < B ? qstat[b].m : 0.f, inv = b < B ? inv_mass(qstat[b].s) : 0.f;
    for (int c = threadIdx.x; c < KB * 2; c += blockDim.x) {   // chunk of 8 consecutive slots
        const int kb = c / 2, g = c % 2;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (qr) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int s = c * 8 + e;
                uint16_t h = 0;
                if (s < n) {
                    h = f32_to_operand(to_weight<QK>(load1<QK>(qr, s), qm, 1.f) * inv);
                    mass += (double)operand_to_f32(h) * (double)row_sum[s];
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
    if (threadIdx.x == 0 && b < B) {
        const double total = (sh[0] + sh[1]) + (sh[2] + sh[3]);
        out_scale[b] = total > 0.0 ? (float)((double)kOperandUnscale * (double)kOperandUnscale / total) : 0.f;
    }
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
// A record of M: read exactly once per launch, so it is loaded non-temporally and leaves the L2 to the A records,
// which every workgroup of an XCD reads again.
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ f16x8 load_once(const f16x8 *p)
{
    return __builtin_bit_cast(f16x8, __builtin_nontemporal_load((const u32x4_t *)p));
}

template <int W, int RB>
__global__ __launch_bounds__(W * 64) void exact_bf16_kernel(const uint16_t *Ap, const uint16_t *Mp, int KB, int N, int B,
                                                            const float *out_scale, float *out, int64_t ldo)
{
    constexpr int RPW = 16 / W;   // B records a wavefront fetches per stage
    __shared__ f16x8 bbuf[2][16][64];
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

    const f16x8 *a_ptr[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) a_ptr[r] = (const f16x8 *)Ap + ((int64_t)(rb0 + r) * KB) * 64 + lane;
    const f16x8 *b_src[RPW];
    int b_rec[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        b_rec[i] = wid * RPW + i;                               // record = jb * 4 + kb within the stage
        const int jb = min(jb0 + b_rec[i] / 4, n_jb - 1);       // surplus column blocks recompute the last one
        b_src[i] = (const f16x8 *)Mp + ((int64_t)jb * KB + b_rec[i] % 4) * 64 + lane;
    }
    // Loads return to a wavefront in issue order, so every load inherits the latency of the slowest one before
    // it.  The B records come from HBM: they are requested three stages ahead and kept in a ring of registers.
    // The A records (L2) are requested two stages ahead, block by block as their registers fall free; the only
    // B request older than an A record at the time it is needed is then two whole stages old.
    // The first requests are issued in the order the stages keep afterwards (A by slot block, at least as many
    // requests behind every record as in the steady state): the wait counts the compiler derives for the first stages
    // of the loop are the minimum over both ways into them, and a different order here would tighten them for good.
    f16x8 a_even[RB][4], a_odd[RB][4], b_ring[3][RPW];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < RB; ++r) a_even[r][kb] = a_ptr[r][kb * 64];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
        for (int i = 0; i < RPW; ++i) b_ring[t][i] = load_once(b_src[i] + (int64_t)min(t, stages - 1) * 4 * 64);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < RB; ++r) a_odd[r][kb] = a_ptr[r][((int64_t)min(1, stages - 1) * 4 + kb) * 64];
    __builtin_amdgcn_sched_barrier(0);
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
        _Pragma("unroll") for (int i = 0; i < RPW; ++i) b_ring[SLOT][i] = load_once(b_src[i] + sb * 4 * 64);         \
        __builtin_amdgcn_sched_barrier(0);                                                                           \
        f16x8 bq[3];                        /* B fragments are read from LDS two MFMA groups ahead */               \
        bq[0] = bbuf[cur][0][lane];                                                                                  \
        bq[1] = bbuf[cur][4][lane];                                                                                  \
        _Pragma("unroll") for (int f = 0; f < 16; ++f) {     /* f = kb * 4 + c */                                    \
            const int kb = f / 4, c = f % 4;                                                                         \
            if (f + 2 < 16) bq[(f + 2) % 3] = bbuf[cur][((f + 2) % 4) * 4 + (f + 2) / 4][lane];                      \
            _Pragma("unroll") for (int r = 0; r < RB; ++r)                                                           \
                acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ACUR[r][kb], bq[f % 3], acc[r][c], 0, 0, 0);     \
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
    float *part;       // fp32 path: [splits, B, N_ld]  (after the A records of that path)
    uint16_t *A;       // bf16 path: [B_pad, n_pad]
    float *out_scale;  // bf16 path: [B]
};

// Split of the slot blocks of the fp32 path: as many wavefronts as the chip holds at one per SIMD (1024) but no more,
// so that they all run side by side (a few left over for a second round would double the time); splits of a whole
// number of ring turns.  blocks = slot blocks per split.
int split_splits(const KernelHandle &h, int B, int *blocks)
{
    const int tiles = ((h.N + kColSet - 1) / kColSet) * ((B + kRowGroup - 1) / kRowGroup);
    const int kb_total = (h.n + kSplitStep - 1) / kSplitStep;
    int want = 1024 / tiles;
    const int maxs = (kb_total + 2 * kSplitRing - 1) / (2 * kSplitRing);    // at least 96 slots per split
    if (want > maxs) want = maxs;
    if (want > 64) want = 64;
    if (want < 1) want = 1;
    const int per = ((kb_total + want - 1) / want + kSplitRing - 1) / kSplitRing * kSplitRing;
    const int splits = (kb_total + per - 1) / per;
    if (blocks) *blocks = per;
    return splits;
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
        int blocks;
        const int splits = split_splits(h, B, &blocks);
        const int KB = splits * blocks;
        const int row_groups = (B + kRowGroup - 1) / kRowGroup;
        const int64_t records = (int64_t)row_groups * 2 * KB;   // of three parts each
        uint16_t *Ap = (uint16_t *)p; p += align_up((size_t)records * 3 * kWave * 8 * sizeof(uint16_t), 256);
        w.part = (float *)p;
        const int64_t ldd = (h.N + 3) / 4 * 4;
        {
            RDK_TIMED_LAUNCH("prep_a_split_kernel", (prep_a_split_kernel<QK>), dim3((unsigned)((records * kWave + 255) / 256)),
                             dim3(256), 0, st, q.ptr, q.ld, w.qstat, h.n, B, KB, records, Ap);
        }
        RDK_LAUNCH_CHECK("prep_a_split_kernel");
        const int tiles = (h.N + kColSet - 1) / kColSet;
        dim3 grid((tiles + kSplitWaves - 1) / kSplitWaves, row_groups, splits);
        if (splits == 1) {
            const bool vec_d = rows_vectorisable(out, ldo, RDK_PROB_F32);
            RDK_TIMED_LAUNCH("exact_f32_split_kernel", exact_f32_split_kernel, grid, dim3(kSplitWaves * kWave), 0, st, Ap, h.dense,
                             h.ldm, h.n, h.N, B, KB, blocks, w.qstat, out, ldo, (int64_t)0, true, vec_d);
            RDK_LAUNCH_CHECK("exact_f32_split_kernel");
        } else {
            RDK_TIMED_LAUNCH("exact_f32_split_kernel", exact_f32_split_kernel, grid, dim3(kSplitWaves * kWave), 0, st, Ap, h.dense,
                             h.ldm, h.n, h.N, B, KB, blocks, w.qstat, w.part, ldd, (int64_t)B * ldd, false, true);
            RDK_LAUNCH_CHECK("exact_f32_split_kernel");
            RDK_TIMED_LAUNCH("exact_reduce_kernel", exact_reduce_kernel, dim3((h.N + 1023) / 1024, B < 32768 ? B : 32768), dim3(256), 0,
                             st, w.part, ldd, (int64_t)B * ldd, splits, w.qstat, h.N, B, out, ldo);
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
        RDK_TIMED_LAUNCH("prep_a_bf16_kernel", (prep_a_bf16_kernel<QK>), dim3(B_pad), dim3(256), 0, st, q.ptr, q.ld, w.qstat,
                         h.row_sum, h.n, KB, B, w.A, w.out_scale);
    }
    RDK_LAUNCH_CHECK("prep_a_bf16_kernel");
    const int n_jb = (h.N + kColBlock - 1) / kColBlock;
    dim3 grid((n_jb + kColBlocksPerWg - 1) / kColBlocksPerWg, B_pad / rows_per_wg);
    {
        if (W == 4 && RB == 1)
            RDK_TIMED_LAUNCH("exact_bf16_kernel", (exact_bf16_kernel<4, 1>), grid, dim3(256), 0, st, w.A, h.packed, KB, h.N, B,
                             w.out_scale, out, ldo);
        else if (W == 8)
            RDK_TIMED_LAUNCH("exact_bf16_kernel", (exact_bf16_kernel<8, 1>), grid, dim3(512), 0, st, w.A, h.packed, KB, h.N, B,
                             w.out_scale, out, ldo);
        else
            RDK_TIMED_LAUNCH("exact_bf16_kernel", (exact_bf16_kernel<4, 4>), grid, dim3(256), 0, st, w.A, h.packed, KB, h.N, B,
                             w.out_scale, out, ldo);
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
        int blocks;
        const int splits = split_splits(h, B, &blocks);
        const size_t records = (size_t)((B + kRowGroup - 1) / kRowGroup) * 2 * splits * blocks;
        bytes += align_up(records * 3 * kWave * 8 * sizeof(uint16_t), 256);
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
