// Device-side helpers: wavefront reductions and scans, typed row loads, Philox4x32-10.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rdk_common.hpp"

namespace rdk {

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// ---- 64-wide reductions and scans on the data-parallel-primitive (DPP) modifiers of the vector ALU: a lane
// reads another lane of its row of 16 at register speed, where a shuffle goes through the LDS crossbar (an
// order of magnitude more latency, which a lone wavefront cannot hide).  Controls: 0xB1 / 0x4E = quad
// permutations [1,0,3,2] / [2,3,0,1], 0x141 / 0x140 = mirror within 8 / 16 lanes, 0x110 + n = shift right by n
// within the row, 0x142 / 0x143 = lane 15 of each row to the next row / lane 31 to rows 2 and 3.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ float dpp_move(float v)   // lanes without a source (or outside ROW_MASK) get 0
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false));
}

template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ double dpp_move(double v)
{
    const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)b, CTRL, ROW_MASK, 0xf, false);
    const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(b >> 32), CTRL, ROW_MASK, 0xf, false);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

// value of lane `src` (the same for all lanes) in every lane
__device__ __forceinline__ int lane_value(int v, int src)
{
    return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(src));
}
__device__ __forceinline__ float lane_value(float v, int src)
{
    return __builtin_bit_cast(float, lane_value(__builtin_bit_cast(int, v), src));
}
__device__ __forceinline__ double lane_value(double v, int src)
{
    const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)lane_value((int)(unsigned)b, src), hi = (unsigned)lane_value((int)(unsigned)(b >> 32), src);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

// sum over each row of 16 lanes, the same bits in all 16
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    return v;
}

// sum over the 64 lanes, the same bits in every lane
template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);   // every lane holds the sum of its row of 16
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_move<0xB1>(v));
    v = fmaxf(v, dpp_move<0x4E>(v));
    v = fmaxf(v, dpp_move<0x141>(v));
    v = fmaxf(v, dpp_move<0x140>(v));
    return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}

// Inclusive prefix sum over the 64 lanes: Hillis-Steele inside each row, then the row totals are handed on.
__device__ __forceinline__ double wave_inclusive_scan(double v)
{
    v += dpp_move<0x111>(v);
    v += dpp_move<0x112>(v);
    v += dpp_move<0x114>(v);
    v += dpp_move<0x118>(v);
    v += dpp_move<0x142, 0xa>(v);   // rows 1 and 3 take the total of the row before
    v += dpp_move<0x143, 0xc>(v);   // rows 2 and 3 take the total of rows 0 and 1
    return v;
}

// exp(x) for x <= 0 (softmax terms) through the hardware base-2 exponential: one multiply and one v_exp_f32
// instead of the dozen instructions of the library routine, which made the logit paths ALU-bound.  The product
// x * log2(e) is rounded once: relative error of the result about |x| * 6e-8, i.e. below 1e-6 for every term
// larger than e^-15 of the row maximum; exp(-inf) = 0.  Every kernel uses this one function, so normalisers
// and terms carry the same rounding.
__device__ __forceinline__ float soft_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }

// The same with the rounding of the product x * log2(e) carried along (its exact residual and the part of log2(e) that
// a float drops): about one ulp for any x <= 0.  Three more instructions: for factors that a whole chunk of ids shares.
__device__ __forceinline__ float soft_exp_fine(float x)
{
    const float hi = x * 1.44269504088896341f;
    const float lo = fmaf(x, 1.44269504088896341f, -hi) + x * 1.92596299e-8f;
    return __builtin_amdgcn_exp2f(hi) * fmaf(0.693147180559945309f, lo, 1.0f);
}

// 1 / (mass of a drafter row), and 0 for a row without mass: Eq. 1 is undefined there, and every redistribution
// then returns the zero row (no token can be drafted from it; verification falls back on the target row alone).
__device__ __forceinline__ float inv_mass(float z) { return z > 0.f ? 1.0f / z : 0.f; }

// ---- softmax statistics (running maximum m and sum of exp(z - m)), merged pairwise
struct SoftStat {
    float m, s;
};

__device__ __forceinline__ SoftStat soft_merge(SoftStat a, SoftStat b)
{
    float m = fmaxf(a.m, b.m);
    SoftStat r;
    r.m = m;
    r.s = (a.s == 0.f ? 0.f : a.s * soft_exp(a.m - m)) + (b.s == 0.f ? 0.f : b.s * soft_exp(b.m - m));
    return r;
}

__device__ __forceinline__ SoftStat wave_soft_merge(SoftStat v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        SoftStat o;
        o.m = __shfl_xor(v.m, off, kWave);
        o.s = __shfl_xor(v.s, off, kWave);
        v = soft_merge(v, o);
    }
    return v;
}

// ---- typed loads of 4 consecutive elements of a row.  `vec` says the address is 16-byte (fp32)
// or 8-byte (bf16) aligned and all four are in range; otherwise elements are read one by one and
// those at or beyond `len` come back as `fill`.
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

template <int KIND>
__device__ __forceinline__ float4 load4(const void *row, int64_t i, int64_t len, bool vec, float fill)
{
    float4 v;
    if (KIND == RDK_LOGIT_BF16) {
        const uint16_t *r = (const uint16_t *)row;
        if (vec && i + 3 < len) {
            uint2 raw = *(const uint2 *)(r + i);
            v.x = __uint_as_float(raw.x << 16);
            v.y = __uint_as_float(raw.x & 0xFFFF0000u);
            v.z = __uint_as_float(raw.y << 16);
            v.w = __uint_as_float(raw.y & 0xFFFF0000u);
        } else {
            v.x = i + 0 < len ? bf16_to_f32(r[i + 0]) : fill;
            v.y = i + 1 < len ? bf16_to_f32(r[i + 1]) : fill;
            v.z = i + 2 < len ? bf16_to_f32(r[i + 2]) : fill;
            v.w = i + 3 < len ? bf16_to_f32(r[i + 3]) : fill;
        }
    } else {
        const float *r = (const float *)row;
        if (vec && i + 3 < len) {
            v = *(const float4 *)(r + i);
        } else {
            v.x = i + 0 < len ? r[i + 0] : fill;
            v.y = i + 1 < len ? r[i + 1] : fill;
            v.z = i + 2 < len ? r[i + 2] : fill;
            v.w = i + 3 < len ? r[i + 3] : fill;
        }
    }
    return v;
}

// The same without any check: the caller knows the four elements are in range and the address is aligned.
// STREAM marks the load non-temporal: for data that is read once and should not displace what the caches hold.
template <int KIND, bool STREAM = false>
__device__ __forceinline__ float4 load4_full(const void *row, int64_t i)
{
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
    if (KIND == RDK_LOGIT_BF16) {
        const u32x2_t *src = (const u32x2_t *)((const uint16_t *)row + i);
        const u32x2_t raw = STREAM ? __builtin_nontemporal_load(src) : *src;
        return make_float4(__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xFFFF0000u), __uint_as_float(raw.y << 16),
                           __uint_as_float(raw.y & 0xFFFF0000u));
    }
    const f32x4_t *src = (const f32x4_t *)((const float *)row + i);
    const f32x4_t v = STREAM ? __builtin_nontemporal_load(src) : *src;
    return make_float4(v.x, v.y, v.z, v.w);
}

// The 16 elements a lane holds of one chunk of kChunk ids (ids base + i*256 + lane*4 .. +3, i = 0..3).  A chunk that
// lies wholly inside the row of a vectorisable input is read by four loads behind ONE wavefront-uniform
// branch; per-load range checks cost a dozen scalar and exec-mask instructions each and made the streaming
// kernels issue-bound.  The loads are non-temporal unless STREAM is false: every user reads its rows once per
// launch, and batches are larger than the caches.
template <int KIND, bool STREAM = true>
__device__ __forceinline__ void load_chunk(const void *row, int64_t base, int64_t len, bool vec, float fill, float4 (&v)[4])
{
    const int64_t first = base + lane_id() * 4;
    if (vec && base + kChunk <= len) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = load4_full<KIND, STREAM>(row, first + i * 256);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = load4<KIND>(row, first + i * 256, len, vec, fill);
    }
}

template <int KIND>
__device__ __forceinline__ float load1(const void *row, int64_t i)
{
    if (KIND == RDK_LOGIT_BF16) return bf16_to_f32(((const uint16_t *)row)[i]);
    return ((const float *)row)[i];
}

template <int KIND>
__device__ __forceinline__ const void *row_ptr(const void *base, int64_t ld, int64_t b)
{
    if (KIND == RDK_LOGIT_BF16) return (const void *)((const uint16_t *)base + b * ld);
    return (const void *)((const float *)base + b * ld);
}

inline bool rows_vectorisable(const void *base, int64_t ld, rdk_input_kind_t kind)
{
    if (kind == RDK_LOGIT_BF16) return ((uintptr_t)base % 8 == 0) && (ld % 4 == 0);
    return ((uintptr_t)base % 16 == 0) && (ld % 4 == 0);
}

// Turns a raw element into the weight the method works with: probabilities pass through, logits
// become exp(z - m) * inv (inv = 1 / sum exp for a normalised softmax, 1 for an unnormalised one).
template <int KIND>
__device__ __forceinline__ float to_weight(float x, float m, float inv)
{
    if (KIND == RDK_PROB_F32) return x;
    return soft_exp(x - m) * inv;
}

// ---- Philox4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0,k1), ten rounds.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t out[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ void position_words(uint64_t seed, uint64_t index, uint32_t w[4])
{
    philox4x32_10((uint32_t)index, (uint32_t)(index >> 32), 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), w);
}

__device__ __forceinline__ double word_to_unit(uint32_t w) { return (double)(w >> 8) * (1.0 / 16777216.0); }

}  // namespace rdk
