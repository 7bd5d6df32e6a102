// Device-side helpers: wavefront reductions and scans, typed row loads, Philox4x32-10.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rdk_common.hpp"

namespace rdk {

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// ---- 64-wide reductions through cross-lane shuffles
template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

// Inclusive prefix sum over the 64 lanes (Hillis-Steele on shuffles).
__device__ __forceinline__ double wave_inclusive_scan(double v)
{
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        double t = __shfl_up(v, off, kWave);
        if (lane >= off) v += t;
    }
    return v;
}

// ---- softmax statistics (running maximum m and sum of exp(z - m)), merged pairwise
struct SoftStat {
    float m, s;
};

__device__ __forceinline__ SoftStat soft_merge(SoftStat a, SoftStat b)
{
    float m = fmaxf(a.m, b.m);
    SoftStat r;
    r.m = m;
    r.s = (a.s == 0.f ? 0.f : a.s * expf(a.m - m)) + (b.s == 0.f ? 0.f : b.s * expf(b.m - m));
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
    return expf(x - m) * inv;
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
