// Per-row statistics of a [B, len] input, a few partials per row:
//   logits        -> running maximum m and sum of exp(z - m)  (softmax normaliser)
//   probabilities -> m = 0 and the plain sum                   (the normaliser of Eq. 1)
#pragma once
#include "rdk_device.hpp"

namespace rdk {

constexpr int kStatThreads = 256;

template <int KIND>
__global__ __launch_bounds__(kStatThreads) void row_stats_kernel(const void *x, int64_t ld, int64_t len, int splits, bool vec,
                                                                 SoftStat *out)
{
    constexpr int kWaves = kStatThreads / kWave;
    const int64_t row = blockIdx.x / splits;
    const int split = blockIdx.x % splits;
    const int nchunks = (int)((len + kChunk - 1) / kChunk);
    const int cpw = (nchunks + splits - 1) / splits;
    const int c_begin = split * cpw, c_end = min(nchunks, c_begin + cpw);
    const void *xr = row_ptr<KIND>(x, ld, row);
    const int wid = threadIdx.x / kWave, lane = lane_id();
    SoftStat st;
    st.m = KIND == RDK_PROB_F32 ? 0.f : -INFINITY;
    st.s = 0.f;
    for (int c = c_begin + wid; c < c_end; c += kWaves) {
        float4 v[4];   // kept cacheable: the kernels that follow read the same rows again
        load_chunk<KIND, false>(xr, (int64_t)c * kChunk, len, vec, KIND == RDK_PROB_F32 ? 0.f : -INFINITY, v);
        if (KIND == RDK_PROB_F32) {
#pragma unroll
            for (int i = 0; i < 4; ++i) st.s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
        } else {
            float mx = st.m;
#pragma unroll
            for (int i = 0; i < 4; ++i) mx = fmaxf(mx, fmaxf(fmaxf(v[i].x, v[i].y), fmaxf(v[i].z, v[i].w)));
            if (mx > -INFINITY) {
                float s = st.s == 0.f ? 0.f : st.s * soft_exp(st.m - mx);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    s += (soft_exp(v[i].x - mx) + soft_exp(v[i].y - mx)) + (soft_exp(v[i].z - mx) + soft_exp(v[i].w - mx));
                st.m = mx;
                st.s = s;
            }
        }
    }
    if (KIND == RDK_PROB_F32) {
        st.s = wave_sum(st.s);
    } else {
        st = wave_soft_merge(st);
    }
    __shared__ SoftStat sh[kWaves];
    if (lane == 0) sh[wid] = st;
    __syncthreads();
    if (threadIdx.x == 0) {
        SoftStat r = sh[0];
        for (int i = 1; i < kWaves; ++i) {
            if (KIND == RDK_PROB_F32) r.s += sh[i].s;
            else r = soft_merge(r, sh[i]);
        }
        out[row * splits + split] = r;
    }
}

// Merge the partials of one row; every lane of the calling wave receives (m, s).
template <int KIND>
__device__ __forceinline__ SoftStat merged_row_stat(const SoftStat *stat, int splits, int64_t row)
{
    SoftStat v;
    v.m = KIND == RDK_PROB_F32 ? 0.f : -INFINITY;
    v.s = 0.f;
    for (int i = lane_id(); i < splits; i += kWave) {
        const SoftStat o = stat[row * splits + i];
        if (KIND == RDK_PROB_F32) v.s += o.s;
        else v = soft_merge(v, o);
    }
    if (KIND == RDK_PROB_F32) v.s = wave_sum(v.s);
    else v = wave_soft_merge(v);
    return v;
}

template <int KIND>
inline rdk_status_t launch_row_stats(RowInput x, int64_t len, int32_t B, int splits, SoftStat *out, hipStream_t st)
{
    {
        RDK_TIMED_LAUNCH("row_stats_kernel", (row_stats_kernel<KIND>), dim3((unsigned)B * splits), dim3(kStatThreads), 0, st,
                         x.ptr, x.ld, len, splits, rows_vectorisable(x.ptr, x.ld, x.kind), out);
    }
    RDK_LAUNCH_CHECK("row_stats_kernel");
    return RDK_OK;
}

// Number of workgroups that share one row so that a batch of B rows fills the chip.
inline int row_splits(int B, int64_t len, int waves_per_block)
{
    const int nchunks = (int)((len + kChunk - 1) / kChunk);
    int want = (2048 + B - 1) / B;
    const int maxs = (nchunks + waves_per_block - 1) / waves_per_block;
    if (want > maxs) want = maxs;
    if (want > kMaxSplits) want = kMaxSplits;
    return want < 1 ? 1 : want;
}

}  // namespace rdk
