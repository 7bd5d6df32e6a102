// Internal declarations shared by the translation units of the RDK HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "rdk.h"

namespace rdk {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kChunk = 1024;     // ids summed by one wavefront step: 64 lanes x 4 x float4
constexpr int kMaxSplits = 64;   // upper bound on workgroups sharing one row

// Host-side description of a built kernel; every pointer points into the caller's storage blob.
struct KernelHandle {
    int32_t N, n, k;
    rdk_kernel_format_t format;
    const int32_t *kept_ids;  // [n]
    const int32_t *chunk_lo;  // [ceil(N / kChunk) + 1]: kept ids below c * kChunk, i.e. the first slot of chunk c
    const int32_t *slot_of;   // [N]  >= 0: kept slot;  < 0: -(pruned slot + 1)
    // [ceil(N / kChunk), 64]: what lane l of a wavefront has to know about its 16 ids of a chunk (ids c * kChunk +
    // 256 i + 4 l + e, i, e = 0..3): bit 4 i + e = the id is kept; bits 16 + 12 i .. 27 + 12 i = kept ids of the chunk
    // below id c * kChunk + 256 i + 4 l.  The slot of a kept id follows from these and chunk_lo[c].
    const uint64_t *lane_map;
    // The kept slots cut into pieces of at most 64 consecutive slots that never cross a chunk: piece k is
    // row_items[k] = {first slot, chunk | (first slot of the chunk mod 4) << 22 | length << 24}, pieces ascend with the
    // slots, and the pieces of chunk c are item_lo[c] .. item_lo[c + 1] - 1 (item_lo has ceil(N / kChunk) + 1 entries).
    const int32_t *item_lo;
    const int2 *row_items;
    // sparse: per pruned slot a row of kk (kept slot, weight) pairs, k real ones then (0, 0) padding
    const int32_t *pruned_ids;  // [N-n] ascending target ids that are not kept
    const int2 *nbr;            // [N-n, kk] pairs (kept slot, weight as fp32 bits): one 128-byte line per 16 entries
    const float *self_w;        // [n] diagonal weights
    int32_t kk;                 // row length of the two tables: k rounded up to a multiple of 16
    // dense fp32
    const float *dense;       // [n, ldm]
    int64_t ldm;
    // dense bf16, packed for MFMA operand loads, plus the fp32 row sums of the rounded rows
    const uint16_t *packed;
    const float *row_sum;     // [n]
    int32_t n_pad, N_pad;     // packed extents
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Records a HIP failure for rdk_last_hip_error() and maps it to RDK_ERR_HIP.
rdk_status_t hip_fail(hipError_t e, const char *what);

#define RDK_HIP(call)                                                   \
    do {                                                                \
        hipError_t e_ = (call);                                         \
        if (e_ != hipSuccess) return ::rdk::hip_fail(e_, #call);        \
    } while (0)

#define RDK_LAUNCH_CHECK(name)                                          \
    do {                                                                \
        hipError_t e_ = hipGetLastError();                              \
        if (e_ != hipSuccess) return ::rdk::hip_fail(e_, name);         \
    } while (0)

struct RowInput {            // a [B, len] input of some kind
    const void *ptr;
    rdk_input_kind_t kind;
    int64_t ld;
};

// One fused redistribute + verify call: inputs, the optional q' output, and the verification outputs.
struct FusedCall {
    rdk_verify_desc_t d;
    RowInput p, q;
    float *q_prime;      // may be NULL: q' is then never written
    int64_t ldo;
    int32_t *draft_ids;
    uint8_t *accept;
    float *alpha, *resid_mass;
    int32_t *resid_ids, *n_accepted, *out_tokens;
};

// Launch of an instrumented kernel.  When the kernel has been selected through rdk_timing_select() it is launched
// with a pair of events that take the dispatch's own begin and end timestamps (hipExtLaunchKernelGGL), so the
// measured time is the kernel's, without launch gaps; otherwise this is a plain launch.  Same argument order as
// hipLaunchKernelGGL after the name.
bool timing_events(const char *kernel_name, hipEvent_t *start, hipEvent_t *stop);

#define RDK_TIMED_LAUNCH(NAME, KERNEL, GRID, BLOCK, SHMEM, ST, ...)                                  \
    do {                                                                                             \
        hipEvent_t rdk_ev_a_ = nullptr, rdk_ev_b_ = nullptr;                                         \
        if (rdk::timing_events(NAME, &rdk_ev_a_, &rdk_ev_b_))                                        \
            hipExtLaunchKernelGGL(KERNEL, GRID, BLOCK, SHMEM, ST, rdk_ev_a_, rdk_ev_b_, 0, __VA_ARGS__); \
        else                                                                                         \
            hipLaunchKernelGGL(KERNEL, GRID, BLOCK, SHMEM, ST, __VA_ARGS__);                          \
    } while (0)

// ---- launchers implemented in the kernel translation units (all enqueue on `st`, none synchronises)

// rdk_build.hip
size_t build_workspace_bytes(const rdk_kernel_desc_t &d);
rdk_status_t launch_slot_of(const int32_t *kept_ids, int32_t n, int32_t N, int32_t *slot_of, hipStream_t st);
rdk_status_t launch_check_kept(const int32_t *kept_ids, int32_t n, int32_t N, int32_t *flag, hipStream_t st);
rdk_status_t launch_features_from_scores(const void *z, rdk_input_kind_t kind, int64_t ldz, int32_t T, int32_t N, float *F,
                                         int64_t ldf, hipStream_t st);
rdk_status_t launch_chunk_lo(const int32_t *kept_ids, int32_t n, int32_t N, int32_t *chunk_lo, hipStream_t st);
rdk_status_t launch_row_items(const int32_t *chunk_lo, int32_t N, int32_t *item_lo, int2 *row_items, hipStream_t st);
rdk_status_t launch_lane_map(const int32_t *slot_of, const int32_t *chunk_lo, int32_t N, int32_t n, uint64_t *lane_map,
                             hipStream_t st);
rdk_status_t launch_pruned_ids(const int32_t *slot_of, int32_t N, int32_t n, int32_t *pruned_ids, hipStream_t st);
rdk_status_t launch_build_sparse(const rdk_kernel_desc_t &d, const int32_t *pruned_ids, int2 *nbr, float *self_w,
                                 int32_t kk, void *ws, hipStream_t st);
rdk_status_t launch_import_sparse(const rdk_kernel_desc_t &d, int2 *nbr, float *self_w, int32_t kk, hipStream_t st);
rdk_status_t launch_export_sparse(const KernelHandle &h, int32_t *idx, float *w, float *self_w, hipStream_t st);
rdk_status_t launch_build_dense(const rdk_kernel_desc_t &d, float *M, int64_t ldm, void *ws, hipStream_t st);
rdk_status_t launch_check_stochastic_dense(const float *M, int64_t ldm, int32_t n, int32_t N, int32_t *flag,
                                           hipStream_t st);
rdk_status_t launch_check_stochastic_sparse(const KernelHandle &h, void *ws, int32_t *flag, hipStream_t st);

// rdk_linear.hip
size_t taylor_workspace_bytes(const KernelHandle &h, int32_t B);
size_t taylor_fused_workspace_bytes(const KernelHandle &h, int32_t B);
// c == NULL: Eq. 3 into `out`; else the fused redistribute + verify call (out may then be NULL)
rdk_status_t launch_taylor(const KernelHandle &h, RowInput p, RowInput q, int32_t B, float *out, int64_t ldo,
                           void *ws, const FusedCall *c, hipStream_t st);
rdk_status_t launch_tli_scatter(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws,
                                hipStream_t st);

// rdk_sparse.hip
size_t sparse_workspace_bytes(const KernelHandle &h, int32_t B);
size_t sparse_fused_workspace_bytes(const KernelHandle &h, int32_t B);
rdk_status_t launch_sparse_fused(const KernelHandle &h, const FusedCall &c, void *ws, hipStream_t st);
rdk_status_t launch_sparse(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws,
                           hipStream_t st);

// rdk_exact.hip
size_t exact_workspace_bytes(const KernelHandle &h, int32_t B);
size_t sparse_draft_workspace_bytes(const KernelHandle &h, int32_t B);
rdk_status_t launch_sparse_draft(const KernelHandle &h, RowInput q, int32_t B, uint64_t seed, uint64_t offset, int32_t *draft_ids,
                                 float *q_draft, float *q_prime, int64_t ldo, void *ws, hipStream_t st);
size_t draft_rows_workspace_bytes(int32_t B, int32_t N);
rdk_status_t launch_draft_from_rows(const float *q_prime, int64_t ldq, int32_t B, int32_t N, uint64_t seed, uint64_t offset,
                                    int32_t *draft_ids, float *q_draft, void *ws, hipStream_t st);
size_t packed_bf16_bytes(int32_t n, int32_t N, int32_t *n_pad, int32_t *N_pad);
rdk_status_t launch_pack_bf16(const float *M, int64_t ldm, int32_t n, int32_t N, uint16_t *packed, float *row_sum,
                              hipStream_t st);
rdk_status_t launch_unpack_bf16(const KernelHandle &h, float *M, int64_t ldm, hipStream_t st);
rdk_status_t launch_exact(const KernelHandle &h, RowInput q, int32_t B, float *out, int64_t ldo, void *ws,
                          hipStream_t st);

// rdk_multi.hip
int multi_max_ids();
int multi_max_candidates();
size_t multi_workspace_bytes(const rdk_multi_desc_t &d, rdk_input_kind_t p_kind);
rdk_status_t launch_verify_multi(const rdk_multi_desc_t &d, RowInput p, const float *q_prime, int64_t ldq, int32_t *cand_ids,
                                 int32_t *accepted, int32_t *token, float *resid_mass, void *ws, hipStream_t st);

rdk_status_t launch_tree_walk(int32_t S, int32_t nodes, int32_t C, const int32_t *child_node, const int32_t *accepted,
                              const int32_t *token, int32_t *n_accepted, int32_t *out_tokens, hipStream_t st);

// rdk_verify.hip
size_t verify_workspace_bytes(const rdk_verify_desc_t &d);
rdk_status_t launch_verify(const rdk_verify_desc_t &d, RowInput p, const float *q_prime, int64_t ldq,
                           int32_t *draft_ids, uint8_t *accept, float *alpha, float *resid_mass,
                           int32_t *resid_ids, int32_t *n_accepted, int32_t *out_tokens, void *ws, hipStream_t st);
size_t verify_static_scratch_limit();
rdk_status_t launch_verify_static(const rdk_verify_desc_t &d, RowInput p, const float *q_prime, int64_t ldq,
                                  int32_t *draft_ids, uint8_t *accept, float *alpha, float *resid_mass,
                                  int32_t *resid_ids, int32_t *n_accepted, int32_t *out_tokens, hipStream_t st);
rdk_status_t launch_philox_words(uint64_t seed, uint64_t offset, int32_t count, uint32_t *words, hipStream_t st);

}  // namespace rdk
