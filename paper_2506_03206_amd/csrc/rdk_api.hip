// C ABI of the RDK library: argument checks, storage / workspace carving, dispatch to the launchers.
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "rdk_common.hpp"

namespace rdk {

static thread_local std::string g_last_hip_error;

rdk_status_t hip_fail(hipError_t e, const char *what)
{
    g_last_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return RDK_ERR_HIP;
}

// ---- optional event timing of selected kernels (used by benchmarks)
namespace {
struct TimedRecord {
    std::string name;
    hipEvent_t start, stop;
};
std::mutex g_timing_mutex;
std::string g_timing_selected;             // "" = off, "*" = every instrumented kernel
long g_timing_every = 1, g_timing_seen = 0;   // of the launches of the selected kernel, every g_timing_every-th is timed
std::vector<TimedRecord> g_timing_records;
std::vector<hipEvent_t> g_timing_free;

hipEvent_t timing_event()
{
    if (!g_timing_free.empty()) {
        hipEvent_t e = g_timing_free.back();
        g_timing_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

bool timing_events(const char *kernel_name, hipEvent_t *start, hipEvent_t *stop)
{
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    if (g_timing_selected.empty()) return false;
    if (g_timing_selected != "*" && g_timing_selected != kernel_name) return false;
    if (g_timing_seen++ % g_timing_every != 0) return false;
    hipEvent_t a = timing_event(), b = timing_event();
    if (!a || !b) return false;
    g_timing_records.push_back(TimedRecord{kernel_name, a, b});
    *start = a;
    *stop = b;
    return true;
}

namespace {

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

bool kind_ok(rdk_input_kind_t k) { return k == RDK_PROB_F32 || k == RDK_LOGIT_F32 || k == RDK_LOGIT_BF16; }

int32_t nbr_row_len(int32_t k) { return ((k < 1 ? 1 : k) + 15) / 16 * 16; }

struct StorageLayout {
    size_t kept_ids, slot_of, pruned_ids, chunk_lo, lane_map, item_lo, row_items, body, body2, body3, total;
    int32_t kk, n_pad, N_pad;
    int64_t ldm;
};

rdk_status_t check_desc(const rdk_kernel_desc_t *d)
{
    if (!d) return RDK_ERR_NULL;
    if (d->N < 1 || d->n < 1 || d->n > d->N) return RDK_ERR_SHAPE;
    if (!d->kept_ids) return RDK_ERR_NULL;
    if (!aligned16(d->kept_ids)) return RDK_ERR_ALIGN;
    switch (d->format) {
        case RDK_IDENTITY:
            return RDK_OK;
        case RDK_SPARSE_TOPK:
            if (d->k < 0 || d->k > 64 || d->k > d->n) return RDK_ERR_SHAPE;
            if (d->sparse_idx || d->sparse_w || d->self_w) {
                if (!d->self_w || (d->k > 0 && d->N > d->n && (!d->sparse_idx || !d->sparse_w))) return RDK_ERR_NULL;
                return RDK_OK;
            }
            if (d->k == 0 || d->N == d->n) return RDK_OK;   // nothing but the diagonal
            break;
        case RDK_DENSE_F32:
        case RDK_DENSE_BF16:
            if (d->dense_M) return aligned16(d->dense_M) ? RDK_OK : RDK_ERR_ALIGN;
            break;
        default:
            return RDK_ERR_DTYPE;
    }
    if (!d->embeddings) return RDK_ERR_NULL;
    if (!aligned16(d->embeddings)) return RDK_ERR_ALIGN;
    if (d->d < 1) return RDK_ERR_SHAPE;
    if (!(d->tau > 0.f)) return RDK_ERR_SHAPE;
    return RDK_OK;
}

StorageLayout layout_of(const rdk_kernel_desc_t &d)
{
    StorageLayout L{};
    size_t off = 0;
    L.kept_ids = off; off += align_up((size_t)d.n * 4, 256);
    L.slot_of = off; off += align_up((size_t)d.N * 4, 256);
    L.pruned_ids = off; off += align_up((size_t)(d.N - d.n + 1) * 4, 256);
    L.chunk_lo = off; off += align_up((size_t)((d.N + kChunk - 1) / kChunk + 1) * 4, 256);
    L.lane_map = off; off += align_up((size_t)((d.N + kChunk - 1) / kChunk) * kWave * 8, 256);
    L.item_lo = off; off += align_up((size_t)((d.N + kChunk - 1) / kChunk + 1) * 4, 256);
    L.row_items = off; off += align_up((size_t)((d.N + kChunk - 1) / kChunk + d.n / 64 + 1) * 8, 256);
    L.kk = nbr_row_len(d.k);
    L.ldm = ((int64_t)d.N + 3) / 4 * 4;
    switch (d.format) {
        case RDK_SPARSE_TOPK:
            L.body = off; off += align_up((size_t)(d.N - d.n) * L.kk * 8 + 512, 256);
            L.body3 = off; off += align_up((size_t)d.n * 4, 256);
            break;
        case RDK_DENSE_F32:
            L.body = off; off += align_up((size_t)d.n * L.ldm * 4, 256);
            break;
        case RDK_DENSE_BF16:
            L.body = off; off += align_up(packed_bf16_bytes(d.n, d.N, &L.n_pad, &L.N_pad), 256);
            L.body2 = off; off += align_up((size_t)d.n * 4, 256);
            break;
        default:
            break;
    }
    L.total = off;
    return L;
}

// scratch of the build: flag word, generic build scratch, and for bf16 the fp32 matrix that gets packed
size_t build_ws_total(const rdk_kernel_desc_t &d, const StorageLayout &L)
{
    size_t b = 256 + build_workspace_bytes(d);
    if (d.format == RDK_DENSE_BF16 && !d.dense_M) b += align_up((size_t)d.n * L.ldm * 4, 256);
    return b;
}

}  // namespace
}  // namespace rdk

using namespace rdk;

struct rdk_kernel {
    KernelHandle h;
};

extern "C" {

const char *rdk_status_string(rdk_status_t s)
{
    switch (s) {
        case RDK_OK: return "ok";
        case RDK_ERR_NULL: return "a required pointer is NULL";
        case RDK_ERR_SHAPE: return "a size, leading dimension or count is out of range";
        case RDK_ERR_DTYPE: return "unknown input kind, kernel format or mode";
        case RDK_ERR_KEPT_IDS: return "kept ids are not strictly ascending ids inside the target vocabulary";
        case RDK_ERR_NOT_STOCHASTIC: return "the supplied kernel is not row-stochastic";
        case RDK_ERR_WORKSPACE: return "workspace or storage too small";
        case RDK_ERR_UNSUPPORTED: return "this combination of kernel format and operation is not offered";
        case RDK_ERR_HIP: return "a HIP call failed";
        case RDK_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
    }
    return "unknown status";
}

const char *rdk_last_hip_error(void) { return g_last_hip_error.c_str(); }

rdk_status_t rdk_kernel_storage_bytes(const rdk_kernel_desc_t *desc, size_t *storage_bytes, size_t *build_workspace_bytes)
{
    rdk_status_t rc = check_desc(desc);
    if (rc != RDK_OK) return rc;
    if (!storage_bytes || !build_workspace_bytes) return RDK_ERR_NULL;
    const StorageLayout L = layout_of(*desc);
    *storage_bytes = L.total;
    *build_workspace_bytes = build_ws_total(*desc, L);
    return RDK_OK;
}

rdk_status_t rdk_features_from_scores(const void *z, rdk_input_kind_t z_kind, int64_t ldz, int32_t T, int32_t N, float *features,
                                      int64_t ldf, void *stream)
{
    if (!z || !features) return RDK_ERR_NULL;
    if (!kind_ok(z_kind)) return RDK_ERR_DTYPE;
    if (T < 2 || N < 1 || ldz < N || ldf < T) return RDK_ERR_SHAPE;
    if (!aligned16(z) || !aligned16(features)) return RDK_ERR_ALIGN;
    return launch_features_from_scores(z, z_kind, ldz, T, N, features, ldf, (hipStream_t)stream);
}

rdk_status_t rdk_build_kernel(const rdk_kernel_desc_t *desc, void *storage, size_t storage_bytes, void *workspace,
                              size_t workspace_bytes, void *stream, rdk_kernel_t **out)
{
    rdk_status_t rc = check_desc(desc);
    if (rc != RDK_OK) return rc;
    if (!storage || !workspace || !out) return RDK_ERR_NULL;
    if (!aligned16(storage) || !aligned16(workspace)) return RDK_ERR_ALIGN;
    const rdk_kernel_desc_t &d = *desc;
    const StorageLayout L = layout_of(d);
    if (storage_bytes < L.total || workspace_bytes < build_ws_total(d, L)) return RDK_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char *sp = (char *)storage;
    int32_t *flag = (int32_t *)workspace;
    char *ws = (char *)workspace + 256;

    KernelHandle h{};
    h.N = d.N; h.n = d.n; h.k = d.format == RDK_SPARSE_TOPK ? d.k : 0;
    h.format = d.format;
    int32_t *kept = (int32_t *)(sp + L.kept_ids);
    int32_t *slot_of = (int32_t *)(sp + L.slot_of);
    h.kept_ids = kept;
    h.slot_of = slot_of;

    if (d.validate) {
        rc = launch_check_kept(d.kept_ids, d.n, d.N, flag, st);
        if (rc != RDK_OK) return rc;
        int32_t bad = 0;
        RDK_HIP(hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, st));
        RDK_HIP(hipStreamSynchronize(st));
        if (bad) return RDK_ERR_KEPT_IDS;
    }
    RDK_HIP(hipMemcpyAsync(kept, d.kept_ids, (size_t)d.n * 4, hipMemcpyDeviceToDevice, st));
    rc = launch_slot_of(kept, d.n, d.N, slot_of, st);
    if (rc != RDK_OK) return rc;
    int32_t *pruned = (int32_t *)(sp + L.pruned_ids);
    h.pruned_ids = pruned;
    rc = launch_pruned_ids(slot_of, d.N, d.n, pruned, st);
    if (rc != RDK_OK) return rc;
    int32_t *chunk_lo = (int32_t *)(sp + L.chunk_lo);
    h.chunk_lo = chunk_lo;
    rc = launch_chunk_lo(kept, d.n, d.N, chunk_lo, st);
    if (rc != RDK_OK) return rc;
    uint64_t *lane_map = (uint64_t *)(sp + L.lane_map);
    h.lane_map = lane_map;
    rc = launch_lane_map(slot_of, chunk_lo, d.N, d.n, lane_map, st);
    if (rc != RDK_OK) return rc;
    int32_t *item_lo = (int32_t *)(sp + L.item_lo);
    int2 *row_items = (int2 *)(sp + L.row_items);
    h.item_lo = item_lo;
    h.row_items = row_items;
    rc = launch_row_items(chunk_lo, d.N, item_lo, row_items, st);
    if (rc != RDK_OK) return rc;

    if (d.format == RDK_SPARSE_TOPK) {
        h.kk = L.kk;
        int2 *nbr = (int2 *)(sp + L.body);
        float *self_w = (float *)(sp + L.body3);
        h.nbr = nbr;
        h.self_w = self_w;
        if (d.self_w) rc = launch_import_sparse(d, nbr, self_w, L.kk, st);
        else rc = launch_build_sparse(d, pruned, nbr, self_w, L.kk, ws, st);
        if (rc != RDK_OK) return rc;
        if (d.validate && d.self_w) {
            rc = launch_check_stochastic_sparse(h, ws, flag, st);
            if (rc != RDK_OK) return rc;
            int32_t bad = 0;
            RDK_HIP(hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, st));
            RDK_HIP(hipStreamSynchronize(st));
            if (bad) return RDK_ERR_NOT_STOCHASTIC;
        }
    } else if (d.format == RDK_DENSE_F32 || d.format == RDK_DENSE_BF16) {
        const bool bf16 = d.format == RDK_DENSE_BF16;
        float *M32 = bf16 ? (float *)(ws + build_workspace_bytes(d)) : (float *)(sp + L.body);
        const float *src = M32;
        int64_t ld_src = L.ldm;
        if (d.dense_M) {
            if (d.validate) {
                rc = launch_check_stochastic_dense(d.dense_M, d.N, d.n, d.N, flag, st);
                if (rc != RDK_OK) return rc;
                int32_t bad = 0;
                RDK_HIP(hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, st));
                RDK_HIP(hipStreamSynchronize(st));
                if (bad) return RDK_ERR_NOT_STOCHASTIC;
            }
            if (bf16) {
                src = d.dense_M;
                ld_src = d.N;
            } else {
                RDK_HIP(hipMemcpy2DAsync(M32, (size_t)L.ldm * 4, d.dense_M, (size_t)d.N * 4, (size_t)d.N * 4, (size_t)d.n,
                                         hipMemcpyDeviceToDevice, st));
            }
        } else {
            rc = launch_build_dense(d, M32, L.ldm, ws, st);
            if (rc != RDK_OK) return rc;
        }
        if (bf16) {
            uint16_t *packed = (uint16_t *)(sp + L.body);
            float *row_sum = (float *)(sp + L.body2);
            rc = launch_pack_bf16(src, ld_src, d.n, d.N, packed, row_sum, st);
            if (rc != RDK_OK) return rc;
            h.packed = packed;
            h.row_sum = row_sum;
            h.n_pad = L.n_pad;
            h.N_pad = L.N_pad;
        } else {
            h.dense = M32;
            h.ldm = L.ldm;
        }
    }
    rdk_kernel *k = new (std::nothrow) rdk_kernel;
    if (!k) return RDK_ERR_WORKSPACE;
    k->h = h;
    *out = k;
    return RDK_OK;
}

rdk_status_t rdk_destroy_kernel(rdk_kernel_t *kernel)
{
    delete kernel;
    return RDK_OK;
}

rdk_status_t rdk_kernel_get_sparse(const rdk_kernel_t *kernel, int32_t *sparse_idx, float *sparse_w, float *self_w,
                                   void *stream)
{
    if (!kernel || !self_w) return RDK_ERR_NULL;
    const KernelHandle &h = kernel->h;
    if (h.format != RDK_SPARSE_TOPK) return RDK_ERR_UNSUPPORTED;
    if (h.k > 0 && h.N > h.n && (!sparse_idx || !sparse_w)) return RDK_ERR_NULL;
    return launch_export_sparse(h, sparse_idx, sparse_w, self_w, (hipStream_t)stream);
}

rdk_status_t rdk_kernel_get_dense(const rdk_kernel_t *kernel, float *dense_M, int64_t ldm, void *stream)
{
    if (!kernel || !dense_M) return RDK_ERR_NULL;
    const KernelHandle &h = kernel->h;
    if (ldm < h.N) return RDK_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    if (h.format == RDK_DENSE_F32) {
        RDK_HIP(hipMemcpy2DAsync(dense_M, (size_t)ldm * 4, h.dense, (size_t)h.ldm * 4, (size_t)h.N * 4, (size_t)h.n,
                                 hipMemcpyDeviceToDevice, st));
        return RDK_OK;
    }
    if (h.format == RDK_DENSE_BF16) return launch_unpack_bf16(h, dense_M, ldm, st);
    return RDK_ERR_UNSUPPORTED;
}

rdk_status_t rdk_workspace_bytes(const rdk_kernel_t *kernel, int32_t B, size_t *bytes)
{
    if (!kernel || !bytes) return RDK_ERR_NULL;
    if (B < 1) return RDK_ERR_SHAPE;
    size_t need = taylor_workspace_bytes(kernel->h, B);
    const size_t b = exact_workspace_bytes(kernel->h, B), c = sparse_workspace_bytes(kernel->h, B);
    if (b > need) need = b;
    if (c > need) need = c;
    *bytes = need + 256;
    return RDK_OK;
}

static rdk_status_t check_rows(const void *ptr, rdk_input_kind_t kind, int64_t ld, int64_t len)
{
    if (!ptr) return RDK_ERR_NULL;
    if (!kind_ok(kind)) return RDK_ERR_DTYPE;
    if (ld < len) return RDK_ERR_SHAPE;
    if (!aligned16(ptr)) return RDK_ERR_ALIGN;
    return RDK_OK;
}

rdk_status_t rdk_redistribute_exact(const rdk_kernel_t *kernel, const void *q, rdk_input_kind_t q_kind, int64_t ldq,
                                    int32_t B, float *q_prime, int64_t ldo, void *workspace, size_t workspace_bytes,
                                    void *stream)
{
    if (!kernel || !q_prime || !workspace) return RDK_ERR_NULL;
    const KernelHandle &h = kernel->h;
    if (B < 1 || ldo < h.N) return RDK_ERR_SHAPE;
    rdk_status_t rc = check_rows(q, q_kind, ldq, h.n);
    if (rc != RDK_OK) return rc;
    if (!aligned16(q_prime) || !aligned16(workspace)) return RDK_ERR_ALIGN;
    if (h.format == RDK_SPARSE_TOPK) return RDK_ERR_UNSUPPORTED;
    size_t need = 0;
    rdk_workspace_bytes(kernel, B, &need);
    if (workspace_bytes < need) return RDK_ERR_WORKSPACE;
    RowInput qi{q, q_kind, ldq};
    if (h.format == RDK_IDENTITY) return launch_tli_scatter(h, qi, B, q_prime, ldo, workspace, (hipStream_t)stream);
    return launch_exact(h, qi, B, q_prime, ldo, workspace, (hipStream_t)stream);
}

rdk_status_t rdk_redistribute_linear(const rdk_kernel_t *kernel, rdk_linear_mode_t mode, const void *p,
                                     rdk_input_kind_t p_kind, int64_t ldp, const void *q, rdk_input_kind_t q_kind,
                                     int64_t ldq, int32_t B, float *q_prime, int64_t ldo, void *workspace,
                                     size_t workspace_bytes, void *stream)
{
    if (!kernel || !q_prime || !workspace) return RDK_ERR_NULL;
    const KernelHandle &h = kernel->h;
    if (mode != RDK_LINEAR_TAYLOR && mode != RDK_LINEAR_SPARSE) return RDK_ERR_DTYPE;
    if (B < 1 || ldo < h.N) return RDK_ERR_SHAPE;
    rdk_status_t rc = check_rows(q, q_kind, ldq, h.n);
    if (rc != RDK_OK) return rc;
    if (!aligned16(q_prime) || !aligned16(workspace)) return RDK_ERR_ALIGN;
    size_t need = 0;
    rdk_workspace_bytes(kernel, B, &need);
    if (workspace_bytes < need) return RDK_ERR_WORKSPACE;
    RowInput qi{q, q_kind, ldq};
    if (mode == RDK_LINEAR_TAYLOR) {
        rc = check_rows(p, p_kind, ldp, h.N);
        if (rc != RDK_OK) return rc;
        RowInput pi{p, p_kind, ldp};
        return launch_taylor(h, pi, qi, B, q_prime, ldo, workspace, nullptr, (hipStream_t)stream);
    }
    if (h.format != RDK_SPARSE_TOPK && h.format != RDK_IDENTITY) return RDK_ERR_UNSUPPORTED;
    if (h.format == RDK_IDENTITY) return launch_tli_scatter(h, qi, B, q_prime, ldo, workspace, (hipStream_t)stream);
    return launch_sparse(h, qi, B, q_prime, ldo, workspace, (hipStream_t)stream);
}

// k = 0 is stored as one padded row of zero weights per pruned id, so the same kernels serve it
static bool sparse_product_kernel_of(const KernelHandle &h) { return h.format == RDK_SPARSE_TOPK; }

rdk_status_t rdk_sample_draft_workspace_bytes(const rdk_kernel_t *kernel, int32_t B, size_t *bytes)
{
    if (!kernel || !bytes) return RDK_ERR_NULL;
    if (B < 1) return RDK_ERR_SHAPE;
    const KernelHandle &h = kernel->h;
    if (sparse_product_kernel_of(h)) {
        *bytes = sparse_draft_workspace_bytes(h, B) + 256;
    } else {
        size_t redistribute = 0;
        rdk_workspace_bytes(kernel, B, &redistribute);
        *bytes = align_up(redistribute, 256) + draft_rows_workspace_bytes(B, h.N) + 256;
    }
    return RDK_OK;
}

rdk_status_t rdk_sample_draft(const rdk_kernel_t *kernel, const void *q, rdk_input_kind_t q_kind, int64_t ldq, int32_t B,
                              uint64_t seed, uint64_t offset, int32_t *draft_ids, float *q_draft, float *q_prime, int64_t ldo,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    if (!kernel || !draft_ids || !workspace) return RDK_ERR_NULL;
    const KernelHandle &h = kernel->h;
    if (B < 1) return RDK_ERR_SHAPE;
    rdk_status_t rc = check_rows(q, q_kind, ldq, h.n);
    if (rc != RDK_OK) return rc;
    if (q_prime && ldo < h.N) return RDK_ERR_SHAPE;
    if (!aligned16(workspace) || (q_prime && !aligned16(q_prime))) return RDK_ERR_ALIGN;
    size_t need = 0;
    rdk_sample_draft_workspace_bytes(kernel, B, &need);
    if (workspace_bytes < need - 256) return RDK_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    RowInput qi{q, q_kind, ldq};
    if (sparse_product_kernel_of(h))
        return launch_sparse_draft(h, qi, B, seed, offset, draft_ids, q_draft, q_prime, ldo, workspace, st);
    if (!q_prime) return RDK_ERR_NULL;
    size_t redistribute = 0;
    rdk_workspace_bytes(kernel, B, &redistribute);
    if (h.format == RDK_IDENTITY || h.format == RDK_SPARSE_TOPK) rc = launch_tli_scatter(h, qi, B, q_prime, ldo, workspace, st);
    else rc = launch_exact(h, qi, B, q_prime, ldo, workspace, st);
    if (rc != RDK_OK) return rc;
    return launch_draft_from_rows(q_prime, ldo, B, h.N, seed, offset, draft_ids, q_draft,
                                  (char *)workspace + align_up(redistribute, 256), st);
}

static rdk_status_t check_verify_desc(const rdk_verify_desc_t *d)
{
    if (!d) return RDK_ERR_NULL;
    if (d->B < 1 || d->N < 1 || d->gamma < 0) return RDK_ERR_SHAPE;
    if (d->gamma > 0 && d->B % d->gamma != 0) return RDK_ERR_SHAPE;
    return RDK_OK;
}

rdk_status_t rdk_verify_workspace_bytes(const rdk_verify_desc_t *desc, size_t *bytes)
{
    rdk_status_t rc = check_verify_desc(desc);
    if (rc != RDK_OK) return rc;
    if (!bytes) return RDK_ERR_NULL;
    *bytes = verify_workspace_bytes(*desc) + 256;
    return RDK_OK;
}

rdk_status_t rdk_verify_sample(const rdk_verify_desc_t *desc, const void *p, rdk_input_kind_t p_kind, int64_t ldp,
                               const float *q_prime, int64_t ldq, int32_t *draft_ids, uint8_t *accept, float *alpha,
                               float *resid_mass, int32_t *resid_ids, int32_t *n_accepted, int32_t *out_tokens,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    rdk_status_t rc = check_verify_desc(desc);
    if (rc != RDK_OK) return rc;
    rc = check_rows(p, p_kind, ldp, desc->N);
    if (rc != RDK_OK) return rc;
    if (!accept || !resid_ids || !workspace) return RDK_ERR_NULL;
    if (q_prime) {
        if (!draft_ids) return RDK_ERR_NULL;
        if (ldq < desc->N) return RDK_ERR_SHAPE;
        if (!aligned16(q_prime)) return RDK_ERR_ALIGN;
    } else if (desc->gamma != 0 || n_accepted || out_tokens) {
        return RDK_ERR_UNSUPPORTED;
    }
    if (desc->gamma == 0 && (n_accepted || out_tokens)) return RDK_ERR_SHAPE;
    if (!aligned16(workspace)) return RDK_ERR_ALIGN;
    if (workspace_bytes < verify_workspace_bytes(*desc)) return RDK_ERR_WORKSPACE;
    RowInput pi{p, p_kind, ldp};
    return launch_verify(*desc, pi, q_prime, ldq, draft_ids, accept, alpha, resid_mass, resid_ids, n_accepted, out_tokens,
                         workspace, (hipStream_t)stream);
}

rdk_status_t rdk_verify_sample_static(const rdk_verify_desc_t *desc, const void *p, rdk_input_kind_t p_kind, int64_t ldp,
                                      const float *q_prime, int64_t ldq, int32_t *draft_ids, uint8_t *accept, float *alpha,
                                      float *resid_mass, int32_t *resid_ids, int32_t *n_accepted, int32_t *out_tokens,
                                      void *stream)
{
    rdk_status_t rc = check_verify_desc(desc);
    if (rc != RDK_OK) return rc;
    rc = check_rows(p, p_kind, ldp, desc->N);
    if (rc != RDK_OK) return rc;
    if (!accept || !resid_ids) return RDK_ERR_NULL;
    if (q_prime) {
        if (!draft_ids) return RDK_ERR_NULL;
        if (ldq < desc->N) return RDK_ERR_SHAPE;
        if (!aligned16(q_prime)) return RDK_ERR_ALIGN;
    } else if (desc->gamma != 0 || n_accepted || out_tokens) {
        return RDK_ERR_UNSUPPORTED;
    }
    if (desc->gamma == 0 && (n_accepted || out_tokens)) return RDK_ERR_SHAPE;
    if (verify_workspace_bytes(*desc) > verify_static_scratch_limit()) return RDK_ERR_WORKSPACE;
    RowInput pi{p, p_kind, ldp};
    return launch_verify_static(*desc, pi, q_prime, ldq, draft_ids, accept, alpha, resid_mass, resid_ids, n_accepted,
                                out_tokens, (hipStream_t)stream);
}

static rdk_status_t check_multi_desc(const rdk_multi_desc_t *d)
{
    if (!d) return RDK_ERR_NULL;
    if (d->B <= 0 || d->N <= 0 || d->C <= 0) return RDK_ERR_SHAPE;
    if (d->C > multi_max_candidates() || d->N > multi_max_ids()) return RDK_ERR_UNSUPPORTED;
    return RDK_OK;
}

rdk_status_t rdk_verify_multi_workspace_bytes(const rdk_multi_desc_t *desc, rdk_input_kind_t p_kind, size_t *bytes)
{
    if (!bytes) return RDK_ERR_NULL;
    rdk_status_t rc = check_multi_desc(desc);
    if (rc != RDK_OK) return rc;
    if (!kind_ok(p_kind)) return RDK_ERR_DTYPE;
    *bytes = multi_workspace_bytes(*desc, p_kind) + 256;
    return RDK_OK;
}

rdk_status_t rdk_verify_multi(const rdk_multi_desc_t *desc, const void *p, rdk_input_kind_t p_kind, int64_t ldp,
                              const float *q_prime, int64_t ldq, int32_t *cand_ids, int32_t *accepted, int32_t *token,
                              float *resid_mass, void *workspace, size_t workspace_bytes, void *stream)
{
    rdk_status_t rc = check_multi_desc(desc);
    if (rc != RDK_OK) return rc;
    rc = check_rows(p, p_kind, ldp, desc->N);
    if (rc != RDK_OK) return rc;
    if (!q_prime || !cand_ids || !accepted || !token || !workspace) return RDK_ERR_NULL;
    if (ldq < desc->N) return RDK_ERR_SHAPE;
    if (!aligned16(q_prime) || !aligned16(workspace)) return RDK_ERR_ALIGN;
    if (workspace_bytes < multi_workspace_bytes(*desc, p_kind)) return RDK_ERR_WORKSPACE;
    RowInput pi{p, p_kind, ldp};
    return launch_verify_multi(*desc, pi, q_prime, ldq, cand_ids, accepted, token, resid_mass, workspace, (hipStream_t)stream);
}

rdk_status_t rdk_tree_walk(int32_t S, int32_t nodes, int32_t C, const int32_t *child_node, const int32_t *accepted,
                           const int32_t *token, int32_t *n_accepted, int32_t *out_tokens, void *stream)
{
    if (S <= 0 || nodes <= 0 || C <= 0) return RDK_ERR_SHAPE;
    if (!child_node || !accepted || !token || !n_accepted || !out_tokens) return RDK_ERR_NULL;
    return launch_tree_walk(S, nodes, C, child_node, accepted, token, n_accepted, out_tokens, (hipStream_t)stream);
}

rdk_status_t rdk_redistribute_verify_workspace_bytes(const rdk_kernel_t *kernel, rdk_linear_mode_t mode,
                                                     const rdk_verify_desc_t *desc, size_t *bytes)
{
    if (!kernel || !bytes) return RDK_ERR_NULL;
    rdk_status_t rc = check_verify_desc(desc);
    if (rc != RDK_OK) return rc;
    const KernelHandle &h = kernel->h;
    if (desc->N != h.N) return RDK_ERR_SHAPE;
    if (mode == RDK_LINEAR_TAYLOR) *bytes = taylor_fused_workspace_bytes(h, desc->B) + 256;
    else if (mode == RDK_LINEAR_SPARSE && h.format == RDK_SPARSE_TOPK)
        *bytes = sparse_fused_workspace_bytes(h, desc->B) + 256;
    else return mode == RDK_LINEAR_SPARSE ? RDK_ERR_UNSUPPORTED : RDK_ERR_DTYPE;
    return RDK_OK;
}

rdk_status_t rdk_redistribute_verify(const rdk_kernel_t *kernel, rdk_linear_mode_t mode, const rdk_verify_desc_t *desc,
                                     const void *p, rdk_input_kind_t p_kind, int64_t ldp, const void *q,
                                     rdk_input_kind_t q_kind, int64_t ldq, float *q_prime, int64_t ldo, int32_t *draft_ids,
                                     uint8_t *accept, float *alpha, float *resid_mass, int32_t *resid_ids,
                                     int32_t *n_accepted, int32_t *out_tokens, void *workspace, size_t workspace_bytes,
                                     void *stream)
{
    size_t need = 0;
    rdk_status_t rc = rdk_redistribute_verify_workspace_bytes(kernel, mode, desc, &need);
    if (rc != RDK_OK) return rc;
    const KernelHandle &h = kernel->h;
    rc = check_rows(p, p_kind, ldp, h.N);
    if (rc != RDK_OK) return rc;
    rc = check_rows(q, q_kind, ldq, h.n);
    if (rc != RDK_OK) return rc;
    if (!draft_ids || !accept || !resid_ids || !workspace) return RDK_ERR_NULL;
    if (q_prime && ldo < h.N) return RDK_ERR_SHAPE;
    if (desc->gamma == 0 && (n_accepted || out_tokens)) return RDK_ERR_SHAPE;
    if ((q_prime && !aligned16(q_prime)) || !aligned16(workspace)) return RDK_ERR_ALIGN;
    if (workspace_bytes < need) return RDK_ERR_WORKSPACE;
    FusedCall c{};
    c.d = *desc;
    c.p = RowInput{p, p_kind, ldp};
    c.q = RowInput{q, q_kind, ldq};
    c.q_prime = q_prime; c.ldo = ldo;
    c.draft_ids = draft_ids; c.accept = accept; c.alpha = alpha; c.resid_mass = resid_mass;
    c.resid_ids = resid_ids; c.n_accepted = n_accepted; c.out_tokens = out_tokens;
    if (mode == RDK_LINEAR_TAYLOR) return launch_taylor(h, c.p, c.q, desc->B, q_prime, ldo, workspace, &c, (hipStream_t)stream);
    return launch_sparse_fused(h, c, workspace, (hipStream_t)stream);
}

rdk_status_t rdk_timing_select(const char *kernel_name)
{
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    g_timing_selected = kernel_name ? kernel_name : "";
    g_timing_every = 1;
    g_timing_seen = 0;
    const size_t slash = g_timing_selected.find('/');   // "name/8": every eighth launch
    if (slash != std::string::npos) {
        const long every = std::atol(g_timing_selected.c_str() + slash + 1);
        g_timing_every = every > 0 ? every : 1;
        g_timing_selected.resize(slash);
    }
    return RDK_OK;
}

rdk_status_t rdk_timing_read(const char *kernel_name, int64_t *launches, double *total_ms)
{
    if (!kernel_name || !launches || !total_ms) return RDK_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    int64_t count = 0;
    double total = 0.0;
    std::vector<TimedRecord> keep;
    for (TimedRecord &r : g_timing_records) {
        if (r.name != kernel_name) {
            keep.push_back(r);
            continue;
        }
        RDK_HIP(hipEventSynchronize(r.stop));
        float ms = 0.f;
        RDK_HIP(hipEventElapsedTime(&ms, r.start, r.stop));
        total += (double)ms;
        ++count;
        g_timing_free.push_back(r.start);
        g_timing_free.push_back(r.stop);
    }
    g_timing_records.swap(keep);
    *launches = count;
    *total_ms = total;
    return RDK_OK;
}

rdk_status_t rdk_philox_words(uint64_t seed, uint64_t offset, int32_t count, uint32_t *words, void *stream)
{
    if (!words) return RDK_ERR_NULL;
    if (count < 1) return RDK_ERR_SHAPE;
    return launch_philox_words(seed, offset, count, words, (hipStream_t)stream);
}

}  // extern "C"
