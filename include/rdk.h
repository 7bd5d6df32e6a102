/*
 * rdk.h -- C ABI of the MI355X (gfx950) library for Redistributing Drafter Kernels (RDK).
 *
 * The library covers the data-parallel hot path of the method: for a batch of B positions it
 * redistributes a vocabulary-pruned drafter's distribution q (n kept ids) onto the target
 * vocabulary (N ids) through a row-stochastic token-affinity kernel M (Alg. 1 of the paper), and
 * runs the accept / residual / sample step of speculative decoding against the target
 * distribution p (Alg. 4, steps 2 and 4-10).
 *
 * Conventions, valid for every entry point unless stated otherwise
 *  - Every data pointer is a DEVICE pointer owned by the caller (any allocator; 16-byte aligned).
 *    The library allocates no device memory: scratch comes in through `workspace`, whose size is
 *    given by the *_bytes queries.  Descriptor structs and out-parameters such as `size_t*` and
 *    `rdk_kernel_t**` are HOST pointers.
 *  - Work is enqueued on the HIP stream passed as `stream` (a hipStream_t cast to void*; NULL is the
 *    default stream).  Calls do not synchronise, except rdk_build_kernel with `validate != 0`.
 *    The redistribution, verification and sampling calls consist of kernel launches on that stream
 *    only (no copy, no memset, no allocation), so they may be recorded into a HIP graph and replayed;
 *    the seed and the counter offset are then those given at capture time.
 *  - Calls that use distinct workspaces may run concurrently on distinct streams; two calls that
 *    share a workspace must be ordered by the caller.
 *  - Matrices are row-major with a leading dimension given in ELEMENTS (ld >= row length).
 *  - Position b of a batch draws its random numbers from the counter-based generator
 *    Philox4x32-10 with key = seed and counter = (offset + b, 0): four words per position, mapped
 *    to [0,1) as (word >> 8) * 2^-24; word 0 picks the draft token, word 1 decides acceptance,
 *    word 2 picks the residual token, word 3 the bonus token.
 *  - Every function returns an rdk_status_t; nothing is written to outputs on error.
 */
#ifndef RDK_H
#define RDK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RDK_OK = 0,
    RDK_ERR_NULL = 1,           /* a required pointer is NULL */
    RDK_ERR_SHAPE = 2,          /* a size, leading dimension or count is out of range */
    RDK_ERR_DTYPE = 3,          /* unknown input kind / kernel format / mode */
    RDK_ERR_KEPT_IDS = 4,       /* kept ids not strictly ascending or outside [0, N) (validate only) */
    RDK_ERR_NOT_STOCHASTIC = 5, /* a supplied kernel has a negative entry or a row sum off 1 by > 1e-3 (validate only) */
    RDK_ERR_WORKSPACE = 6,      /* workspace or storage smaller than the *_bytes query says */
    RDK_ERR_UNSUPPORTED = 7,    /* combination not offered (e.g. exact redistribution with a sparse kernel) */
    RDK_ERR_HIP = 8,            /* a HIP call failed; see rdk_last_hip_error() */
    RDK_ERR_ALIGN = 9           /* a device pointer is not 16-byte aligned */
} rdk_status_t;

/* How the token-affinity kernel M (n x N, row = kept slot, column = target id) is stored. */
typedef enum {
    RDK_DENSE_F32 = 0,   /* every entry, fp32 */
    RDK_DENSE_BF16 = 1,  /* every entry, rounded to bf16, 16 bits per entry, packed for the matrix cores */
    RDK_SPARSE_TOPK = 2, /* per pruned id its k strongest kept neighbours; per kept id itself only */
    RDK_IDENTITY = 3     /* M = identity on the kept ids: RDK reduces to token-level intersection */
} rdk_kernel_format_t;

/* What a [B, len] input holds. */
typedef enum {
    RDK_PROB_F32 = 0,   /* non-negative fp32 weights (need not be normalised where noted) */
    RDK_LOGIT_F32 = 1,  /* fp32 logits; the softmax is applied on the fly */
    RDK_LOGIT_BF16 = 2  /* bf16 logits (uint16 bit patterns); widened to fp32, then softmax */
} rdk_input_kind_t;

typedef enum {
    RDK_LINEAR_TAYLOR = 0, /* first-order closed form, Eq. 3 of the paper; needs p, no matrix */
    RDK_LINEAR_SPARSE = 1  /* Alg. 1 step 2 with the top-k sparse kernel; O(N k) */
} rdk_linear_mode_t;

typedef struct rdk_kernel rdk_kernel_t; /* opaque host object; points into caller-owned device storage */

/*
 * Inputs of the kernel construction (section 3, "Token-affinity priors", Eq. 2):
 *   M_ij = exp(Omega_ij / tau) / sum_k exp(Omega_ik / tau),  i a kept id, j any target id.
 * Omega is given either through embeddings (Omega_ij = cosine similarity of rows kept_ids[i] and j,
 * the stand-in for the covariance statistics of the paper) or not at all, when the caller brings a
 * finished kernel (dense_M, or the sparse triple).
 *
 * Sparse format (RDK_SPARSE_TOPK): row i keeps the diagonal entry (i, kept_ids[i]) and, for every
 * pruned id j that ranks slot i among its k most similar kept slots (ties: lower slot), the entry
 * (i, j); Eq. 2 is applied over the retained entries, so rows still sum to one.  Its interchange
 * form is keyed by pruned slot u (the u-th id not in kept_ids, ascending):
 *   sparse_idx[u*k + t] = kept slot, sparse_w[u*k + t] = M[slot, id(u)], self_w[i] = M[i, kept_ids[i]].
 */
typedef struct {
    int32_t N;                 /* target vocabulary size |T| */
    int32_t n;                 /* number of kept ids |I|, 1 <= n <= N */
    int32_t d;                 /* embedding width (ignored without embeddings) */
    int32_t k;                 /* neighbours per pruned id, 0 <= k <= min(n, 64); RDK_SPARSE_TOPK only */
    const int32_t *kept_ids;   /* [n] device: the kept target ids, strictly ascending */
    const float *embeddings;   /* [N, d] device, row-major, or NULL */
    const float *dense_M;      /* [n, N] device, row-major, row-stochastic, or NULL (dense formats) */
    const int32_t *sparse_idx; /* [(N-n), k] device or NULL (sparse format) */
    const float *sparse_w;     /* [(N-n), k] device or NULL */
    const float *self_w;       /* [n] device or NULL */
    float tau;                 /* temperature of Eq. 2, > 0 (ignored without embeddings) */
    rdk_kernel_format_t format;
    int32_t validate;          /* != 0: check kept_ids (and a supplied kernel) on the device, then synchronise */
} rdk_kernel_desc_t;

/* Bytes of device storage the finished kernel occupies, and of scratch the build needs. */
rdk_status_t rdk_kernel_storage_bytes(const rdk_kernel_desc_t *desc, size_t *storage_bytes,
                                      size_t *build_workspace_bytes);

/*
 * Token features from data (Sec. 3, "Token-affinity priors": Omega is estimated from data).  z [T, ldz] holds T
 * sampled score rows over the N target ids (target logits, fp32 or bf16, or probabilities); features [N, ldf]
 * receives  F[j, t] = z[t, j] - mean_t z[., j].  Passed as `embeddings` (d = T, row stride T: use ldf = T) to
 * rdk_build_kernel, Omega_ij becomes the correlation of the scores of tokens i and j over the sample, i.e. the
 * covariance matrix of the standardised scores; it is 1 on the diagonal and at most 1 elsewhere, as Eq. 2's
 * evaluation here assumes.  T >= 2; a token whose score never varies has no direction and must not be passed on.
 * No workspace; enqueues on `stream`.
 */
rdk_status_t rdk_features_from_scores(const void *z, rdk_input_kind_t z_kind, int64_t ldz, int32_t T, int32_t N,
                                      float *features, int64_t ldf, void *stream);

/*
 * Build M into `storage` (Eq. 2; a one-off preprocessing step, Sec. 3).  `storage` must stay
 * alive and untouched for the life of the kernel object; `workspace` may be reused once the
 * stream has passed the build.  *out receives the host handle.
 */
rdk_status_t rdk_build_kernel(const rdk_kernel_desc_t *desc, void *storage, size_t storage_bytes,
                              void *workspace, size_t workspace_bytes, void *stream,
                              rdk_kernel_t **out);

/* Frees the host object only; the device storage belongs to the caller. */
rdk_status_t rdk_destroy_kernel(rdk_kernel_t *kernel);

/* Copy a sparse kernel out in the interchange form described above (device buffers). */
rdk_status_t rdk_kernel_get_sparse(const rdk_kernel_t *kernel, int32_t *sparse_idx, float *sparse_w,
                                   float *self_w, void *stream);

/* Copy a dense kernel out as fp32 [n, ldm] (bf16 storage is widened). */
rdk_status_t rdk_kernel_get_dense(const rdk_kernel_t *kernel, float *dense_M, int64_t ldm,
                                  void *stream);

/* Scratch needed by either redistribute call for B positions with this kernel. */
rdk_status_t rdk_workspace_bytes(const rdk_kernel_t *kernel, int32_t B, size_t *bytes);

/*
 * Alg. 1, steps 1-2, exact form:  q_prime[b, :] = M^T TLI(q[b, :]).
 *   q        [B, ldq]  drafter weights or logits over the n kept slots (slot s <-> id kept_ids[s]).
 *            PROB: any non-negative row; step 1 (Eq. 1) divides by its sum.  A row whose sum is zero has no
 *            image under Eq. 1: every redistribution call (exact, both linear forms, the fused call and the
 *            draft draw) returns the zero row for it, so that verification sees alpha = 0, resid_mass = sum(p),
 *            draft_ids = -1, accept = 0, and draws resid_ids from the target row alone.
 *            LOGIT: the softmax over the n slots, which equals Eq. 1 applied to a full softmax.
 *   q_prime  [B, ldo]  fp32, the redistributed drafter over all N target ids.
 * Kernel format must be DENSE_F32, DENSE_BF16 or IDENTITY.  With DENSE_BF16 the kernel entries are rounded to
 * bf16 and the normalised drafter rows to eleven significant bits (both are fed to the matrix cores as fp16 numbers
 * scaled by 2^15; values below 2^-29 count as zero), products accumulate in fp32 and each output row is rescaled
 * to sum to one: every output is within 2e-3 (relative, plus 1e-7) of the exact product with the kernel as stored.
 */
rdk_status_t rdk_redistribute_exact(const rdk_kernel_t *kernel, const void *q,
                                    rdk_input_kind_t q_kind, int64_t ldq, int32_t B,
                                    float *q_prime, int64_t ldo, void *workspace,
                                    size_t workspace_bytes, void *stream);

/*
 * Alg. 1, steps 1-2, linear-time forms.
 *   RDK_LINEAR_TAYLOR (Eq. 3): theta = p^T q', pt_j = (N q'_j + theta p_j) / (N + p_j),
 *     q_prime = pt / sum(pt), with q' = TLI(q) scattered to the kept ids.  Needs p [B, ldp]
 *     (PROB rows must sum to one); uses only kept_ids of the kernel (any format).
 *   RDK_LINEAR_SPARSE: q_prime = M^T q' with the top-k sparse kernel (format RDK_SPARSE_TOPK or
 *     RDK_IDENTITY); p is ignored and may be NULL.
 */
rdk_status_t rdk_redistribute_linear(const rdk_kernel_t *kernel, rdk_linear_mode_t mode,
                                     const void *p, rdk_input_kind_t p_kind, int64_t ldp,
                                     const void *q, rdk_input_kind_t q_kind, int64_t ldq,
                                     int32_t B, float *q_prime, int64_t ldo, void *workspace,
                                     size_t workspace_bytes, void *stream);

/* Verification of a batch (Alg. 4, steps 2 and 4-10). */
typedef struct {
    int32_t B;            /* positions */
    int32_t N;            /* target vocabulary size */
    int32_t gamma;        /* draft tokens per sequence; 0 = no per-sequence scan; else B % gamma == 0 */
    int32_t sample_draft; /* != 0: draw d ~ q_prime into draft_ids; 0: draft_ids holds the caller's tokens */
    uint64_t seed;        /* Philox key */
    uint64_t offset;      /* Philox counter of position 0 */
} rdk_verify_desc_t;

rdk_status_t rdk_verify_workspace_bytes(const rdk_verify_desc_t *desc, size_t *bytes);

/*
 * Per position b, with q' = q_prime[b, :] and p = the target row:
 *   alpha[b]      = sum_j min(p_j, q'_j)                                  (Def. 2.1)
 *   resid_mass[b] = sum_j max(0, p_j - q'_j)                              (denominator of Alg. 4 step 8)
 *   draft_ids[b]  = smallest j with prefix_j(q') > u0 * sum(q')           (step 2; only if sample_draft)
 *   accept[b]     = 1 iff u1 * q'_d < p_d, d = draft_ids[b]               (step 6; d outside [0,N) -> 0)
 *   resid_ids[b]  = smallest j with prefix_j(max(0, p - q')) > u2 * resid_mass, or -1 if resid_mass = 0
 * and per sequence s of gamma consecutive positions (steps 4-10), when gamma > 0:
 *   n_accepted[s] = length of the accepted prefix,
 *   out_tokens[s, 0..gamma] = accepted drafts, then the residual token of the first rejected position,
 *                             then -1 (no bonus token is drawn here: that needs one more target row).
 * q_prime == NULL draws only the bonus token t ~ p (step 8, else-branch) into resid_ids with u3;
 * then alpha = 0, accept = 0, resid_mass = sum(p), draft_ids is untouched, gamma must be 0.
 * p: PROB_F32 rows are used as given; LOGIT kinds go through the softmax.  Any of alpha,
 * resid_mass, n_accepted, out_tokens may be NULL.  Sums run in fp32 per 1024-id block and in
 * fp64 across blocks; token ids can differ from an exact evaluation only where the threshold lies
 * within rounding (about 1e-6 of the total) of a prefix-sum step.
 */
rdk_status_t rdk_verify_sample(const rdk_verify_desc_t *desc, const void *p, rdk_input_kind_t p_kind,
                               int64_t ldp, const float *q_prime, int64_t ldq, int32_t *draft_ids,
                               uint8_t *accept, float *alpha, float *resid_mass, int32_t *resid_ids,
                               int32_t *n_accepted, int32_t *out_tokens, void *workspace,
                               size_t workspace_bytes, void *stream);

/*
 * rdk_verify_sample for callers that can neither allocate device memory nor hand in a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation): same arguments without the workspace, same
 * kernels, same outputs bit for bit.  The scratch (the per-block sums, and the softmax statistics of logit rows) lives
 * in a device array inside the library, 4 MiB per GPU, held until the process ends; the call allocates and frees
 * nothing.  A batch whose scratch need (rdk_verify_workspace_bytes minus its 256 bytes of slack, about
 * 12 * B * ceil(N / 1024) bytes) exceeds 4 MiB is refused with RDK_ERR_WORKSPACE and nothing is launched.  All calls
 * on one GPU share the one array: calls that overlap on one GPU (different streams, or different threads) race and
 * must be ordered by the caller; nothing in it needs clearing between calls.  Runs on the current device.
 */
rdk_status_t rdk_verify_sample_static(const rdk_verify_desc_t *desc, const void *p, rdk_input_kind_t p_kind,
                                      int64_t ldp, const float *q_prime, int64_t ldq, int32_t *draft_ids,
                                      uint8_t *accept, float *alpha, float *resid_mass, int32_t *resid_ids,
                                      int32_t *n_accepted, int32_t *out_tokens, void *stream);

/*
 * Alg. 1 steps 1-2 and Alg. 4 steps 2, 4-10 in one call: the outputs of rdk_redistribute_linear(mode)
 * followed by rdk_verify_sample on its result, without the round trip of q' through HBM.  The
 * redistributed rows are produced tile by tile, summed against p on the spot, and re-computed for the
 * two blocks in which the sampled ids fall.  q_prime may be NULL (then it is never written); otherwise
 * it receives the same rows rdk_redistribute_linear writes.  Block sums run over 64 ids (sparse) or
 * 1024 ids (Eq. 3), so fp32 rounding, and with it an id that sits on a prefix-sum step, can differ
 * from the two-call path within the tolerance stated at rdk_verify_sample.  desc->N must equal the
 * kernel's N; draft_ids is required (in/out as in rdk_verify_sample).  RDK_LINEAR_SPARSE needs a
 * RDK_SPARSE_TOPK kernel (k = 0 included: token-level intersection).
 */
rdk_status_t rdk_redistribute_verify_workspace_bytes(const rdk_kernel_t *kernel, rdk_linear_mode_t mode,
                                                     const rdk_verify_desc_t *desc, size_t *bytes);
rdk_status_t rdk_redistribute_verify(const rdk_kernel_t *kernel, rdk_linear_mode_t mode,
                                     const rdk_verify_desc_t *desc, const void *p, rdk_input_kind_t p_kind,
                                     int64_t ldp, const void *q, rdk_input_kind_t q_kind, int64_t ldq,
                                     float *q_prime, int64_t ldo, int32_t *draft_ids, uint8_t *accept,
                                     float *alpha, float *resid_mass, int32_t *resid_ids, int32_t *n_accepted,
                                     int32_t *out_tokens, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Alg. 4 step 2 on the drafter's side, before any target row exists: the draft token of every position is drawn
 * from the redistributed row q' = M^T TLI(q), out-of-vocabulary ids included (the use Sec. 1 and Sec. 3 name:
 * sampling tokens the drafter's vocabulary does not hold):
 *   draft_ids[b] = smallest j with prefix_j(q'_b) > u0 * sum_j q'_b(j),  u0 = word 0 of Philox(seed, offset + b)
 * -- the draw rdk_verify_sample and rdk_redistribute_verify make when sample_draft = 1, so verifying later with
 * sample_draft = 0 and these ids gives what the fused call gives.  q_draft (optional, [B]) receives q'_b(draft_ids[b]).
 *   RDK_SPARSE_TOPK kernel: q' is summed per 64-id block as it is produced and only the block of the
 *     crossing is re-computed; q_prime (optional, [B, ldo]) receives the rows if given.
 *   any other kernel (identity, dense fp32 / bf16): the rows are produced by the matching redistribution
 *     into q_prime, which is then required, and drawn from there.
 * draft_ids[b] = -1 (and q_draft[b] = 0) for a row without mass.  Workspace: rdk_sample_draft_workspace_bytes.
 * Errors as rdk_redistribute_linear.
 */
rdk_status_t rdk_sample_draft_workspace_bytes(const rdk_kernel_t *kernel, int32_t B, size_t *bytes);
rdk_status_t rdk_sample_draft(const rdk_kernel_t *kernel, const void *q, rdk_input_kind_t q_kind, int64_t ldq, int32_t B,
                              uint64_t seed, uint64_t offset, int32_t *draft_ids, float *q_draft, float *q_prime,
                              int64_t ldo, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Verification of several candidates per position.  The paper's introduction (Sec. 1) names multi-candidate / tree
 * verification among the related work; the steps are those of the method cited there (multi-step speculative
 * sampling) with the redistributed drafter q' in the drafter's place, per position b:
 *   r <- p_b;  for i = 0 .. C-1:  candidate x_i;  keep x_i when  u * q'_b(x_i) < r(x_i)  and stop;
 *              otherwise  r <- max(0, r - q'_b) / sum_j max(0, r(j) - q'_b(j));
 *   no candidate kept:  t drawn from r by the inverse CDF (smallest j whose prefix exceeds u * total).
 * With C = 1 this is rdk_verify_sample for one position (same draft, same decision, same residual token).  The
 * emitted token follows p_b exactly whatever q'_b is.
 *   sample_candidates = 1: the C candidates are drawn from q'_b by the inverse CDF and written to cand_ids;
 *   sample_candidates = 0: cand_ids [B, C] is input; an id >= N is a candidate that is never kept, a negative id
 *     ends the list of the position (fewer than C candidates; none at all: the token is drawn from p_b).
 * Uniforms: the m-th uniform of position b is word m % 4 of Philox4x32-10 with key = seed and counter
 * (offset + b as two words, m / 4, 0);  m = i for the draw of candidate i, C + i for its test, 2C for the final draw.
 * Outputs (device): accepted [B] = index of the kept candidate, or C; token [B] = the emitted id (-1 when the last
 * residual is empty); resid_mass [B, C] (optional) = sum_j max(0, r(j) - q'_b(j)) after each rejection, 0 for rounds
 * that were not reached.  p [B, ldp] of kind p_kind, q_prime [B, ldq] fp32; 1 <= C <= 16, N <= 2 097 152.
 * Errors: RDK_ERR_NULL, RDK_ERR_SHAPE (B, N, C, strides), RDK_ERR_DTYPE, RDK_ERR_ALIGN (rows not 16-byte aligned),
 * RDK_ERR_UNSUPPORTED (N or C above the limits), RDK_ERR_WORKSPACE, RDK_ERR_HIP.
 */
typedef struct {
    int32_t B, N, C;            /* positions, target ids, candidates per position */
    uint64_t seed, offset;      /* Philox key and counter base */
    int sample_candidates;      /* 1: draw the candidates from q_prime; 0: cand_ids is input */
} rdk_multi_desc_t;
rdk_status_t rdk_verify_multi_workspace_bytes(const rdk_multi_desc_t *desc, rdk_input_kind_t p_kind, size_t *bytes);
rdk_status_t rdk_verify_multi(const rdk_multi_desc_t *desc, const void *p, rdk_input_kind_t p_kind, int64_t ldp,
                              const float *q_prime, int64_t ldq, int32_t *cand_ids, int32_t *accepted, int32_t *token,
                              float *resid_mass, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Verification of token trees (the other variant Sec. 1 names among the related work), in two calls: rdk_verify_multi
 * on every node with the tokens of its children as the node's candidates (position s * nodes + v = node v of tree s,
 * node 0 the root; p and q' of a node are the target and the redistributed drafter distribution after the prefix that
 * ends at the node), then this walk: from the root, emit token[.] of the node; if its verification kept candidate i
 * (accepted[.] = i < C) go on to child_node[., i], else stop -- the token was the residual draw, or the draw from p at
 * a leaf.  A chain of nodes is Alg. 4 steps 4-10 on one sequence.
 *   child_node [S, nodes, C] (device): node index of the child behind candidate slot i (> the node's own index).
 *   accepted, token [S * nodes] (device): outputs of rdk_verify_multi.
 *   n_accepted [S]: candidates kept along the path; out_tokens [S, nodes]: the emitted ids, -1 beyond them.
 * Integer work only (bit-exact).  Errors: RDK_ERR_NULL, RDK_ERR_SHAPE, RDK_ERR_HIP.
 */
rdk_status_t rdk_tree_walk(int32_t S, int32_t nodes, int32_t C, const int32_t *child_node, const int32_t *accepted,
                           const int32_t *token, int32_t *n_accepted, int32_t *out_tokens, void *stream);

/* The four Philox words of `count` consecutive positions, [count, 4] uint32 on the device (for
 * checking the random stream against an independent implementation). */
rdk_status_t rdk_philox_words(uint64_t seed, uint64_t offset, int32_t count, uint32_t *words,
                              void *stream);

/*
 * Kernel timing for benchmarks.  After rdk_timing_select(name) every launch of the library kernel
 * of that name ("*" = every kernel of the redistribute / verify calls, NULL or "" = none) is
 * bracketed by two HIP events on the launch stream; "name/8" brackets every eighth launch only
 * (an event pair costs the host and the stream several microseconds, which a short step would
 * otherwise show).  rdk_timing_read(name, ...) waits for the
 * recorded events of that kernel, returns how many launches were recorded and their summed
 * elapsed time in milliseconds, and forgets them.  Both take HOST strings.  Names:
 * row_stats_kernel, row_block_sums_kernel, verify_stream_kernel, verify_finalize_kernel, draft_finalize_kernel,
 * sequence_scan_kernel, taylor_stats_kernel, taylor_write_kernel, taylor_row_kernel, tli_scatter_kernel, tree_walk_kernel, verify_multi_kernel,
 * q_transpose_kernel, sparse_product_kernel, prep_a_split_kernel, exact_f32_split_kernel,
 * exact_reduce_kernel, prep_a_bf16_kernel, exact_bf16_kernel.
 */
rdk_status_t rdk_timing_select(const char *kernel_name);
rdk_status_t rdk_timing_read(const char *kernel_name, int64_t *launches, double *total_ms);

const char *rdk_status_string(rdk_status_t status);

/* Text of the last HIP error seen by the calling thread ("" if none). */
const char *rdk_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RDK_H */
