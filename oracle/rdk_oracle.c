/*
 * rdk_oracle.c -- reference ("oracle") implementation of Redistributing Drafter
 * Kernels (RDK) and of the speculative-decoding verification that follows it.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, sequential fp64 program
 * whose only job is to be checkable against the paper by eye.  It shares no code,
 * header, table or constant with the GPU library, and nothing in the product path
 * may link or call it.  Only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg use it.
 *
 * Every loop runs in index order, every sum is a left-to-right fp64 sum, there is
 * no blocking, fusion or threading.  Inputs are the caller's fp32/bf16 values
 * widened exactly to fp64 before they get here.
 *
 * Pins (see tests/test_oracle_*.py): the m=2 worked example of Thm 4.3; the
 * identities of Lemma 2.3; Thm 4.1, Thm 4.2, Lemma B.1 inequalities; identity
 * kernel == TLI; library softmax / matmul on the same data; closed forms of
 * Eq. 3; Monte-Carlo acceptance and losslessness of Alg. 4; published
 * known-answer vectors of Philox4x32-10; verification of several candidates:
 * its reduction to Alg. 4 with one candidate, a hand-computed example, and the
 * law of the emitted token (equal to p), also for lists of any length; the
 * walk through verified token trees: a chain is Alg. 4 on a sequence, and a
 * hand-made tree.
 * Parity unpinned: none of the functions below is without a pin; the size of the
 * exact-vs-first-order gap (Thm 4.4) is only reported, since the theorem's
 * constants are not given.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Softmax, as defined below Eq. 4:  p_i = exp(z_i) / sum_j exp(z_j).         */
/* The maximum is subtracted first; this does not change the value.          */
/* Returns 0, or -1 when n <= 0.                                             */
int orc_softmax(const double *z, int64_t n, double *out)
{
    if (n <= 0) return -1;
    double m = z[0];
    for (int64_t i = 1; i < n; ++i)
        if (z[i] > m) m = z[i];
    double sum = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        out[i] = exp(z[i] - m);
        sum += out[i];
    }
    for (int64_t i = 0; i < n; ++i) out[i] /= sum;
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Token-level intersection, Eq. 1 / Alg. 2 step 1, in the pruning case       */
/* D subset of T: the drafter only has mass on the n kept ids, so q0 is the   */
/* drafter vector divided by its own sum.  q_hat and q_tli are indexed by     */
/* kept slot.  Returns -1 when the sum is not positive (Eq. 1 undefined).     */
int orc_tli(const double *q_hat, int64_t n, double *q_tli)
{
    double Z = 0.0;
    for (int64_t s = 0; s < n; ++s) Z += q_hat[s];
    if (!(Z > 0.0)) return -1;
    for (int64_t s = 0; s < n; ++s) q_tli[s] = q_hat[s] / Z;
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Alg. 1 step 2 with an explicit kernel:  p' = M^T q'.                       */
/* M is n x N row-major (row = kept slot, column = target id); only rows of   */
/* kept ids are ever used because q' vanishes elsewhere.                      */
void orc_redistribute_dense(const double *q_tli, const double *M, int64_t n, int64_t N,
                            double *p_prime)
{
    for (int64_t j = 0; j < N; ++j) {
        double acc = 0.0;
        for (int64_t s = 0; s < n; ++s) acc += q_tli[s] * M[s * N + j];
        p_prime[j] = acc;
    }
}

/* ------------------------------------------------------------------------- */
/* The same product for a kernel that keeps, per pruned target id, only its   */
/* k strongest kept neighbours, and per kept id only itself.                  */
/*   kept id  (slot s):   p'_j = self_w[s] * q'_s                             */
/*   pruned id (slot u):  p'_j = sum_t nbr_w[u,t] * q'_{nbr_idx[u,t]}         */
/* Pruned slots number the ids outside kept_ids in ascending id order.        */
void orc_redistribute_sparse(const double *q_tli, int64_t n, int64_t N, int64_t k,
                             const int32_t *kept_ids, const int32_t *nbr_idx,
                             const double *nbr_w, const double *self_w, double *p_prime)
{
    int64_t s = 0, u = 0;
    for (int64_t j = 0; j < N; ++j) {
        if (s < n && kept_ids[s] == j) {
            p_prime[j] = self_w[s] * q_tli[s];
            ++s;
        } else {
            double acc = 0.0;
            for (int64_t t = 0; t < k; ++t) acc += nbr_w[u * k + t] * q_tli[nbr_idx[u * k + t]];
            p_prime[j] = acc;
            ++u;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* First-order form, Eq. 3:                                                   */
/*   theta = p^T q',   p~_i = (N q'_i + theta p_i) / (N + p_i),               */
/*   p_Taylor = p~ / sum_j p~_j,   with N = |T| (Thm 4.4).                    */
/* q' is given per kept slot and is zero on every other id.                   */
int orc_taylor(const double *p, const double *q_tli, const int32_t *kept_ids, int64_t n,
               int64_t N, double *p_taylor, double *theta_out, double *S_out)
{
    double *q_full = (double *)calloc((size_t)N, sizeof(double));
    if (!q_full) return -2;
    for (int64_t s = 0; s < n; ++s) q_full[kept_ids[s]] = q_tli[s];
    double theta = 0.0;
    for (int64_t j = 0; j < N; ++j) theta += p[j] * q_full[j];
    double S = 0.0;
    for (int64_t j = 0; j < N; ++j) {
        p_taylor[j] = ((double)N * q_full[j] + theta * p[j]) / ((double)N + p[j]);
        S += p_taylor[j];
    }
    free(q_full);
    if (!(S > 0.0)) return -1;
    for (int64_t j = 0; j < N; ++j) p_taylor[j] /= S;
    if (theta_out) *theta_out = theta;
    if (S_out) *S_out = S;
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Def. 2.1: alpha = sum_x min(p(x), q(x)); and the numerator mass of the     */
/* residual of Alg. 4: R = sum_x (p(x) - min(p(x), q(x))).                    */
void orc_overlap(const double *p, const double *q, int64_t N, double *alpha, double *resid_mass)
{
    double a = 0.0, r = 0.0;
    for (int64_t j = 0; j < N; ++j) {
        double mn = p[j] < q[j] ? p[j] : q[j];
        a += mn;
        r += p[j] - mn;
    }
    *alpha = a;
    *resid_mass = r;
}

/* Def. 2.2: ||k||_1 with k(x) = max(0, q(x) - p(x)). */
double orc_kernel_l1(const double *p, const double *q, int64_t N)
{
    double s = 0.0;
    for (int64_t j = 0; j < N; ++j)
        if (q[j] > p[j]) s += q[j] - p[j];
    return s;
}

/* ------------------------------------------------------------------------- */
/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random    */
/* numbers: as easy as 1, 2, 3", SC'11): a 128-bit counter, a 64-bit key.     */
/* One round maps (c0,c1,c2,c3) to                                           */
/*   (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0));                */
/* the key grows by the two Weyl constants between rounds.                    */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t MUL0 = 0xD2511F53u, MUL1 = 0xCD9E8D57u;
    const uint32_t WEYL0 = 0x9E3779B9u, WEYL1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += WEYL0;
            k1 += WEYL1;
        }
        uint64_t prod0 = MUL0 * (uint64_t)c0;
        uint64_t prod1 = MUL1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(prod1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)prod1;
        uint32_t n2 = (uint32_t)(prod0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)prod0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Four uniforms in [0,1) for one position: key = seed, counter = (index,0,0) */
/* as 64-bit halves; each word keeps its top 24 bits, u = (w >> 8) * 2^-24,   */
/* which is exact in fp32 and fp64 alike.                                     */
/* u[0]: draft token, u[1]: accept test, u[2]: residual token, u[3]: bonus.   */
void orc_uniforms(uint64_t seed, uint64_t index, double u[4])
{
    uint32_t ctr[4] = {(uint32_t)index, (uint32_t)(index >> 32), 0u, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    for (int i = 0; i < 4; ++i) u[i] = (double)(w[i] >> 8) * (1.0 / 16777216.0);
}

/* ------------------------------------------------------------------------- */
/* Inverse-CDF draw from non-negative weights w (Alg. 4 step 2 and step 8):   */
/* the smallest j whose inclusive prefix sum exceeds u times the total.       */
/* Zero-weight ids are never returned.  -1 when the total is not positive.    */
int64_t orc_sample_cdf(const double *w, int64_t N, double u)
{
    double total = 0.0;
    for (int64_t j = 0; j < N; ++j) total += w[j];
    if (!(total > 0.0)) return -1;
    double thr = u * total, c = 0.0;
    int64_t last_positive = -1;
    for (int64_t j = 0; j < N; ++j) {
        c += w[j];
        if (w[j] > 0.0) last_positive = j;
        if (c > thr) return j;
    }
    return last_positive; /* unreachable for u < 1; guards rounding only */
}

/* Alg. 4 step 6: keep the draft d with probability min(1, p(d)/q(d)):        */
/* accept iff u1 * q(d) < p(d), u1 in [0,1).  No division, so q(d)=0 is fine. */
int orc_accept(double u1, double q_d, double p_d) { return (u1 * q_d < p_d) ? 1 : 0; }

/* Alg. 4 step 8: t ~ r with r(t) proportional to p(t) - min(p(t), q(t)).     */
/* q == NULL stands for q = 0, i.e. the draw t ~ p of the no-rejection case.  */
int64_t orc_sample_residual(const double *p, const double *q, int64_t N, double u)
{
    double *r = (double *)malloc((size_t)N * sizeof(double));
    if (!r) return -2;
    for (int64_t j = 0; j < N; ++j) {
        double mn = (q && q[j] < p[j]) ? q[j] : (q ? p[j] : 0.0);
        r[j] = p[j] - mn;
    }
    int64_t t = orc_sample_cdf(r, N, u);
    free(r);
    return t;
}

/* ------------------------------------------------------------------------- */
/* Alg. 4 steps 4-10 for S sequences of gamma draft positions each: count     */
/* the accepted prefix, then emit d_1..d_j followed by the residual token of  */
/* the first rejected position (or -1 when nothing was rejected: the bonus    */
/* draw needs a target row that the caller holds, not this routine).          */
void orc_sequence_scan(const uint8_t *accept, const int32_t *draft_ids, const int32_t *resid_ids,
                       int64_t S, int64_t gamma, int32_t *n_accepted, int32_t *out_tokens)
{
    for (int64_t q = 0; q < S; ++q) {
        int64_t j = 0;
        while (j < gamma && accept[q * gamma + j]) ++j;
        n_accepted[q] = (int32_t)j;
        for (int64_t i = 0; i <= gamma; ++i) out_tokens[q * (gamma + 1) + i] = -1;
        for (int64_t i = 0; i < j; ++i) out_tokens[q * (gamma + 1) + i] = draft_ids[q * gamma + i];
        if (j < gamma) out_tokens[q * (gamma + 1) + j] = resid_ids[q * gamma + j];
    }
}

/* ------------------------------------------------------------------------- */
/* Affinity prior.  Omega_ij is the cosine similarity of embedding rows       */
/* (the stand-in for the covariance of section 3).                            */
static void unit_rows(const double *E, int64_t N, int64_t d, double *U)
{
    for (int64_t j = 0; j < N; ++j) {
        double ss = 0.0;
        for (int64_t c = 0; c < d; ++c) ss += E[j * d + c] * E[j * d + c];
        double nrm = sqrt(ss);
        for (int64_t c = 0; c < d; ++c) U[j * d + c] = E[j * d + c] / nrm;
    }
}

static double dot(const double *a, const double *b, int64_t d)
{
    double s = 0.0;
    for (int64_t c = 0; c < d; ++c) s += a[c] * b[c];
    return s;
}

/* Sec. 3, "Token-affinity priors": Omega is estimated from data.  Token features */
/* from T sampled score rows z[t, :] (target logits or probabilities at T        */
/* positions): F[j, t] = z[t, j] - mean_t z[., j].  With these rows as the        */
/* embeddings of Eq. 2, Omega_ij (the cosine of rows i and j) is the covariance   */
/* of the scores of tokens i and j divided by their standard deviations, i.e.     */
/* the covariance matrix of the standardised scores.                              */
void orc_features_from_scores(const double *z /* [T, N] */, int64_t T, int64_t N, double *F /* [N, T] */)
{
    for (int64_t j = 0; j < N; ++j) {
        double mean = 0.0;
        for (int64_t t = 0; t < T; ++t) mean += z[t * N + j];
        mean /= (double)T;
        for (int64_t t = 0; t < T; ++t) F[j * T + t] = z[t * N + j] - mean;
    }
}

/* Eq. 2: M_ij = exp(Omega_ij / tau) / sum_k exp(Omega_ik / tau), i kept, j in T. */
int orc_build_dense(const double *E, int64_t N, int64_t d, const int32_t *kept_ids, int64_t n,
                    double tau, double *M /* [n, N] */)
{
    double *U = (double *)malloc((size_t)(N * d) * sizeof(double));
    double *row = (double *)malloc((size_t)N * sizeof(double));
    if (!U || !row) { free(U); free(row); return -2; }
    unit_rows(E, N, d, U);
    for (int64_t s = 0; s < n; ++s) {
        for (int64_t j = 0; j < N; ++j) row[j] = dot(U + (int64_t)kept_ids[s] * d, U + j * d, d) / tau;
        orc_softmax(row, N, M + s * N);
    }
    free(U);
    free(row);
    return 0;
}

/* Top-k sparse form of Eq. 2.  Retained entries of row s (kept slot s): the   */
/* diagonal (s, kept_ids[s]) with affinity exactly 1, and (s, j) for every     */
/* pruned id j that ranks s among its k most similar kept slots (ties: lower   */
/* slot first).  Eq. 2 is then applied over the retained entries only, so each */
/* row still sums to 1 (Assumption 3.1).  Output is keyed by pruned slot u:    */
/* nbr_idx[u,t] (kept slot), nbr_w[u,t] = M[nbr_idx[u,t], id(u)], in order of  */
/* falling affinity; self_w[s] = M[s, kept_ids[s]].                            */
int orc_build_sparse(const double *E, int64_t N, int64_t d, const int32_t *kept_ids, int64_t n,
                     double tau, int64_t k, int32_t *nbr_idx, double *nbr_w, double *self_w,
                     double *nbr_omega /* optional [N-n, k+1]: affinities of the k chosen and the best not chosen */)
{
    if (k > n) return -1;
    double *U = (double *)malloc((size_t)(N * d) * sizeof(double));
    double *om = (double *)malloc((size_t)n * sizeof(double));
    uint8_t *taken = (uint8_t *)malloc((size_t)n);
    double *Z = (double *)malloc((size_t)n * sizeof(double));
    if (!U || !om || !taken || !Z) { free(U); free(om); free(taken); free(Z); return -2; }
    unit_rows(E, N, d, U);
    for (int64_t s = 0; s < n; ++s) Z[s] = 1.0; /* exp((1 - 1)/tau): the diagonal */
    int64_t s_next = 0, u = 0;
    for (int64_t j = 0; j < N; ++j) {
        if (s_next < n && kept_ids[s_next] == j) { ++s_next; continue; }
        for (int64_t s = 0; s < n; ++s) om[s] = dot(U + (int64_t)kept_ids[s] * d, U + j * d, d);
        memset(taken, 0, (size_t)n);
        for (int64_t t = 0; t <= k; ++t) { /* selection by repeated maximum; the (k+1)-th is only reported */
            int64_t best = -1;
            for (int64_t s = 0; s < n; ++s)
                if (!taken[s] && (best < 0 || om[s] > om[best])) best = s;
            if (t < k) {
                taken[best] = 1;
                nbr_idx[u * k + t] = (int32_t)best;
                /* unnormalised exp(Omega/tau), scaled by exp(-1/tau) in every row alike */
                nbr_w[u * k + t] = exp((om[best] - 1.0) / tau);
                Z[best] += nbr_w[u * k + t];
                if (nbr_omega) nbr_omega[u * (k + 1) + t] = om[best];
            } else if (nbr_omega) {
                nbr_omega[u * (k + 1) + k] = best >= 0 ? om[best] : -2.0;
            }
        }
        ++u;
    }
    for (int64_t i = 0; i < u * k; ++i) nbr_w[i] /= Z[nbr_idx[i]];
    for (int64_t s = 0; s < n; ++s) self_w[s] = 1.0 / Z[s];
    free(U); free(om); free(taken); free(Z);
    return 0;
}

/* Scatter a sparse kernel into the dense n x N matrix it stands for. */
void orc_densify_sparse(int64_t n, int64_t N, int64_t k, const int32_t *kept_ids,
                        const int32_t *nbr_idx, const double *nbr_w, const double *self_w,
                        double *M /* [n, N], zero-filled here */)
{
    memset(M, 0, (size_t)(n * N) * sizeof(double));
    int64_t s = 0, u = 0;
    for (int64_t j = 0; j < N; ++j) {
        if (s < n && kept_ids[s] == j) {
            M[s * N + j] = self_w[s];
            ++s;
        } else {
            for (int64_t t = 0; t < k; ++t) M[(int64_t)nbr_idx[u * k + t] * N + j] += nbr_w[u * k + t];
            ++u;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Alg. 4 steps 2 and 4-8 for one position, given p and the redistributed     */
/* drafter q' on the full target vocabulary.                                  */
/* sample_draft != 0: d ~ q' with u[0]; else *draft_id is the caller's token. */
/* q_prime == NULL: only the bonus draw t ~ p is made (with u[3]).            */
void orc_verify_position(const double *p, const double *q_prime, int64_t N, uint64_t seed,
                         uint64_t index, int sample_draft, int32_t *draft_id, uint8_t *accept,
                         double *alpha, double *resid_mass, int32_t *resid_id)
{
    double u[4];
    orc_uniforms(seed, index, u);
    if (!q_prime) {
        *alpha = 0.0;
        *resid_mass = 0.0;
        for (int64_t j = 0; j < N; ++j) *resid_mass += p[j];
        *accept = 0;
        *resid_id = (int32_t)orc_sample_residual(p, NULL, N, u[3]);
        return;
    }
    orc_overlap(p, q_prime, N, alpha, resid_mass);
    if (sample_draft) *draft_id = (int32_t)orc_sample_cdf(q_prime, N, u[0]);
    int32_t dtok = *draft_id;
    *accept = (dtok >= 0 && dtok < N) ? (uint8_t)orc_accept(u[1], q_prime[dtok], p[dtok]) : 0;
    *resid_id = (*resid_mass > 0.0) ? (int32_t)orc_sample_residual(p, q_prime, N, u[2]) : -1;
}

/* ------------------------------------------------------------------------- */
/* Verification of SEVERAL candidates for one position.  The paper names      */
/* multi-candidate (tree) verification only among the related work of its     */
/* introduction; the routine follows the publication cited there (Miao et     */
/* al., "SpecInfer", ASPLOS 2024: multi-step speculative sampling) with the   */
/* redistributed drafter q' in the drafter's place.  In that paper's steps:   */
/*   r <- p                                                                    */
/*   for i = 0 .. C-1:  x_i ~ q' (or the caller's);  accept x_i with           */
/*        probability min(1, r(x_i) / q'(x_i));  on acceptance emit x_i, stop; */
/*        otherwise  r <- normalize(max(0, r - q'))                            */
/*   no candidate accepted: emit t ~ r.                                        */
/* With C = 1 this is steps 2 and 6-8 of Alg. 4.  The emitted token follows p  */
/* exactly (the pin of this routine).                                          */
/* Uniforms: the m-th uniform of a position is word m % 4 of the Philox block  */
/* with counter (index, m / 4, 0); m = i for the draw of candidate i, C + i    */
/* for its acceptance test, 2C for the final draw (C = 1: the words of         */
/* orc_uniforms in the order draft, accept, residual).                         */
/* A position may have fewer than C candidates: a negative id ends its list    */
/* (the token is then drawn from the r reached so far; an empty list gives     */
/* t ~ p, the draw at a leaf of a token tree).  An id >= N is a candidate that */
/* is never kept.  The uniforms keep the indices above whatever the length.    */
/* Outputs: cand_ids[C] (written when sampled), *accepted = index of the       */
/* accepted candidate or C, *token = emitted id (-1 when the last residual is  */
/* empty), resid_mass[C] = sum of max(0, r - q') after each rejection (0 for   */
/* rounds that were not reached).  Returns 0, or -2 when memory runs out.      */
static double multi_uniform(uint64_t seed, uint64_t index, int64_t m)
{
    uint32_t ctr[4] = {(uint32_t)index, (uint32_t)(index >> 32), (uint32_t)(m / 4), 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    return (double)(w[m % 4] >> 8) * (1.0 / 16777216.0);
}

int orc_verify_multi(const double *p, const double *q_prime, int64_t N, int64_t C, uint64_t seed,
                     uint64_t index, int sample_candidates, int32_t *cand_ids, int32_t *accepted,
                     int32_t *token, double *resid_mass)
{
    double *r = (double *)malloc((size_t)N * sizeof(double));
    if (!r) return -2;
    for (int64_t j = 0; j < N; ++j) r[j] = p[j];
    for (int64_t i = 0; i < C; ++i) resid_mass[i] = 0.0;
    if (sample_candidates)
        for (int64_t i = 0; i < C; ++i)
            cand_ids[i] = (int32_t)orc_sample_cdf(q_prime, N, multi_uniform(seed, index, i));
    *accepted = (int32_t)C;
    *token = -1;
    for (int64_t i = 0; i < C; ++i) {
        int32_t x = cand_ids[i];
        if (x < 0) break; /* end of this position's list */
        if (x < N && orc_accept(multi_uniform(seed, index, C + i), q_prime[x], r[x])) {
            *accepted = (int32_t)i;
            *token = x;
            free(r);
            return 0;
        }
        double Z = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            r[j] = r[j] > q_prime[j] ? r[j] - q_prime[j] : 0.0;
            Z += r[j];
        }
        resid_mass[i] = Z;
        if (Z > 0.0)
            for (int64_t j = 0; j < N; ++j) r[j] /= Z;
    }
    *token = (int32_t)orc_sample_cdf(r, N, multi_uniform(seed, index, 2 * C));
    free(r);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Walk through verified token trees.  Every tree has `nodes` nodes, node 0   */
/* the root (the context so far); node v of tree s is position s * nodes + v  */
/* of a batch that orc_verify_multi has gone through with the tokens of v's   */
/* children as its candidates, so accepted[.] and token[.] hold, for every    */
/* node, what the verification would emit if the walk came there.             */
/* child_node[(s * nodes + v) * C + i] = node reached by candidate i of v.    */
/* From the root: emit token[v]; if a candidate was kept (accepted < C) go to  */
/* its node, else stop (token[v] was the residual draw, or the draw from p at  */
/* a leaf).  n_accepted[s] = candidates kept on the way; out_tokens[s, 0 ..]   */
/* = the emitted ids, -1 beyond them ([S, nodes]).                             */
void orc_tree_walk(const int32_t *child_node, const int32_t *accepted, const int32_t *token,
                   int64_t S, int64_t nodes, int64_t C, int32_t *n_accepted, int32_t *out_tokens)
{
    for (int64_t s = 0; s < S; ++s) {
        for (int64_t i = 0; i < nodes; ++i) out_tokens[s * nodes + i] = -1;
        int64_t v = 0, len = 0;
        while (len < nodes) {
            int64_t pos = s * nodes + v;
            out_tokens[s * nodes + len] = token[pos];
            ++len;
            if (accepted[pos] >= C) break;
            int32_t next = child_node[pos * C + accepted[pos]];
            if (next <= v || next >= nodes) break; /* not a tree: stop rather than loop */
            v = next;
        }
        /* the last emitted token is the residual / leaf draw unless the walk was cut short */
        n_accepted[s] = (int32_t)(len - 1);
    }
}
