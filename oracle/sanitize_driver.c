/*
 * TEST INFRASTRUCTURE ONLY.  A driver that takes every function of the CPU oracle (rdk_oracle.c) through one
 * small, exactly sized problem each, so that a build with -fsanitize=address,undefined reports any access
 * outside an array, use of an uninitialised allocation size, signed overflow or misaligned access in the
 * oracle itself.  All buffers are heap allocations of exactly the documented sizes.  Exit status 0 = every
 * call returned and the results passed a coarse sanity check (the numerical pins live in the Python tests).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int orc_softmax(const double *z, int64_t n, double *out);
int orc_tli(const double *q_hat, int64_t n, double *q_tli);
void orc_redistribute_dense(const double *q_tli, const double *M, int64_t n, int64_t N, double *p_prime);
void orc_redistribute_sparse(const double *q_tli, int64_t n, int64_t N, int64_t k, const int32_t *kept_ids,
                             const int32_t *nbr_idx, const double *nbr_w, const double *self_w, double *p_prime);
int orc_taylor(const double *p, const double *q_tli, const int32_t *kept_ids, int64_t n, int64_t N, double *p_taylor,
               double *theta_out, double *S_out);
void orc_overlap(const double *p, const double *q, int64_t N, double *alpha, double *resid_mass);
double orc_kernel_l1(const double *p, const double *q, int64_t N);
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void orc_uniforms(uint64_t seed, uint64_t index, double u[4]);
int64_t orc_sample_cdf(const double *w, int64_t N, double u);
int orc_accept(double u1, double q_d, double p_d);
int64_t orc_sample_residual(const double *p, const double *q, int64_t N, double u);
void orc_sequence_scan(const uint8_t *accept, const int32_t *draft_ids, const int32_t *resid_ids, int64_t S, int64_t gamma,
                       int32_t *n_accepted, int32_t *out_tokens);
void orc_features_from_scores(const double *z, int64_t T, int64_t N, double *F);
int orc_build_dense(const double *E, int64_t N, int64_t d, const int32_t *kept_ids, int64_t n, double tau, double *M);
int orc_build_sparse(const double *E, int64_t N, int64_t d, const int32_t *kept_ids, int64_t n, double tau, int64_t k,
                     int32_t *nbr_idx, double *nbr_w, double *self_w, double *nbr_omega);
void orc_densify_sparse(int64_t n, int64_t N, int64_t k, const int32_t *kept_ids, const int32_t *nbr_idx,
                        const double *nbr_w, const double *self_w, double *M);
void orc_verify_position(const double *p, const double *q_prime, int64_t N, uint64_t seed, uint64_t index, int sample_draft,
                         int32_t *draft_id, uint8_t *accept, double *alpha, double *resid_mass, int32_t *resid_id);
int orc_verify_multi(const double *p, const double *q_prime, int64_t N, int64_t C, uint64_t seed, uint64_t index,
                     int sample_candidates, int32_t *cand_ids, int32_t *accepted, int32_t *token, double *resid_mass);
void orc_tree_walk(const int32_t *child_node, const int32_t *accepted, const int32_t *token, int64_t S, int64_t nodes,
                   int64_t C, int32_t *n_accepted, int32_t *out_tokens);

static uint64_t lcg_state = 0x2506032060ULL;
static double unit(void)   /* a plain linear congruential draw in (0, 1) */
{
    lcg_state = lcg_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return ((double)(lcg_state >> 11) + 0.5) / 9007199254740992.0;
}

#define NEW(type, count) ((type *)malloc((size_t)(count) * sizeof(type)))
#define CHECK(cond)                                                      \
    do {                                                                 \
        if (!(cond)) {                                                   \
            fprintf(stderr, "sanitize_driver: check failed: %s (line %d)\n", #cond, __LINE__); \
            return 1;                                                    \
        }                                                                \
    } while (0)

static double sum_of(const double *v, int64_t len)
{
    double s = 0.0;
    for (int64_t i = 0; i < len; ++i) s += v[i];
    return s;
}

int main(void)
{
    enum { N = 97, n = 23, k = 4, d = 8, T = 11, C = 3 };
    /* kept ids: every fourth id and a few more, ascending */
    int32_t *kept = NEW(int32_t, n);
    for (int s = 0; s < n; ++s) kept[s] = 4 * s + (s % 3 == 0 ? 1 : 0);
    double *E = NEW(double, N * d);
    for (int i = 0; i < N * d; ++i) E[i] = unit() - 0.5;

    /* softmax, TLI */
    double *z = NEW(double, N), *p = NEW(double, N), *qz = NEW(double, n), *q_hat = NEW(double, n), *q_tli = NEW(double, n);
    for (int j = 0; j < N; ++j) z[j] = 6.0 * unit();
    for (int s = 0; s < n; ++s) qz[s] = 6.0 * unit();
    CHECK(orc_softmax(z, N, p) == 0 && fabs(sum_of(p, N) - 1.0) < 1e-12);
    CHECK(orc_softmax(qz, n, q_hat) == 0);
    CHECK(orc_softmax(z, 0, p) != 0);
    for (int s = 0; s < n; ++s) q_hat[s] *= 0.37;
    CHECK(orc_tli(q_hat, n, q_tli) == 0 && fabs(sum_of(q_tli, n) - 1.0) < 1e-12);

    /* kernel construction: dense, sparse, densified sparse */
    double *M = NEW(double, n * N), *Ms = NEW(double, n * N);
    CHECK(orc_build_dense(E, N, d, kept, n, 0.3, M) == 0);
    for (int s = 0; s < n; ++s) CHECK(fabs(sum_of(M + s * N, N) - 1.0) < 1e-12);
    int32_t *nbr_idx = NEW(int32_t, (N - n) * k);
    double *nbr_w = NEW(double, (N - n) * k), *self_w = NEW(double, n), *omega = NEW(double, (N - n) * (k + 1));
    CHECK(orc_build_sparse(E, N, d, kept, n, 0.3, k, nbr_idx, nbr_w, self_w, omega) == 0);
    CHECK(orc_build_sparse(E, N, d, kept, n, 0.3, k, nbr_idx, nbr_w, self_w, NULL) == 0);
    orc_densify_sparse(n, N, k, kept, nbr_idx, nbr_w, self_w, Ms);
    for (int s = 0; s < n; ++s) CHECK(fabs(sum_of(Ms + s * N, N) - 1.0) < 1e-12);

    /* the three redistributions */
    double *pd = NEW(double, N), *ps = NEW(double, N), *pt = NEW(double, N), *pds = NEW(double, N);
    orc_redistribute_dense(q_tli, M, n, N, pd);
    orc_redistribute_sparse(q_tli, n, N, k, kept, nbr_idx, nbr_w, self_w, ps);
    orc_redistribute_dense(q_tli, Ms, n, N, pds);
    CHECK(fabs(sum_of(pd, N) - 1.0) < 1e-12 && fabs(sum_of(ps, N) - 1.0) < 1e-12);
    for (int j = 0; j < N; ++j) CHECK(fabs(ps[j] - pds[j]) < 1e-14);
    double theta, S;
    CHECK(orc_taylor(p, q_tli, kept, n, N, pt, &theta, &S) == 0 && fabs(sum_of(pt, N) - 1.0) < 1e-12);

    /* overlap, sampling, verification */
    double alpha, rmass;
    orc_overlap(p, ps, N, &alpha, &rmass);
    CHECK(alpha > 0.0 && alpha <= 1.0 + 1e-12 && fabs(alpha + rmass - 1.0) < 1e-12);
    CHECK(fabs(orc_kernel_l1(p, ps, N) - (1.0 - alpha)) < 1e-12);
    uint32_t ctr[4] = {1u, 2u, 3u, 4u}, key[2] = {5u, 6u}, words[4];
    orc_philox4x32_10(ctr, key, words);
    double u[4];
    orc_uniforms(77u, 1ull << 40, u);
    for (int i = 0; i < 4; ++i) CHECK(u[i] >= 0.0 && u[i] < 1.0);
    CHECK(orc_sample_cdf(ps, N, u[0]) >= 0 && orc_sample_cdf(ps, N, 0.0) >= 0 && orc_sample_cdf(ps, N, 0.999999) < N);
    CHECK(orc_accept(0.5, 0.2, 0.3) == 1 && orc_accept(0.9, 0.5, 0.1) == 0);
    CHECK(orc_sample_residual(p, ps, N, u[2]) >= 0 && orc_sample_residual(p, NULL, N, u[3]) >= 0);
    CHECK(orc_sample_residual(p, p, N, 0.5) == -1);
    enum { S_ = 3, G = 4, B = S_ * G };
    int32_t draft[B], resid[B], n_acc[S_], out_tok[S_ * (G + 1)];
    uint8_t acc[B];
    for (int b = 0; b < B; ++b) {
        double a_, r_;
        orc_verify_position(p, b % 2 ? ps : pt, N, 9u, 100u + (uint64_t)b, 1, &draft[b], &acc[b], &a_, &r_, &resid[b]);
        CHECK(draft[b] >= 0 && draft[b] < N);
    }
    int32_t given = 5;
    uint8_t acc1;
    int32_t resid1;
    orc_verify_position(p, ps, N, 9u, 3u, 0, &given, &acc1, &alpha, &rmass, &resid1);
    orc_verify_position(p, NULL, N, 9u, 3u, 0, &given, &acc1, &alpha, &rmass, &resid1);   /* the draw t ~ p */
    orc_sequence_scan(acc, draft, resid, S_, G, n_acc, out_tok);
    for (int s = 0; s < S_; ++s) CHECK(n_acc[s] >= 0 && n_acc[s] <= G);

    /* several candidates per position, token trees */
    enum { NODES = 4 };
    int32_t cand[NODES * C], accepted[NODES], token[NODES];
    double rm[NODES * C];
    for (int v = 0; v < NODES; ++v)
        CHECK(orc_verify_multi(p, ps, N, C, 9u, 40u + (uint64_t)v, 1, cand + v * C, &accepted[v], &token[v], rm + v * C) == 0);
    int32_t short_list[C] = {7, -1, -1};
    int32_t acc_m, tok_m;
    CHECK(orc_verify_multi(p, ps, N, C, 9u, 50u, 0, short_list, &acc_m, &tok_m, rm) == 0 && tok_m >= 0 && tok_m < N);
    int32_t child[NODES * C] = {1, 2, -1, 3, -1, -1, -1, -1, -1, -1, -1, -1};
    int32_t n_walk[1], walk[NODES];
    orc_tree_walk(child, accepted, token, 1, NODES, C, n_walk, walk);
    CHECK(n_walk[0] >= 0 && n_walk[0] < NODES);

    /* features from sampled scores */
    double *zs = NEW(double, T * N), *F = NEW(double, N * T);
    for (int i = 0; i < T * N; ++i) zs[i] = unit();
    orc_features_from_scores(zs, T, N, F);
    for (int j = 0; j < N; ++j) CHECK(fabs(sum_of(F + j * T, T)) < 1e-12);

    free(kept); free(E); free(z); free(p); free(qz); free(q_hat); free(q_tli); free(M); free(Ms); free(nbr_idx); free(nbr_w);
    free(self_w); free(omega); free(pd); free(ps); free(pt); free(pds); free(zs); free(F);
    printf("sanitize_driver: every oracle function ran clean\n");
    return 0;
}
