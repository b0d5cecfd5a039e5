/*
 * Runs the CPU reference (oracle/goodroute_oracle.c) on a fleet read from a file, so that the
 * reference can be exercised under AddressSanitizer and UndefinedBehaviorSanitizer
 * (tests/test_oracle_sanitized.py builds both files with -fsanitize=address,undefined, runs this
 * program and compares what it writes with the ordinary build's results, bit for bit).
 * Test infrastructure only.
 *
 * Input file: int64 header {n_inst, n_class, n_act, n_q, n_req, n_hits, has_cap, has_exclude},
 * then the arrays in the order read below.  Output file: the arrays in the order written below.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct gro_fleet gro_fleet;
gro_fleet *gro_simulate(int32_t, int32_t, const double *, const double *, const double *, const double *,
                        const int32_t *, const int32_t *, const int32_t *, const int32_t *, const int32_t *,
                        const int32_t *, const int32_t *, const int32_t *, const int32_t *, double *, double *);
void gro_free(gro_fleet *);
void gro_status(const gro_fleet *, double *, double *, int32_t *);
void gro_step_table(const gro_fleet *, int32_t, double *);
void gro_pair_T(const gro_fleet *, int64_t, const int32_t *, const int32_t *, const int32_t *, const int32_t *,
                const int32_t *, double *);
void gro_route(const gro_fleet *, int64_t, const int32_t *, const int32_t *, const double *, const int32_t *,
               const int32_t *, const int32_t *, const int32_t *, int32_t *, double *, uint8_t *, double *);
void gro_band(const gro_fleet *, int64_t, const int32_t *, const int32_t *, const double *, const int32_t *,
              const int32_t *, const int32_t *, const int32_t *, const int32_t *, double, const int32_t *,
              int32_t *, int32_t *, double *, int32_t *, int32_t *, double *);

static void *take(FILE *f, size_t n, size_t elem)
{
    void *p = malloc(n * elem ? n * elem : 1);      /* exact sizes: an overrun by one element is seen */
    if (!p || fread(p, elem, n, f) != n) { fprintf(stderr, "short input\n"); exit(2); }
    return p;
}

static void put(FILE *f, const void *p, size_t n, size_t elem)
{
    if (fwrite(p, elem, n, f) != n) { fprintf(stderr, "short output\n"); exit(2); }
}

int main(int argc, char **argv)
{
    if (argc != 3) { fprintf(stderr, "usage: %s input output\n", argv[0]); return 2; }
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) { fprintf(stderr, "cannot open files\n"); return 2; }
    int64_t h[8];
    if (fread(h, sizeof(int64_t), 8, in) != 8) return 2;
    const int64_t M = h[0], C = h[1], na = h[2], nq = h[3], R = h[4], nh = h[5];
    double *delta = take(in, C, 8), *alpha = take(in, C, 8), *beta = take(in, C, 8), *gamma = take(in, C, 8);
    int32_t *inst_class = take(in, M, 4);
    int32_t *act_off = take(in, M + 1, 4), *act_prompt = take(in, na, 4), *act_gen = take(in, na, 4),
            *act_rem = take(in, na, 4);
    int32_t *q_off = take(in, M + 1, 4), *q_prompt = take(in, nq, 4), *q_len = take(in, nq, 4);
    int32_t *cap = h[6] ? take(in, M, 4) : NULL;
    int32_t *c0 = take(in, R, 4), *len = take(in, R, 4);
    double *deadline = take(in, R, 8);
    int32_t *exclude = h[7] ? take(in, R, 4) : NULL;
    int32_t *hit_off = nh >= 0 ? take(in, R + 1, 4) : NULL;
    int32_t *hit_inst = nh >= 0 ? take(in, nh, 4) : NULL, *hit_len = nh >= 0 ? take(in, nh, 4) : NULL;
    int32_t *rank = take(in, M, 4), *picked = take(in, R, 4);

    double *a_fin = malloc((na ? na : 1) * 8), *q_fin = malloc((nq ? nq : 1) * 8);
    gro_fleet *f = gro_simulate((int32_t)M, (int32_t)C, delta, alpha, beta, gamma, inst_class, act_off, act_prompt,
                                act_gen, act_rem, q_off, q_prompt, q_len, cap, a_fin, q_fin);
    if (!f) { fprintf(stderr, "gro_simulate failed\n"); return 2; }
    double *q = malloc(M * 8), *d = malloc(M * 8);
    int32_t *smax = malloc(M * 4);
    gro_status(f, q, d, smax);
    put(out, a_fin, na, 8); put(out, q_fin, nq, 8); put(out, q, M, 8); put(out, d, M, 8); put(out, smax, M, 4);
    for (int64_t g = 0; g < M; ++g) {
        double *w = malloc(((size_t)smax[g] + 1) * 8);
        gro_step_table(f, (int32_t)g, w);
        put(out, w, (size_t)smax[g] + 1, 8);
        free(w);
    }
    double *T = malloc((R * M ? R * M : 1) * 8);
    gro_pair_T(f, R, c0, len, hit_off, hit_inst, hit_len, T);
    put(out, T, R * M, 8);
    int32_t *o_inst = malloc((R ? R : 1) * 4);
    double *o_slack = malloc((R ? R : 1) * 8), *o_T = malloc((R ? R : 1) * 8);
    uint8_t *o_fb = malloc(R ? R : 1);
    gro_route(f, R, c0, len, deadline, exclude, hit_off, hit_inst, hit_len, o_inst, o_slack, o_fb, o_T);
    put(out, o_inst, R, 4); put(out, o_slack, R, 8); put(out, o_fb, R, 1); put(out, o_T, R, 8);
    int32_t *sure = malloc((R ? R : 1) * 4), *maybe = malloc((R ? R : 1) * 4), *near = malloc((R ? R : 1) * 4),
            *equal = malloc((R ? R : 1) * 4);
    double *tmin = malloc((R ? R : 1) * 8), *pT = malloc((R ? R : 1) * 8);
    gro_band(f, R, c0, len, deadline, exclude, hit_off, hit_inst, hit_len, rank, 1e-4, picked, sure, maybe, tmin,
             near, equal, pT);
    put(out, sure, R, 4); put(out, maybe, R, 4); put(out, tmin, R, 8); put(out, near, R, 4); put(out, equal, R, 4);
    put(out, pT, R, 8);
    gro_free(f);
    free(sure); free(maybe); free(near); free(equal); free(tmin); free(pT);
    free(o_inst); free(o_slack); free(o_T); free(o_fb); free(T); free(q); free(d); free(smax); free(a_fin); free(q_fin);
    free(delta); free(alpha); free(beta); free(gamma); free(inst_class); free(act_off); free(act_prompt);
    free(act_gen); free(act_rem); free(q_off); free(q_prompt); free(q_len); free(cap); free(c0); free(len);
    free(deadline); free(exclude); free(hit_off); free(hit_inst); free(hit_len); free(rank); free(picked);
    fclose(in);
    if (fclose(out) != 0) return 2;
    return 0;
}
