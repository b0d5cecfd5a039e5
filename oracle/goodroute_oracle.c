/*
 * CPU reference for the routing math of GoodServe (predict-and-rectify
 * request routing): TEST INFRASTRUCTURE ONLY.
 *
 * Nothing in the product path links, loads or calls this file; it exists so
 * that the tests, the smoke check and the benchmark's CPU-baseline leg can
 * compare the GPU library against a plain definition.  It shares no code,
 * header, table or constant with the GPU library.
 *
 * What it is: every instance's continuous-batching queue is simulated one
 * decode step at a time in fp64, and every request is scored against every
 * instance by an exhaustive scan.  No sorting, no closed forms, no blocking.
 *
 *   - The end-to-end latency keeps the decomposition of Eq. 2 (Sec. 3.1):
 *     queuing delay + prefill of the uncached prompt + decode time.
 *   - The per-instance status (q_g, p_g, d_g), which Sec. 3.3 estimates
 *     black-box, is here the white-box linear model the synthetic fleets are
 *     defined with: prefill costs delta seconds per prompt token; one decode
 *     step of a batch of B requests whose context lengths sum to C costs
 *     alpha + beta*B + gamma*C seconds.
 *   - Selection is Alg. 1 (Appendix, "Backend Selection Algorithm"): feasible
 *     iff T <= D; among feasible instances the one with the largest d_g;
 *     otherwise the one with the smallest T - D.  Ties go to the lowest
 *     instance index.
 *   - The risk re-check is Sec. 3.4, second half: a request is at risk when
 *     its expected finish exceeds its deadline, and is then re-routed among
 *     the other instances with the same rule; migration moves token IDs, so
 *     the target prefills prompt + generated tokens again.
 *
 * Every function is pinned by tests that do not call it to produce their
 * expectation: a pure-Python re-simulation with the request appended to the
 * instance's queue, hand-worked values, closed forms of special cases and
 * invariants of the model.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct gro_fleet {
    int32_t n_inst, n_class;
    double *delta, *alpha, *beta, *gamma; /* per class */
    int32_t *inst_class;                  /* per instance */
    double *q;                            /* queuing delay of instance g: all queued prefills */
    double *d;                            /* duration of the instance's next decode step */
    int32_t *smax;                        /* number of simulated steps of instance g */
    double **w;                           /* w[g][s], s = 0..smax[g]: time of the first s steps */
} gro_fleet;

void gro_free(gro_fleet *f)
{
    if (!f) return;
    if (f->w) for (int32_t g = 0; g < f->n_inst; ++g) free(f->w[g]);
    free(f->w); free(f->smax); free(f->d); free(f->q); free(f->inst_class);
    free(f->delta); free(f->alpha); free(f->beta); free(f->gamma);
    free(f);
}

static double *dup_d(const double *src, size_t n)
{
    double *p = (double *)malloc(n * sizeof(double));
    if (p) memcpy(p, src, n * sizeof(double));
    return p;
}

/*
 * Simulate one instance (Sec. 3.3's "batched serving mode", made explicit).
 *
 * At most `cap` requests decode together (Sec. 3.1: the number of requests an
 * instance serves concurrently is bounded by its memory).  Queued requests are
 * admitted in queue order whenever the batch has room, at time 0 and after
 * every decode step: an admission prefills the request (prefill has priority
 * and stalls decoding) and puts it into the batch.  With room for everybody
 * (cap larger than the number of requests) all queued requests are prefilled
 * back to back at time 0.  Requests that are already running keep running even
 * if they outnumber the cap.  One step emits one token for every batch member:
 * its remaining length drops by one and its context grows by one; a request
 * whose remaining length reaches zero finishes at the end of that step.
 * Times are measured from now = 0.
 *
 * A request that arrives now is last in the queue: q_out is the time at which
 * it would be admitted (the queue ahead of it is in, and the batch has room),
 * and w_out[s] the time of the s decode steps after that moment (nobody else
 * joins any more).  d_out is the duration of the next decode step that runs.
 */
static int simulate_instance(double delta, double alpha, double beta, double gamma, int32_t cap,
                             int32_t n_act, const int32_t *a_prompt, const int32_t *a_gen,
                             const int32_t *a_rem,
                             int32_t n_q, const int32_t *q_prompt, const int32_t *q_len,
                             double *a_finish, double *q_finish,
                             double *q_out, double *d_out, int32_t *smax_out, double **w_out)
{
    int32_t n = n_act + n_q;
    int32_t *rem = (int32_t *)malloc((size_t)(n ? n : 1) * sizeof(int32_t));
    int64_t *ctx = (int64_t *)malloc((size_t)(n ? n : 1) * sizeof(int64_t));
    int32_t *who = (int32_t *)malloc((size_t)(n ? n : 1) * sizeof(int32_t));
    if (!rem || !ctx || !who) { free(rem); free(ctx); free(who); return -1; }

    double t = 0.0;
    int32_t nb = n_act, next_q = 0;
    for (int32_t i = 0; i < n_act; ++i) {        /* actives are already in the batch */
        rem[i] = a_rem[i];
        ctx[i] = (int64_t)a_prompt[i] + a_gen[i];
        who[i] = i;
    }

    double *w = NULL;
    double t_admit = 0.0;      /* when a request arriving now would be admitted */
    int32_t s_admit = -1;      /* decode steps done by then; -1: not reached yet */
    int32_t s = 0, smax = 0;
    int have_d = 0;
    double elapsed = 0.0;      /* decode time since t_admit */
    *d_out = alpha;            /* an idle instance would take alpha */

    for (;;) {
        while (next_q < n_q && nb < cap) {       /* admit the head of the queue */
            t += delta * (double)q_prompt[next_q];
            rem[nb] = q_len[next_q];
            ctx[nb] = q_prompt[next_q];
            who[nb] = n_act + next_q;
            ++nb; ++next_q;
        }
        if (s_admit < 0 && next_q == n_q && nb < cap) {
            t_admit = t;
            s_admit = s;
            for (int32_t j = 0; j < nb; ++j) if (rem[j] > smax) smax = rem[j];
            w = (double *)malloc((size_t)(smax + 1) * sizeof(double));
            if (!w) { free(rem); free(ctx); free(who); return -1; }
            w[0] = 0.0;
        }
        if (nb == 0) break;
        int64_t c = 0;
        for (int32_t j = 0; j < nb; ++j) c += ctx[j];
        double step = fma(gamma, (double)c, fma(beta, (double)nb, alpha));
        if (!have_d) { *d_out = step; have_d = 1; }
        ++s;
        if (s_admit >= 0) {                      /* no admissions any more: decode time adds up on its own */
            elapsed += step;
            w[s - s_admit] = elapsed;
            t = t_admit + elapsed;
        } else {
            t += step;
        }
        int32_t m = 0;
        for (int32_t j = 0; j < nb; ++j) {
            rem[j] -= 1;
            ctx[j] += 1;
            if (rem[j] <= 0) {
                if (who[j] < n_act) { if (a_finish) a_finish[who[j]] = t; }
                else if (q_finish) q_finish[who[j] - n_act] = t;
            } else {
                rem[m] = rem[j]; ctx[m] = ctx[j]; who[m] = who[j]; ++m;
            }
        }
        nb = m;
    }
    *q_out = t_admit;
    *smax_out = smax;
    *w_out = w;
    free(rem); free(ctx); free(who);
    return 0;
}

/*
 * Simulate every instance; returns a handle holding q_g, d_g and the step
 * table of each instance, and writes each request's expected finish time.
 * a_finish / q_finish may be NULL.  All arrays are host arrays; act_off and
 * q_off are CSR offsets of length n_inst + 1; cap[g] bounds the batch of
 * instance g (NULL: unbounded).
 */
gro_fleet *gro_simulate(int32_t n_inst, int32_t n_class,
                        const double *delta, const double *alpha,
                        const double *beta, const double *gamma,
                        const int32_t *inst_class,
                        const int32_t *act_off, const int32_t *act_prompt,
                        const int32_t *act_gen, const int32_t *act_rem,
                        const int32_t *q_off, const int32_t *q_prompt, const int32_t *q_len,
                        const int32_t *cap /* per instance, may be NULL: no bound */,
                        double *a_finish, double *q_finish)
{
    gro_fleet *f = (gro_fleet *)calloc(1, sizeof(gro_fleet));
    if (!f) return NULL;
    f->n_inst = n_inst; f->n_class = n_class;
    f->delta = dup_d(delta, n_class); f->alpha = dup_d(alpha, n_class);
    f->beta = dup_d(beta, n_class);   f->gamma = dup_d(gamma, n_class);
    f->inst_class = (int32_t *)malloc((size_t)(n_inst ? n_inst : 1) * sizeof(int32_t));
    f->q = (double *)calloc((size_t)(n_inst ? n_inst : 1), sizeof(double));
    f->d = (double *)calloc((size_t)(n_inst ? n_inst : 1), sizeof(double));
    f->smax = (int32_t *)calloc((size_t)(n_inst ? n_inst : 1), sizeof(int32_t));
    f->w = (double **)calloc((size_t)(n_inst ? n_inst : 1), sizeof(double *));
    if (!f->delta || !f->alpha || !f->beta || !f->gamma || !f->inst_class ||
        !f->q || !f->d || !f->smax || !f->w) { gro_free(f); return NULL; }
    memcpy(f->inst_class, inst_class, (size_t)n_inst * sizeof(int32_t));

    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t g = 0; g < n_inst; ++g) {
        int c = inst_class[g];
        int32_t a0 = act_off[g], q0 = q_off[g];
        int rc = simulate_instance(delta[c], alpha[c], beta[c], gamma[c], cap ? cap[g] : INT32_MAX,
                                   act_off[g + 1] - a0, act_prompt + a0, act_gen + a0, act_rem + a0,
                                   q_off[g + 1] - q0, q_prompt + q0, q_len + q0,
                                   a_finish ? a_finish + a0 : NULL, q_finish ? q_finish + q0 : NULL,
                                   &f->q[g], &f->d[g], &f->smax[g], &f->w[g]);
        if (rc) {
#pragma omp atomic write
            failed = 1;
        }
    }
    if (failed) { gro_free(f); return NULL; }
    return f;
}

void gro_status(const gro_fleet *f, double *q, double *d, int32_t *smax)
{
    for (int32_t g = 0; g < f->n_inst; ++g) {
        if (q) q[g] = f->q[g];
        if (d) d[g] = f->d[g];
        if (smax) smax[g] = f->smax[g];
    }
}

/* copy of instance g's step table, w[0..smax] */
void gro_step_table(const gro_fleet *f, int32_t g, double *w)
{
    memcpy(w, f->w[g], (size_t)(f->smax[g] + 1) * sizeof(double));
}

/*
 * Eq. 2 for one (request, instance) pair.  The request waits q_g, prefills the
 * part of its c0 tokens that is not already cached on the instance (H of them
 * are: Eq. 2's "hit prefix token length"), then takes len decode steps in a
 * batch that holds it and whoever of the instance's requests is still running:
 * the first len step times of the instance, plus what its own presence adds to
 * each of them (one more batch member, its context c0 + s - 1 at step s: cached
 * tokens are still context).  Past the instance's last request only the new
 * request is left.
 */
static double pair_T(const gro_fleet *f, int32_t g, int64_t c0, int64_t len, int64_t hit)
{
    int c = f->inst_class[g];
    double alpha = f->alpha[c], beta = f->beta[c], gamma = f->gamma[c], delta = f->delta[c];
    int32_t smax = f->smax[g];
    double base = (len <= smax) ? f->w[g][len]
                                : f->w[g][smax] + (double)(len - smax) * alpha;
    double tri = (double)(len * (len - 1) / 2);
    double own = beta * (double)len + gamma * ((double)(c0 * len) + tri);
    return f->q[g] + delta * (double)(c0 - hit) + base + own;
}

/*
 * Reusable prefix of request r on instance g: the hits of request r are
 * entries hit_off[r] .. hit_off[r+1]-1 of (hit_inst, hit_len).  No entry: 0.
 * Should an instance be named twice the longer prefix counts; a prefix is
 * never longer than the request's tokens nor negative.
 */
static int64_t reusable_prefix(const int32_t *hit_off, const int32_t *hit_inst, const int32_t *hit_len,
                               int64_t r, int32_t g, int64_t c0)
{
    if (!hit_off) return 0;
    int64_t h = 0;
    for (int32_t k = hit_off[r]; k < hit_off[r + 1]; ++k)
        if (hit_inst[k] == g && hit_len[k] > h) h = hit_len[k];
    return h > c0 ? c0 : h;
}

/* T for every pair: out[r * n_inst + g]; hit_off may be NULL (no cached prefixes) */
void gro_pair_T(const gro_fleet *f, int64_t n_req, const int32_t *c0, const int32_t *len,
                const int32_t *hit_off, const int32_t *hit_inst, const int32_t *hit_len,
                double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_req; ++r)
        for (int32_t g = 0; g < f->n_inst; ++g)
            out[r * f->n_inst + g] =
                pair_T(f, g, c0[r], len[r], reusable_prefix(hit_off, hit_inst, hit_len, r, g, c0[r]));
}

/*
 * Alg. 1 for a batch, every request against the same snapshot of the fleet.
 * exclude (may be NULL) names an instance a request may not be sent to
 * (-1: none).  hit_off (may be NULL) lists cached prefixes, see above.
 * out_inst = -1 when no instance is allowed at all.
 */
void gro_route(const gro_fleet *f, int64_t n_req, const int32_t *c0, const int32_t *len,
               const double *deadline, const int32_t *exclude,
               const int32_t *hit_off, const int32_t *hit_inst, const int32_t *hit_len,
               int32_t *out_inst, double *out_slack, uint8_t *out_fallback, double *out_T)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_req; ++r) {
        int32_t ex = exclude ? exclude[r] : -1;
        double D = deadline[r];
        int32_t best_feas = -1, best_any = -1;
        double best_feas_d = 0.0, best_feas_T = 0.0, best_any_T = 0.0;
        for (int32_t g = 0; g < f->n_inst; ++g) {
            if (g == ex) continue;
            double T = pair_T(f, g, c0[r], len[r],
                              reusable_prefix(hit_off, hit_inst, hit_len, r, g, c0[r]));
            if (T <= D) {
                if (best_feas < 0 || f->d[g] > best_feas_d) {
                    best_feas = g; best_feas_d = f->d[g]; best_feas_T = T;
                }
            }
            if (best_any < 0 || T < best_any_T) { best_any = g; best_any_T = T; }
        }
        int32_t pick = best_feas >= 0 ? best_feas : best_any;
        double T = best_feas >= 0 ? best_feas_T : best_any_T;
        out_inst[r] = pick;
        if (out_slack) out_slack[r] = pick >= 0 ? D - T : 0.0;
        if (out_fallback) out_fallback[r] = (uint8_t)(best_feas < 0);
        if (out_T) out_T[r] = pick >= 0 ? T : 0.0;
    }
}

/*
 * How firmly Alg. 1's answer for each request stands when every latency may be
 * off by a relative eps (the GPU forms T in fp32): the same exhaustive scan as
 * gro_route, keeping per request what a comparison of another implementation's
 * answer needs.  rank[g] is the position of instance g in capability order
 * (largest d_g first, equal d_g by index); "first" below means smallest rank.
 *
 *   sure[r]    rank of the first instance with T*(1+eps) <= D (feasible whatever the error), n_inst if none
 *   maybe[r]   rank of the first instance with T*(1-eps) <= D (feasible for some error), n_inst if none
 *   tmin[r]    smallest T over the allowed instances (+inf if none is allowed)
 *   near[r]    number of allowed instances with T <= tmin*(1+2 eps)
 *   equal[r]   number of allowed instances with T == tmin, bit for bit
 *   picked_T[r]  T(r, picked[r]) (+inf when picked[r] is no allowed instance)
 *
 * It decides nothing itself.
 */
void gro_band(const gro_fleet *f, int64_t n_req, const int32_t *c0, const int32_t *len,
              const double *deadline, const int32_t *exclude,
              const int32_t *hit_off, const int32_t *hit_inst, const int32_t *hit_len,
              const int32_t *rank, double eps, const int32_t *picked,
              int32_t *sure, int32_t *maybe, double *tmin, int32_t *near, int32_t *equal,
              double *picked_T)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_req; ++r) {
        int32_t ex = exclude ? exclude[r] : -1;
        double D = deadline[r];
        int32_t s1 = f->n_inst, p1 = f->n_inst;
        double lo = INFINITY;
        for (int32_t g = 0; g < f->n_inst; ++g) {
            if (g == ex) continue;
            double T = pair_T(f, g, c0[r], len[r],
                              reusable_prefix(hit_off, hit_inst, hit_len, r, g, c0[r]));
            if (T * (1.0 + eps) <= D && rank[g] < s1) s1 = rank[g];
            if (T * (1.0 - eps) <= D && rank[g] < p1) p1 = rank[g];
            if (T < lo) lo = T;
        }
        int32_t n_near = 0, n_equal = 0;
        for (int32_t g = 0; g < f->n_inst; ++g) {
            if (g == ex) continue;
            double T = pair_T(f, g, c0[r], len[r],
                              reusable_prefix(hit_off, hit_inst, hit_len, r, g, c0[r]));
            if (T <= lo * (1.0 + 2.0 * eps)) ++n_near;
            if (T == lo) ++n_equal;
        }
        int32_t pk = picked[r];
        sure[r] = s1; maybe[r] = p1; tmin[r] = lo; near[r] = n_near; equal[r] = n_equal;
        picked_T[r] = (pk >= 0 && pk < f->n_inst && pk != ex)
                          ? pair_T(f, pk, c0[r], len[r],
                                   reusable_prefix(hit_off, hit_inst, hit_len, r, pk, c0[r]))
                          : INFINITY;
    }
}

int32_t gro_threads(void)
{
    int32_t n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
