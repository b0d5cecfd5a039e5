/*
 * libgoodroute: the batched routing math of GoodServe's predict-and-rectify
 * request router, for one AMD MI355X (gfx950).
 *
 * The three calls follow the paper's statement of the routing problem:
 *
 *   gr_build_status  the per-instance status that Eq. 2 (Sec. 3.1) needs (queuing
 *                    delay q_g, decode speed d_g) and the expected end-to-end
 *                    finish time of every request an instance already holds;
 *   gr_score_route   Alg. 1 ("Backend Selection Algorithm", Appendix) for a
 *                    batch of incoming requests: T(r,g) of Eq. 2 for every
 *                    (request, instance) pair, feasibility T <= D_r, the
 *                    just-enough choice of Sec. 3.4, the least-violation
 *                    fallback;
 *   gr_risk_scan     the periodic SLO-violation re-check of Sec. 3.4 over all
 *                    active requests, with a just-enough migration target for
 *                    every request found at risk.
 *
 * Time model.  Sec. 3.3 estimates q_g, p_g, d_g black-box; this library takes
 * them from an explicit model of a continuously batching instance of GPU
 * class c:  prefill costs delta_c seconds per prompt token, and one decode
 * step of a batch of B requests whose context lengths sum to C costs
 * alpha_c + beta_c*B + gamma_c*C seconds.  Queued requests are prefilled back
 * to back before decoding resumes; every step emits one token per batch
 * member.  "Now" is time 0 of every call.
 *
 * Conventions.  Every function returns GR_OK (0) or a negative GR_ERR_* code;
 * nothing throws or aborts.  Pointers marked DEVICE are device memory owned by
 * the caller (readable/writable by kernels on the current device); pointers
 * marked HOST are ordinary host memory read during the call.  Work is queued
 * on the given HIP stream (a hipStream_t passed as void*, NULL = default
 * stream) and the calls do not wait for it; outputs are valid once the stream
 * has been synchronised.  The handle owns its tables and workspace, sized at
 * gr_create; no call after gr_create allocates.  Calls on one handle must not
 * overlap.  Token counts are int32; times are seconds.
 *
 * The calls that take a stream only launch kernels on it (no copy, no memset,
 * no synchronisation), so a sequence of them can be recorded into a HIP graph
 * and replayed on the same buffers.  What the host decides at call time is
 * recorded with it: sizes, the blend weight and caps in force, and how a
 * batch is scored (gr_set_small_batch_pairs).  gr_create, gr_destroy, the
 * gr_set_* calls, gr_profile_* and gr_device_status copy or synchronise and
 * are not for use inside a capture.
 *
 * Input contract for device data (not validated on the host): remaining and
 * predicted lengths in [1, max_len]; prompt >= 1; generated >= 0; entries per
 * instance <= max_entries_per_inst; CSR offsets non-decreasing, starting at 0.
 * Kernels stay in bounds when the contract is broken (lengths are clamped,
 * surplus entries dropped) and raise a sticky bit readable with
 * gr_device_status.
 */
#ifndef GOODROUTE_H
#define GOODROUTE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gr_fleet gr_fleet;

enum {
    GR_OK = 0,
    GR_ERR_INVALID_ARG = -1, /* NULL where a pointer is required, negative size, bad class id */
    GR_ERR_TOO_LARGE = -2,   /* a size exceeds what the handle was created for, or a hard limit */
    GR_ERR_HIP = -3,         /* a HIP runtime call failed */
    GR_ERR_NO_STATUS = -4,   /* gr_score_route before any gr_build_status / gr_risk_scan; a blend before gr_observe */
    GR_ERR_NOMEM = -5        /* host or device allocation failed in gr_create */
};

/* bits of gr_device_status */
enum {
    GR_DEV_LEN_CLAMPED = 1,   /* a length outside [0, max_len] was clamped */
    GR_DEV_ENTRIES_DROPPED = 2 /* an instance held more than max_entries_per_inst entries */
};

/*
 * Create a fleet handle on the current HIP device.
 *   n_inst, n_class           M instances of n_class GPU classes (n_class <= 64)
 *   delta, alpha, beta, gamma HOST, n_class doubles each, all >= 0: the model above
 *   inst_class                HOST, n_inst class ids in [0, n_class)
 *   max_entries_per_inst      upper bound of active + queued requests on one instance
 *   max_len                   upper bound of any remaining / predicted decode length
 *   max_requests              upper bound of n_req of one gr_score_route call
 * Hard limits: max_entries_per_inst <= 2048; max_len <= 32767.
 * Device memory held by the handle until gr_destroy, all of it allocated here: with
 * cap = max_entries_per_inst rounded up to 64, 128, .. 2048, M' = n_inst rounded up to a
 * multiple of 128 and N = max(max_requests, n_inst * max_entries_per_inst),
 *   18 * n_inst * cap bytes          instance tables and the lists of feedback routing,
 *   8 * n_inst * max_entries_per_inst bytes   per held request (its instance, a spare finish time),
 *   4.25 * M' * min(max_len + 1, N) bytes     the per-(distinct length, instance) table of a scoring
 *                                    pass, reserved for the worst case whatever the batches turn
 *                                    out to be (285 MB for 4 096 instances and max_len 16 384),
 *   16.2 * N bytes                   the requests of a scoring pass in grouped order,
 * plus a few arrays of n_inst or max_len + 1 words.
 */
int gr_create(gr_fleet** out, int32_t n_inst, int32_t n_class,
              const double* delta, const double* alpha, const double* beta, const double* gamma,
              const int32_t* inst_class,
              int32_t max_entries_per_inst, int32_t max_len, int64_t max_requests);

/* Free the handle and its device memory (waits for the device first). NULL is allowed. */
int gr_destroy(gr_fleet* f);

/*
 * Step 1 (Eq. 2's per-instance terms; "expected finish time" of Sec. 3.4).
 * For every instance: q_g = delta * (sum of queued prompts); the requests it
 * holds are ordered by remaining length, which turns the step-by-step run of
 * its batch into a closed form; out come the finish time of every request,
 * d_g = duration of the instance's next decode step (alpha for an idle
 * instance), the capability rank used by Alg. 1's argmax d_g, and the
 * instance tables kept in the handle for gr_score_route.
 *
 *   act_off        DEVICE int32[n_inst+1]  CSR offsets of active requests by instance
 *   act_prompt     DEVICE int32[n_active]  prompt tokens
 *   act_gen        DEVICE int32[n_active]  tokens generated so far
 *   act_rem        DEVICE int32[n_active]  predicted remaining decode length
 *   q_off          DEVICE int32[n_inst+1]  CSR offsets of queued requests by instance
 *   q_prompt,q_len DEVICE int32[n_queued]  prompt tokens, predicted decode length
 *   n_active, n_queued                     array lengths (host values)
 *   out_act_finish DEVICE float[n_active]  expected finish time, same order as inputs
 *   out_q_finish   DEVICE float[n_queued]  may be NULL
 *   out_d          DEVICE double[n_inst]   may be NULL
 *   out_rank       DEVICE int32[n_inst]    may be NULL; 0 = largest d_g, ties by index
 */
int gr_build_status(gr_fleet* f,
                    const int32_t* act_off, const int32_t* act_prompt,
                    const int32_t* act_gen, const int32_t* act_rem, int64_t n_active,
                    const int32_t* q_off, const int32_t* q_prompt, const int32_t* q_len,
                    int64_t n_queued,
                    float* out_act_finish, float* out_q_finish,
                    double* out_d, int32_t* out_rank, void* hip_stream);

/*
 * Step 2 (Alg. 1 on a batch; every request is scored against the same
 * snapshot: the tables of the last gr_build_status / gr_risk_scan).
 * A request that goes to instance g waits q_g, prefills its ctx0 tokens
 * (no cached prefix), then decodes pred_len steps in g's batch:
 *   T(r,g) = q_g + delta*ctx0 + [time of g's next pred_len steps with r in the batch].
 * Feasible iff T <= budget.  Choice: the feasible instance with the largest
 * d_g (ties: lowest index); if none, the instance with the smallest T (ties:
 * lowest index).
 *
 *   n_req          number of requests (0 allowed)
 *   ctx0           DEVICE int32[n_req]  tokens to prefill (prompt; prompt+generated when migrating)
 *   pred_len       DEVICE int32[n_req]  predicted decode length
 *   budget         DEVICE float[n_req]  D_r, seconds from now
 *   exclude_inst   DEVICE int32[n_req]  instance a request may not go to, -1 none; may be NULL
 *   out_inst       DEVICE int32[n_req]  chosen instance (-1 if every instance is excluded)
 *   out_slack      DEVICE float[n_req]  budget - T(r, chosen)
 *   out_fallback   DEVICE uint8[n_req]  1 if no instance was feasible; may be NULL
 *   out_T          DEVICE float[n_req*n_inst], row-major; may be NULL. Every pair's
 *                  T, for checking; costs 4 bytes of traffic per pair.
 */
int gr_score_route(gr_fleet* f, int64_t n_req,
                   const int32_t* ctx0, const int32_t* pred_len, const float* budget,
                   const int32_t* exclude_inst,
                   int32_t* out_inst, float* out_slack, uint8_t* out_fallback,
                   float* out_T, void* hip_stream);

/*
 * gr_score_route for callers that cannot allocate device memory or call anything that might:
 * code under HIP graph capture, tight serving loops, harnesses that forbid it.  Same inputs,
 * outputs and answers as gr_score_route's pair-by-pair pass (a thread per (request, instance)
 * pair, whatever gr_set_small_batch_pairs says; no out_T), for at most
 * GR_NOALLOC_MAX_REQUESTS requests per call; more is GR_ERR_TOO_LARGE.  The running
 * selections of the pass (16 bytes per request) live in a fixed array of 64 KiB in the
 * library's device image instead of the handle's workspace; the call queues three kernels on
 * the stream (one sets the array's slots for this batch; two more, for the capability order,
 * on the first scoring call after a status build and whenever the stream is being captured)
 * and calls no hipMalloc, hipFree,
 * memset, copy or synchronisation.  Every GPU holds one such array for the life of the
 * process and every call on that GPU uses it, whatever the handle: calls that overlap on one
 * GPU (two streams, two threads, two handles) race and must be serialised by the caller.
 * The handle must have been created on the current device (the array's address is looked up
 * once per device, in gr_create).
 */
#define GR_NOALLOC_MAX_REQUESTS 4096
int gr_score_route_noalloc(gr_fleet* f, int64_t n_req,
                           const int32_t* ctx0, const int32_t* pred_len, const float* budget,
                           const int32_t* exclude_inst,
                           int32_t* out_inst, float* out_slack, uint8_t* out_fallback,
                           void* hip_stream);

/*
 * Step 2 with cached prefixes (Eq. 2's hit prefix token length H_{r,g};
 * Alg. 1's prefix-reuse lookup before T(r,g) is formed).  As gr_score_route,
 * but request r already has hit_len[k] of its ctx0 tokens cached on instance
 * hit_inst[k] for k = hit_off[r] .. hit_off[r+1]-1; those tokens are not
 * prefilled again (they still count as context while decoding):
 *   T(r,g) = q_g + delta*(ctx0 - H_{r,g}) + [decode time as in gr_score_route].
 * Pairs without an entry have H = 0.  An instance named more than once for a
 * request counts with its longest prefix; a prefix is cut to [0, ctx0].
 *
 *   hit_off    DEVICE int32[n_req+1]  CSR offsets by request, non-decreasing, hit_off[0] = 0
 *   hit_inst   DEVICE int32[n_hits]   instance of each cached prefix (entries outside [0, n_inst) are ignored)
 *   hit_len    DEVICE int32[n_hits]   its length in tokens
 *   n_hits     number of entries (0 allowed: same as gr_score_route)
 * out_T, when given, holds T with the prefixes applied.
 */
int gr_score_route_cached(gr_fleet* f, int64_t n_req,
                          const int32_t* ctx0, const int32_t* pred_len, const float* budget,
                          const int32_t* exclude_inst,
                          const int32_t* hit_off, const int32_t* hit_inst, const int32_t* hit_len,
                          int64_t n_hits,
                          int32_t* out_inst, float* out_slack, uint8_t* out_fallback,
                          float* out_T, void* hip_stream);

/*
 * Step 2 with the status kept up to date between decisions.  The paper's proxy
 * runs Alg. 1 request after request, refreshing the instances' status before
 * each decision, so that a request sees the ones routed before it; a batch
 * scored against one snapshot sends every similar request to the same
 * instance.  Here the batch is taken `chunk` requests at a time, in order: a
 * chunk is decided as by gr_score_route, then each of its requests joins the
 * queue of the instance it was sent to (prompt = ctx0, length = pred_len; it is
 * prefilled behind the queue and decodes with the batch), the status is
 * rebuilt, and the next chunk is decided.  chunk = 1 is the paper's order;
 * chunk >= n_req is gr_score_route.  On return the handle's tables hold the
 * status with all n_req requests in place; the next gr_build_status or
 * gr_risk_scan starts from the caller's arrays again.
 *
 * The arrays passed to the last gr_build_status / gr_risk_scan are read again
 * and must still be valid and unchanged.  An instance takes routed requests
 * while it holds fewer than max_entries_per_inst entries; beyond that the
 * request is still reported but no longer counted (GR_DEV_ENTRIES_DROPPED).
 * Cost: one scoring pass and one status rebuild per chunk; the rebuild leaves
 * instances that were given nothing in the chunk as they are (unless the blend
 * weight, the observations or the caps have changed since the tables were built:
 * then the first rebuild of the call takes every instance).
 *
 *   chunk      requests per decision round, >= 1 (cut to max_requests)
 * Other arguments as gr_score_route (no out_T).
 */
int gr_route_feedback(gr_fleet* f, int64_t n_req, int64_t chunk,
                      const int32_t* ctx0, const int32_t* pred_len, const float* budget,
                      const int32_t* exclude_inst,
                      int32_t* out_inst, float* out_slack, uint8_t* out_fallback, void* hip_stream);

/*
 * Step 3 (Sec. 3.4, periodic re-check).  Rebuilds the status from refreshed
 * remaining lengths (as gr_build_status, replacing the handle's tables), flags
 * every active request whose expected finish exceeds its budget
 * (finish > budget, compared in fp64), and for every flagged request runs
 * Alg. 1 over all other instances with ctx0 = prompt + generated (migration
 * moves token IDs, the target prefills them again), pred_len = its refreshed
 * remaining length and D = its budget.  Targets are scored against the
 * refreshed snapshot, the request still counted where it runs now.
 *
 *   act_budget       DEVICE float[n_active]  arrival + SLO - now (may be negative)
 *   out_flag         DEVICE uint8[n_active]
 *   out_finish       DEVICE float[n_active]
 *   out_target       DEVICE int32[n_active]  -1 if not flagged (or no other instance)
 *   out_target_slack DEVICE float[n_active]  0 if not flagged
 *   out_n_flagged    DEVICE int32[1]         may be NULL
 */
int gr_risk_scan(gr_fleet* f,
                 const int32_t* act_off, const int32_t* act_prompt,
                 const int32_t* act_gen, const int32_t* act_rem_refreshed, int64_t n_active,
                 const int32_t* q_off, const int32_t* q_prompt, const int32_t* q_len,
                 int64_t n_queued,
                 const float* act_budget,
                 uint8_t* out_flag, float* out_finish,
                 int32_t* out_target, float* out_target_slack, int32_t* out_n_flagged,
                 void* hip_stream);

/*
 * The paper's own status estimate (Sec. 3.3; Alg. 1 before it forms T(r,g)):
 * q_g, p_g, d_g taken black-box from what was recently observed on the
 * instance and smoothed by an exponential moving average,
 *   x_g <- weight * sample_g + (1 - weight) * x_g,
 * for each of the three terms that comes with a new sample (a term's first
 * sample is its estimate).  Samples: the average waiting time of instance g,
 * its prefill seconds per token, its decode seconds per token (TPOT).
 *
 *   weight       in [0, 1]
 *   obs_wait, obs_prefill, obs_decode   DEVICE float[n_inst] each; NULL = no new sample of that term
 * The estimates live in the handle, in double precision.  Tables and capability order of the
 * last gr_build_status / gr_risk_scan keep the estimates they were built with: new samples show
 * from the next build on.
 */
int gr_observe(gr_fleet* f, double weight, const float* obs_wait, const float* obs_prefill,
               const float* obs_decode, void* hip_stream);

/*
 * How much of that black-box estimate enters every figure the library
 * produces.  With weight w every estimate is
 *   (1 - w) * [white-box value] + w * [Eq. 2 with the smoothed q_g, p_g, d_g]:
 * T(r,g) = q_g + p_g*(ctx0 - H) + d_g*pred_len for a pair; d_g itself for
 * Alg. 1's argmax; d_g per remaining token for the finish time of a running
 * request, q_g + p_g*prompt + d_g*length for a queued one.  w = 0 (the state
 * after gr_create) is the white-box model alone, w = 1 the paper's estimator
 * alone.  Takes effect at the next gr_build_status / gr_risk_scan.  Host call.
 * GR_ERR_NO_STATUS if w > 0 before all three terms have been observed.
 */
int gr_set_blend(gr_fleet* f, double black_box_weight);

/*
 * The paper's second constraint (Sec. 3.1): the number of requests an instance
 * serves concurrently is bounded by its memory.  With a cap B_g, at most B_g
 * requests of instance g decode together: queued requests are admitted in
 * queue order whenever the batch has room (at time 0 and after every decode
 * step); an admission prefills the request, stalling the batch, and puts it
 * into the batch.  Requests already running keep running even if they
 * outnumber the cap.  A request that arrives now is last in the queue, so
 *   q_g = the time at which it would be admitted,
 * after which nobody else joins and T(r,g) = q_g + delta*(ctx0 - H) + [its
 * pred_len decode steps in the batch as it is then].  d_g is the duration of
 * the next decode step that runs.  Every call uses the caps from the next
 * gr_build_status / gr_risk_scan on.  With room for everybody and a newcomer
 * (B_g > entries of g) nothing changes.
 *
 *   cap   HOST int32[n_inst], each >= 1; NULL removes the caps.
 * Host call; waits for the device.
 *
 * With gr_route_feedback under caps, the requests of a chunk queue up on their instances in
 * the order of the batch, whatever the chunk size (without caps the order of a queue shows
 * in no output and is not kept).
 */
int gr_set_batch_cap(gr_fleet* f, const int32_t* cap);

/*
 * How a batch is scored.  Alg. 1 is the same either way; the work is laid out
 * differently.  A large batch is grouped by predicted length, the decode term
 * of Eq. 2 is tabulated once per (distinct length, instance), and tiles of 32
 * requests run against all instances.  A batch of a few requests (the paper
 * routes one arriving request at a time) skips grouping and table: a thread
 * per (request, instance) pair finds its own segment by binary search.
 *
 *   max_pairs   gr_score_route and gr_route_feedback score a batch (a chunk)
 *               pair by pair when n_req * (n_inst rounded up to 128) is at
 *               most this and n_req <= 4096.  0: never.  Default 262 144.
 * gr_score_route_cached and gr_risk_scan always take the grouped path.
 * Equal latencies go to the lowest instance index either way.
 */
int gr_set_small_batch_pairs(gr_fleet* f, int64_t max_pairs);

/*
 * Synchronises the device and returns the OR of the GR_DEV_* bits raised by
 * kernels since gr_create (HOST int32 out).  Not for the hot path.
 */
int gr_device_status(gr_fleet* f, int32_t* out_bits);

/*
 * Per-kernel timing, for benchmarks (not cited from the paper: a measuring aid).
 * gr_profile_enable(f, n) with n > 0 makes every kernel launch of the following
 * calls record a pair of HIP events on the call's stream, up to n launches
 * (events are created here, not in the calls); n = 0 switches timing off.
 * gr_profile_read synchronises the device, adds up the elapsed time and the
 * number of launches per kernel id since the last read into HOST arrays of
 * n_kernels entries, and forgets them.  Kernel ids run from 0 to
 * gr_profile_kernel_count() - 1; gr_profile_kernel_name gives a static name.
 * gr_profile_select restricts the timing to the kernel ids whose bit is set in
 * kernel_mask (all of them after gr_create): an event pair costs a few
 * microseconds of stream time, which adds up over a dozen short launches.
 * gr_profile_read_launches is gr_profile_read launch by launch, in launch order:
 * kernel id and elapsed milliseconds of up to max_launches recorded launches
 * into HOST arrays, their number into *n_launches (for medians and percentiles).
 */
int gr_profile_enable(gr_fleet* f, int32_t max_launches);
int gr_profile_select(gr_fleet* f, uint64_t kernel_mask);
int gr_profile_read(gr_fleet* f, int32_t n_kernels, double* total_ms, int64_t* launches);
int gr_profile_read_launches(gr_fleet* f, int32_t max_launches, int32_t* kernel_id, float* ms, int32_t* n_launches);
int32_t gr_profile_kernel_count(void);
const char* gr_profile_kernel_name(int32_t id);

/* Static, human-readable text for a return code. */
const char* gr_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* GOODROUTE_H */
