// Host entry points of libgoodroute: the fleet handle, argument checks and the
// order in which the kernels of status.hip and score.hip are queued.
#include <cstdlib>
#include <new>

#include "common.h"

namespace gr {
namespace {

const char* const kKernelNames[kNumKernels] = {
    "k_build", "k_rank_count", "k_rank_final",
    "k_hist<route>", "k_scan<route>", "k_group<route>", "k_tile<route>",
    "k_hist<migrate>", "k_scan<migrate>", "k_group<migrate>", "k_tile<migrate>",
    "k_hits<route>", "k_direct", "k_direct_finish"};

template <typename T>
bool dev_alloc(T** p, size_t n)
{
    return hipMalloc(reinterpret_cast<void**>(p), (n ? n : 1) * sizeof(T)) == hipSuccess;
}

bool status_args_ok(const gr_fleet* f, const int32_t* act_off, const int32_t* act_prompt,
                    const int32_t* act_gen, const int32_t* act_rem, int64_t n_active,
                    const int32_t* q_off, const int32_t* q_prompt, const int32_t* q_len, int64_t n_queued,
                    int* rc)
{
    *rc = GR_ERR_INVALID_ARG;
    if (!f || !act_off || !q_off || n_active < 0 || n_queued < 0) return false;
    if (n_active > 0 && (!act_prompt || !act_gen || !act_rem)) return false;
    if (n_queued > 0 && (!q_prompt || !q_len)) return false;
    *rc = GR_ERR_TOO_LARGE;
    if (n_active > f->max_active || n_queued > f->max_active) return false;
    *rc = GR_OK;
    return true;
}

}  // namespace
}  // namespace gr

using namespace gr;

extern "C" {

int gr_create(gr_fleet** out, int32_t n_inst, int32_t n_class,
              const double* delta, const double* alpha, const double* beta, const double* gamma,
              const int32_t* inst_class, int32_t max_entries_per_inst, int32_t max_len,
              int64_t max_requests)
{
    if (!out) return GR_ERR_INVALID_ARG;
    *out = nullptr;
    if (n_inst <= 0 || n_class <= 0 || !delta || !alpha || !beta || !gamma || !inst_class ||
        max_entries_per_inst < 0 || max_len < 1 || max_requests < 0)
        return GR_ERR_INVALID_ARG;
    if (n_class > kMaxClasses || max_entries_per_inst > kMaxEntries || max_len > kMaxLen ||
        max_requests > (int64_t(1) << 30) || n_inst > (1 << 20))
        return GR_ERR_TOO_LARGE;
    for (int c = 0; c < n_class; ++c)
        if (!(delta[c] >= 0) || !(alpha[c] >= 0) || !(beta[c] >= 0) || !(gamma[c] >= 0))
            return GR_ERR_INVALID_ARG;
    for (int g = 0; g < n_inst; ++g)
        if (inst_class[g] < 0 || inst_class[g] >= n_class) return GR_ERR_INVALID_ARG;
    if ((int64_t)n_inst * max_entries_per_inst > (int64_t(1) << 30)) return GR_ERR_TOO_LARGE;

    gr_fleet* f = new (std::nothrow) gr_fleet;
    if (!f) return GR_ERR_NOMEM;
    f->n_inst = n_inst; f->n_class = n_class;
    f->max_entries = max_entries_per_inst; f->max_len = max_len; f->max_requests = max_requests;
    f->max_active = (int64_t)n_inst * max_entries_per_inst;
    f->req_cap = f->max_active > max_requests ? f->max_active : max_requests;
    f->epl = 1;
    while (kWave * f->epl < max_entries_per_inst) f->epl *= 2;
    f->cap = kWave * f->epl;
    f->m_pad = ((n_inst + 2 * kWave - 1) / (2 * kWave)) * (2 * kWave);
    f->bins = max_len + 1;
    f->row_cap = f->req_cap < f->bins ? f->req_cap : f->bins;
    if (f->row_cap < 1) f->row_cap = 1;
    if (hipGetDevice(&f->device) != hipSuccess) { delete f; return GR_ERR_HIP; }
    if (score_lds_bytes(f) > 160 * 1024) { delete f; return GR_ERR_TOO_LARGE; }

    const size_t tab = (size_t)n_inst * f->cap;
    const bool ok =
        dev_alloc(&f->cls, n_class) && dev_alloc(&f->inst_class, n_inst) &&
        dev_alloc(&f->tabR, tab) && dev_alloc(&f->tabGH, tab) && dev_alloc(&f->headGH, n_inst) &&
        dev_alloc(&f->hN, n_inst) && dev_alloc(&f->hD, n_inst) &&
        dev_alloc(&f->emaQ, n_inst) && dev_alloc(&f->emaP, n_inst) && dev_alloc(&f->emaD, n_inst) &&
        dev_alloc(&f->rank_acc, n_inst) && dev_alloc(&f->rank, n_inst) && dev_alloc(&f->order, f->m_pad) && dev_alloc(&f->posK, f->m_pad) &&
        dev_alloc(&f->act_inst, f->max_active) && dev_alloc(&f->counters, 1) &&
        dev_alloc(&f->pend_cnt, n_inst) && dev_alloc(&f->commit_mark, n_inst) && dev_alloc(&f->pend_touched, n_inst) && dev_alloc(&f->pend_prompt, tab) && dev_alloc(&f->pend_len, tab) &&
        dev_alloc(&f->scratch_finish, f->max_active) && dev_alloc(&f->batch_cap, n_inst) &&
        dev_alloc(&f->len_cnt, f->bins) && dev_alloc(&f->len_base, f->bins) &&
        dev_alloc(&f->row_len, f->row_cap) && dev_alloc(&f->row_off, f->row_cap + 1) &&
        dev_alloc(&f->tile_off, f->row_cap + 1) && dev_alloc(&f->len_row, f->bins) && dev_alloc(&f->len_ceil, f->bins) && dev_alloc(&f->totals, 4) &&
        dev_alloc(&f->recs, f->req_cap) && dev_alloc(&f->memo, (size_t)f->row_cap * f->m_pad) &&
        dev_alloc(&f->tile_row, (size_t)(f->req_cap / kTileReq + f->row_cap + 1)) &&
        dev_alloc(&f->grp_min, (size_t)f->row_cap * (f->m_pad / kMemoP)) && dev_alloc(&f->grp_k, f->m_pad / kMemoP) &&
        dev_alloc(&f->direct_best, 2 * (size_t)kDirectMax);
    if (!ok) { gr_destroy(f); return GR_ERR_NOMEM; }

    ClassCoef* host = static_cast<ClassCoef*>(malloc(sizeof(ClassCoef) * n_class));
    if (!host) { gr_destroy(f); return GR_ERR_NOMEM; }
    for (int c = 0; c < n_class; ++c) host[c] = ClassCoef{delta[c], alpha[c], beta[c], gamma[c]};
    const hipError_t e1 = hipMemcpy(f->cls, host, sizeof(ClassCoef) * n_class, hipMemcpyHostToDevice);
    const hipError_t e2 = hipMemcpy(f->inst_class, inst_class, sizeof(int) * n_inst, hipMemcpyHostToDevice);
    const hipError_t e3 = hipMemset(f->counters, 0, sizeof(int));
    const hipError_t e4 = hipMemset(f->len_cnt, 0, sizeof(int) * f->bins);
    const hipError_t e5 = hipMemset(f->totals, 0, sizeof(int) * 4);
    const hipError_t e6 = hipMemset(f->pend_cnt, 0, sizeof(int) * n_inst);
    const hipError_t e8 = hipMemset(f->pend_touched, 0, sizeof(int) * n_inst);
    const hipError_t e9 = hipMemset(f->commit_mark, 0, sizeof(int) * n_inst);
    const hipError_t e7 = hipMemset(f->direct_best, 0xFF, sizeof(unsigned long long) * 2 * kDirectMax);
    free(host);
    if (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess || e4 != hipSuccess || e5 != hipSuccess || e6 != hipSuccess || e7 != hipSuccess || e8 != hipSuccess || e9 != hipSuccess ||
        hipDeviceSynchronize() != hipSuccess) {
        gr_destroy(f);
        return GR_ERR_HIP;
    }
    if (score_prepare(f) != GR_OK || status_prepare() != GR_OK) { gr_destroy(f); return GR_ERR_HIP; }
    {   // the address of the fixed scratch array on this device, for gr_score_route_noalloc
        unsigned long long* unused = nullptr;
        const int rc = static_scratch(f->device, &unused);
        if (rc != GR_OK && rc != GR_ERR_TOO_LARGE) { gr_destroy(f); return rc; }
    }
    *out = f;
    return GR_OK;
}

int gr_destroy(gr_fleet* f)
{
    if (!f) return GR_OK;
    (void)hipDeviceSynchronize();
    void* ptrs[] = {f->cls, f->inst_class, f->tabR, f->tabGH, f->headGH, f->hN, f->hD, f->emaQ, f->emaP, f->emaD, f->rank_acc,
                    f->rank, f->order, f->posK, f->act_inst, f->pend_cnt, f->commit_mark, f->pend_touched, f->pend_prompt, f->pend_len,
                    f->scratch_finish, f->batch_cap, f->counters, f->len_cnt, f->len_base, f->row_len,
                    f->row_off, f->tile_off, f->len_row, f->len_ceil, f->totals, f->recs, f->memo, f->tile_row, f->grp_min, f->grp_k, f->direct_best};
    int rc = GR_OK;
    for (void* p : ptrs)
        if (p && hipFree(p) != hipSuccess) rc = GR_ERR_HIP;
    for (hipEvent_t e : f->prof.events) (void)hipEventDestroy(e);
    delete f;
    return rc;
}

int gr_build_status(gr_fleet* f, const int32_t* act_off, const int32_t* act_prompt,
                    const int32_t* act_gen, const int32_t* act_rem, int64_t n_active,
                    const int32_t* q_off, const int32_t* q_prompt, const int32_t* q_len,
                    int64_t n_queued, float* out_act_finish, float* out_q_finish,
                    double* out_d, int32_t* out_rank, void* hip_stream)
{
    int rc;
    if (!status_args_ok(f, act_off, act_prompt, act_gen, act_rem, n_active, q_off, q_prompt, q_len,
                        n_queued, &rc))
        return rc;
    if (n_active > 0 && !out_act_finish) return GR_ERR_INVALID_ARG;
    StatusIn in{};
    in.act_off = act_off; in.act_prompt = act_prompt; in.act_gen = act_gen; in.act_rem = act_rem;
    in.q_off = q_off; in.q_prompt = q_prompt; in.q_len = q_len;
    in.n_active = n_active; in.n_queued = n_queued;
    in.out_act_finish = out_act_finish; in.out_q_finish = out_q_finish;
    in.out_d = out_d; in.out_rank = out_rank;
    return launch_status(f, in, static_cast<hipStream_t>(hip_stream));
}

namespace {
// gr_score_route; `small_batch_ok`: a batch of a few requests may be scored pair by pair,
// which leaves no table of per-length values behind
int score_route(gr_fleet* f, int64_t n_req, const int32_t* ctx0, const int32_t* pred_len,
                const float* budget, const int32_t* exclude_inst, int32_t* out_inst,
                float* out_slack, uint8_t* out_fallback, float* out_T, void* hip_stream, bool small_batch_ok)
{
    if (!f || n_req < 0) return GR_ERR_INVALID_ARG;
    if (!f->has_status) return GR_ERR_NO_STATUS;
    if (n_req == 0) return GR_OK;
    if (!ctx0 || !pred_len || !budget || !out_inst || !out_slack) return GR_ERR_INVALID_ARG;
    if (n_req > f->max_requests) return GR_ERR_TOO_LARGE;
    ReqSrc src{};
    src.ctx0 = ctx0; src.pred_len = pred_len; src.budget = budget; src.exclude = exclude_inst;
    src.n = n_req;
    ScoreOut o{};
    o.inst = out_inst; o.slack = out_slack; o.fallback = out_fallback; o.T = out_T;
    return launch_score(f, src, false, o, static_cast<hipStream_t>(hip_stream), small_batch_ok);
}
}  // namespace

int gr_score_route(gr_fleet* f, int64_t n_req, const int32_t* ctx0, const int32_t* pred_len,
                   const float* budget, const int32_t* exclude_inst, int32_t* out_inst,
                   float* out_slack, uint8_t* out_fallback, float* out_T, void* hip_stream)
{
    return score_route(f, n_req, ctx0, pred_len, budget, exclude_inst, out_inst, out_slack, out_fallback, out_T,
                       hip_stream, true);
}

int gr_score_route_noalloc(gr_fleet* f, int64_t n_req, const int32_t* ctx0, const int32_t* pred_len,
                           const float* budget, const int32_t* exclude_inst, int32_t* out_inst,
                           float* out_slack, uint8_t* out_fallback, void* hip_stream)
{
    if (!f || n_req < 0) return GR_ERR_INVALID_ARG;
    if (n_req > GR_NOALLOC_MAX_REQUESTS) return GR_ERR_TOO_LARGE;
    if (!f->has_status) return GR_ERR_NO_STATUS;
    if (n_req == 0) return GR_OK;
    if (!ctx0 || !pred_len || !budget || !out_inst || !out_slack) return GR_ERR_INVALID_ARG;
    ReqSrc src{};
    src.ctx0 = ctx0; src.pred_len = pred_len; src.budget = budget; src.exclude = exclude_inst;
    src.n = n_req;
    ScoreOut o{};
    o.inst = out_inst; o.slack = out_slack; o.fallback = out_fallback;
    return launch_score_static(f, src, o, static_cast<hipStream_t>(hip_stream));
}

int gr_score_route_cached(gr_fleet* f, int64_t n_req, const int32_t* ctx0, const int32_t* pred_len,
                          const float* budget, const int32_t* exclude_inst,
                          const int32_t* hit_off, const int32_t* hit_inst, const int32_t* hit_len,
                          int64_t n_hits, int32_t* out_inst, float* out_slack, uint8_t* out_fallback,
                          float* out_T, void* hip_stream)
{
    if (n_hits < 0 || (n_req > 0 && !hit_off) || (n_hits > 0 && (!hit_inst || !hit_len)))
        return GR_ERR_INVALID_ARG;
    // (the correction below reads the per-length table of the grouped pass)
    const int rc = score_route(f, n_req, ctx0, pred_len, budget, exclude_inst, out_inst, out_slack,
                               out_fallback, out_T, hip_stream, false);
    if (rc != GR_OK || n_req == 0) return rc;
    ReqSrc src{};
    src.ctx0 = ctx0; src.pred_len = pred_len; src.budget = budget; src.exclude = exclude_inst;
    src.n = n_req;
    ScoreOut o{};
    o.inst = out_inst; o.slack = out_slack; o.fallback = out_fallback; o.T = out_T;
    return launch_hits(f, src, hit_off, hit_inst, hit_len, n_hits, o, static_cast<hipStream_t>(hip_stream));
}

int gr_route_feedback(gr_fleet* f, int64_t n_req, int64_t chunk, const int32_t* ctx0,
                      const int32_t* pred_len, const float* budget, const int32_t* exclude_inst,
                      int32_t* out_inst, float* out_slack, uint8_t* out_fallback, void* hip_stream)
{
    if (!f || n_req < 0 || chunk < 1) return GR_ERR_INVALID_ARG;
    if (!f->has_status) return GR_ERR_NO_STATUS;
    if (n_req == 0) return GR_OK;
    if (!ctx0 || !pred_len || !budget || !out_inst || !out_slack) return GR_ERR_INVALID_ARG;
    if (chunk > f->max_requests) chunk = f->max_requests;
    if (chunk < 1) return GR_ERR_TOO_LARGE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // rebuilds start from the caller's last status inputs; what they report goes to scratch
    StatusIn in = f->last_in;
    in.use_pending = 1;
    in.act_budget = nullptr; in.out_flag = nullptr;
    in.out_act_finish = f->scratch_finish; in.out_q_finish = nullptr; in.out_d = nullptr; in.out_rank = nullptr;
    for (int64_t s0 = 0; s0 < n_req; s0 += chunk) {
        const int64_t n = n_req - s0 < chunk ? n_req - s0 : chunk;
        ReqSrc src{};
        src.ctx0 = ctx0 + s0; src.pred_len = pred_len + s0; src.budget = budget + s0;
        src.exclude = exclude_inst ? exclude_inst + s0 : nullptr;
        src.n = n;
        ScoreOut o{};
        o.inst = out_inst + s0; o.slack = out_slack + s0; o.fallback = out_fallback ? out_fallback + s0 : nullptr;
        int rc = launch_score(f, src, false, o, s, true);
        if (rc == GR_OK) rc = launch_commit(f, n, out_inst + s0, ctx0 + s0, pred_len + s0, s);
        // instances that were given nothing keep their tables, unless those are from an earlier blend
        // weight or earlier caps
        in.only_touched = f->tables_current ? 1 : 0;
        if (rc == GR_OK) rc = launch_status(f, in, s);
        if (rc != GR_OK) return rc;
    }
    return GR_OK;
}

int gr_risk_scan(gr_fleet* f, const int32_t* act_off, const int32_t* act_prompt,
                 const int32_t* act_gen, const int32_t* act_rem_refreshed, int64_t n_active,
                 const int32_t* q_off, const int32_t* q_prompt, const int32_t* q_len,
                 int64_t n_queued, const float* act_budget, uint8_t* out_flag, float* out_finish,
                 int32_t* out_target, float* out_target_slack, int32_t* out_n_flagged,
                 void* hip_stream)
{
    int rc;
    if (!status_args_ok(f, act_off, act_prompt, act_gen, act_rem_refreshed, n_active, q_off, q_prompt,
                        q_len, n_queued, &rc))
        return rc;
    if (n_active > 0 && (!act_budget || !out_flag || !out_finish || !out_target || !out_target_slack))
        return GR_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    StatusIn in{};
    in.act_off = act_off; in.act_prompt = act_prompt; in.act_gen = act_gen; in.act_rem = act_rem_refreshed;
    in.q_off = q_off; in.q_prompt = q_prompt; in.q_len = q_len;
    in.act_budget = act_budget;
    in.n_active = n_active; in.n_queued = n_queued;
    in.out_act_finish = out_finish; in.out_flag = out_flag;
    rc = launch_status(f, in, s);
    if (rc != GR_OK) return rc;
    ReqSrc src{};
    src.act_prompt = act_prompt; src.act_gen = act_gen; src.act_rem = act_rem_refreshed;
    src.act_inst = f->act_inst; src.flag = out_flag; src.act_budget = act_budget;
    src.n = n_active;
    ScoreOut o{};
    o.inst = out_target; o.slack = out_target_slack; o.n_selected = out_n_flagged;
    return launch_score(f, src, true, o, s);
}

int gr_observe(gr_fleet* f, double weight, const float* obs_wait, const float* obs_prefill,
               const float* obs_decode, void* hip_stream)
{
    if (!f || !(weight >= 0.0 && weight <= 1.0)) return GR_ERR_INVALID_ARG;
    if (!obs_wait && !obs_prefill && !obs_decode) return GR_OK;
    f->tables_current = false;      // (a blended table holds the smoothed status)
    // the capability order of the current tables carries the prefill estimate as it is now
    if (f->has_status && !f->ranks_current) {
        const int rc = launch_ranks(f, nullptr, static_cast<hipStream_t>(hip_stream));
        if (rc != GR_OK) return rc;
    }
    return launch_ema(f, weight, obs_wait, obs_prefill, obs_decode, static_cast<hipStream_t>(hip_stream));
}

int gr_set_blend(gr_fleet* f, double black_box_weight)
{
    if (!f || !(black_box_weight >= 0.0 && black_box_weight <= 1.0)) return GR_ERR_INVALID_ARG;
    if (black_box_weight > 0.0 && !(f->have_q && f->have_p && f->have_d)) return GR_ERR_NO_STATUS;
    f->lam = black_box_weight;
    f->tables_current = false;
    return GR_OK;
}

int gr_set_small_batch_pairs(gr_fleet* f, int64_t max_pairs)
{
    if (!f || max_pairs < 0) return GR_ERR_INVALID_ARG;
    f->small_batch_pairs = max_pairs;
    return GR_OK;
}

int gr_set_batch_cap(gr_fleet* f, const int32_t* cap)
{
    if (!f) return GR_ERR_INVALID_ARG;
    f->tables_current = false;
    if (!cap) { f->has_cap = false; return GR_OK; }
    for (int g = 0; g < f->n_inst; ++g)
        if (cap[g] < 1) return GR_ERR_INVALID_ARG;
    if (hipDeviceSynchronize() != hipSuccess) return GR_ERR_HIP;
    if (hipMemcpy(f->batch_cap, cap, sizeof(int) * f->n_inst, hipMemcpyHostToDevice) != hipSuccess) return GR_ERR_HIP;
    f->has_cap = true;
    return GR_OK;
}

int gr_device_status(gr_fleet* f, int32_t* out_bits)
{
    if (!f || !out_bits) return GR_ERR_INVALID_ARG;
    if (hipDeviceSynchronize() != hipSuccess) return GR_ERR_HIP;
    int v = 0;
    if (hipMemcpy(&v, f->counters, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return GR_ERR_HIP;
    *out_bits = v;
    return GR_OK;
}

int gr_profile_enable(gr_fleet* f, int32_t max_launches)
{
    if (!f || max_launches < 0) return GR_ERR_INVALID_ARG;
    Profiler& p = f->prof;
    if (hipDeviceSynchronize() != hipSuccess) return GR_ERR_HIP;
    p.ids.clear();
    p.on = max_launches > 0;
    p.ids.reserve((size_t)max_launches);
    while (p.events.size() < (size_t)max_launches * 2) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) { p.on = false; return GR_ERR_HIP; }
        p.events.push_back(e);
    }
    return GR_OK;
}

int gr_profile_select(gr_fleet* f, uint64_t kernel_mask)
{
    if (!f) return GR_ERR_INVALID_ARG;
    f->prof.mask = kernel_mask;
    return GR_OK;
}

int gr_profile_read(gr_fleet* f, int32_t n_kernels, double* total_ms, int64_t* launches)
{
    if (!f || n_kernels < 0 || (n_kernels > 0 && (!total_ms || !launches))) return GR_ERR_INVALID_ARG;
    if (hipDeviceSynchronize() != hipSuccess) return GR_ERR_HIP;
    Profiler& p = f->prof;
    for (int k = 0; k < n_kernels; ++k) { total_ms[k] = 0.0; launches[k] = 0; }
    for (size_t i = 0; i < p.ids.size(); ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.events[2 * i], p.events[2 * i + 1]) != hipSuccess) return GR_ERR_HIP;
        if (p.ids[i] < n_kernels) { total_ms[p.ids[i]] += ms; launches[p.ids[i]] += 1; }
    }
    p.ids.clear();
    return GR_OK;
}

int gr_profile_read_launches(gr_fleet* f, int32_t max_launches, int32_t* kernel_id, float* ms, int32_t* n_launches)
{
    if (!f || max_launches < 0 || !n_launches || (max_launches > 0 && (!kernel_id || !ms))) return GR_ERR_INVALID_ARG;
    if (hipDeviceSynchronize() != hipSuccess) return GR_ERR_HIP;
    Profiler& p = f->prof;
    const size_t n = p.ids.size() < (size_t)max_launches ? p.ids.size() : (size_t)max_launches;
    for (size_t i = 0; i < n; ++i) {
        if (hipEventElapsedTime(&ms[i], p.events[2 * i], p.events[2 * i + 1]) != hipSuccess) return GR_ERR_HIP;
        kernel_id[i] = p.ids[i];
    }
    *n_launches = (int32_t)n;
    p.ids.clear();
    return GR_OK;
}

int32_t gr_profile_kernel_count(void) { return kNumKernels; }

const char* gr_profile_kernel_name(int32_t id)
{
    return id >= 0 && id < kNumKernels ? kKernelNames[id] : "";
}

const char* gr_strerror(int code)
{
    switch (code) {
        case GR_OK: return "ok";
        case GR_ERR_INVALID_ARG: return "invalid argument";
        case GR_ERR_TOO_LARGE: return "size exceeds what the handle was created for or a hard limit";
        case GR_ERR_HIP: return "HIP runtime error";
        case GR_ERR_NO_STATUS: return "no status yet: gr_build_status / gr_risk_scan (or gr_observe) must come first";
        case GR_ERR_NOMEM: return "out of memory";
        default: return "unknown error";
    }
}

}  // extern "C"
