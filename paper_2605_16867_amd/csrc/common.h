// Internal declarations shared by the source files of libgoodroute (gfx950).
// The public interface and the time model are in goodroute.h.
//
// Closed form used throughout.  Let instance g hold N requests with remaining
// lengths R_i and contexts c_i.  Under continuous batching with step time
// alpha + beta*B + gamma*C, the time of its next L steps is
//     W_g(L) = alpha*L + beta*sum_i min(R_i,L) + gamma*sum_i [c_i*min(R_i,L) + tri(min(R_i,L))]
// with tri(x) = x(x-1)/2, because request i is in the batch for min(R_i,L) of
// those steps and its context at its s-th step is c_i + s - 1.  With the
// requests sorted by R and k = #{i : R_i <= L} this is
//     W_g(L) = alpha*L + beta*(Y_k + (N-k)*L) + gamma*(X_k + L*S_{k+1} + (N-k)*tri(L))
//     Y_k = sum_{i<=k} R_i,  X_k = sum_{i<=k} (c_i*R_i + tri(R_i)),  S_{k+1} = sum_{i>k} c_i,
// three integer prefix sums, exact in 64-bit.  A request r routed to g is one
// more batch member with R = L, so Eq. 2 reads
//     T(r,g) = q_g + delta*c0 + W_g(L) + beta*L + gamma*(c0*L + tri(L))
//            = E_g(L) + c0 * kappa_g(L),
//     E_g(L)     = q_g + W_g(L) + beta*L + gamma*tri(L)      (instance and length only)
//     kappa_g(L) = delta + gamma*L.
// On the segment R_k <= L < R_{k+1}, with n = N - k requests still running:
//     E_g(L) = [q_g + beta*Y_k + gamma*X_k] + L*[alpha + beta*(n+1) + gamma*S_{k+1}] + tri(L)*gamma*(n+1).
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <vector>

#include "goodroute.h"

namespace gr {

constexpr int kBlock = 256;
constexpr int kWave = 64;
constexpr int kWaves = kBlock / kWave;
constexpr int kMaxEntries = 2048;
constexpr int kMaxClasses = 64;
constexpr int kMaxLen = 32767;     // one LDS counter per length in the grouping kernels
constexpr int kTileReq = 32;       // requests of one length scored together by one wave
constexpr int kGroupBlock = 1024;  // threads per workgroup of the grouping kernels (their cost is the pass over the LDS bins)
constexpr int kMemoU = 256;        // lengths per pass of a workgroup of the memo kernel
constexpr int kDirectMax = 4096;   // most requests of a batch scored pair by pair, without grouping
constexpr int kMemoP = 16;         // instances (waves) per workgroup of the memo kernel

struct ClassCoef {
    double delta, alpha, beta, gamma;
};

// One request in grouped order.
struct ReqRec {
    float c0;   // tokens to prefill
    float D;    // budget
    int pex;    // excluded instance as a position in capability order, -1 none
    int orig;   // index in the caller's arrays
};

// Where a batch of requests comes from: the caller's arrays (routing) or the
// flagged active requests (migration).
struct ReqSrc {
    const int *ctx0, *pred_len;
    const float* budget;
    const int* exclude;
    const int *act_prompt, *act_gen, *act_rem, *act_inst;
    const uint8_t* flag;
    const float* act_budget;
    int64_t n;
};

struct ScoreOut {
    int* inst;
    float* slack;
    uint8_t* fallback;   // may be null
    float* T;            // may be null: every pair's latency
    int* n_selected;     // may be null: number of requests scored
};

enum KernelId {
    kBuild = 0, kRankCount, kRankFinal, kHistRoute, kScanRoute, kGroupRoute, kTileRoute,
    kHistMigrate, kScanMigrate, kGroupMigrate, kTileMigrate, kHitsRoute, kDirect, kDirectFinish,
    kNumKernels
};

struct Profiler {
    bool on = false;
    uint64_t mask = ~0ull;           // bit k: launches of kernel id k are timed
    std::vector<hipEvent_t> events;  // pairs: start, stop
    std::vector<int> ids;            // kernel id of each recorded pair
};

struct StatusIn {
    const int *act_off, *act_prompt, *act_gen, *act_rem;
    const int *q_off, *q_prompt, *q_len;
    const float* act_budget;  // null unless flags are wanted
    int64_t n_active, n_queued;
    float *out_act_finish, *out_q_finish;
    double* out_d;
    int* out_rank;
    uint8_t* out_flag;
    int use_pending = 0;      // count the requests routed since the caller's status (feedback routing)
    int only_touched = 0;     // rebuild only the instances that have been given requests since the last build
};

}  // namespace gr

struct gr_fleet {
    gr::Profiler prof;
    int n_inst = 0, n_class = 0, max_entries = 0, max_len = 0;
    int64_t max_requests = 0;
    int64_t max_active = 0;
    int64_t req_cap = 0;   // requests one scoring pass may hold
    int epl = 0;           // sort words per lane of the status build: 1, 2, 4 .. 32
    int cap = 0;           // 64 * epl >= max_entries: table entries per instance
    int m_pad = 0;         // instances rounded up to a multiple of 128 (two blocks of 64 positions)
    int bins = 0;          // max_len + 1
    int64_t row_cap = 0;   // rows of the memo table
    int device = 0;
    bool has_status = false;
    // smoothed black-box status (Sec. 3.3) and the weight it is blended in with
    double lam = 0.0;        // as set; takes effect at the next status build
    double lam_built = 0.0;  // the weight the current tables were built with
    bool have_q = false, have_p = false, have_d = false;
    double *emaQ = nullptr, *emaP = nullptr, *emaD = nullptr;   // [M] each
    // device memory: fleet description
    gr::ClassCoef* cls = nullptr;
    int* inst_class = nullptr;
    // per-instance tables written by the status build
    // E_g(L) = Gq + L*H + tri(L)*gamma*(n+1) on the segment after the k shortest requests (n still running)
    uint16_t* tabR = nullptr; // [M][cap] remaining lengths, ascending; 0xFFFF past the last entry
    float2* tabGH = nullptr;  // [M][cap] (Gq, H) of segment k = index + 1
    float2* headGH = nullptr; // [M] (Gq, H) of segment 0: (q_g, alpha + beta*(N+1) + gamma*sum of contexts)
    int* hN = nullptr;       // [M] entries per instance
    double* hD = nullptr;    // [M] d_g
    int* rank_acc = nullptr; // [M] partial counts of the rank kernels
    int* rank = nullptr;     // [M]
    int* order = nullptr;    // [m_pad] order[rank[g]] = g
    float2* posK = nullptr;  // [m_pad] (delta, gamma) of the instance at each position of the capability order
    int* act_inst = nullptr; // [max_active] instance of each active request
    // feedback routing: the caller's last status inputs, and the requests routed since, per instance
    gr::StatusIn last_in{};
    int* pend_cnt = nullptr;      // [M]
    int* commit_mark = nullptr;   // [M] 1: chosen by a request of the chunk being committed (all zero between commits)
    int* pend_prompt = nullptr;   // [M][cap]
    int* pend_len = nullptr;      // [M][cap]
    float* scratch_finish = nullptr;  // [max_active] finish times of rebuilds nobody asked to see
    int* batch_cap = nullptr;     // [M] requests that may decode together on each instance
    bool has_cap = false;
    int* counters = nullptr; // [1] GR_DEV_* bits
    // scoring workspace
    int* len_cnt = nullptr;   // [bins] requests per length; all zero between calls
    int* len_base = nullptr;  // [bins] next free slot of each length in grouped order
    int* row_len = nullptr;   // [row_cap] the distinct lengths, ascending
    int* row_off = nullptr;   // [row_cap+1] first request of each distinct length
    int* tile_off = nullptr;  // [row_cap+1] first tile of each distinct length
    int* len_row = nullptr;   // [bins] row of each length present in the last batch
    int* len_ceil = nullptr;  // [bins] rows shorter than each length = the first row at least that long
    int* totals = nullptr;    // [4] requests, distinct lengths, tiles
    gr::ReqRec* recs = nullptr;  // [req_cap] requests in grouped order
    float* memo = nullptr;       // [row_cap][m_pad] E per distinct length and position
    int* tile_row = nullptr;     // [req_cap / kTileReq + row_cap + 1] the row of every tile
    float* grp_min = nullptr;    // [m_pad / kMemoP][row_cap] least E of each run of kMemoP positions, per row
    float2* grp_k = nullptr;     // [m_pad / kMemoP] least delta and least gamma of each run
    bool tables_current = false;   // every instance's table is from the last inputs, blend weight and caps
    bool ranks_current = false;    // rank, order and posK belong to the current d_g (else the next scoring pass makes them)
    int* pend_touched = nullptr;   // [M] 1: given requests since its table was built
    int64_t small_batch_pairs = int64_t(1) << 18;   // largest batch, in pairs, scored pair by pair
    unsigned long long* direct_best = nullptr;   // [2][kDirectMax] running selections of a small batch (all ones between calls)
};

namespace gr {

// Brackets one kernel launch with a pair of events when timing is switched on.
struct ProfScope {
    Profiler& p;
    hipStream_t s;
    size_t slot = SIZE_MAX;
    ProfScope(gr_fleet* f, int id, hipStream_t stream) : p(f->prof), s(stream)
    {
        if (!p.on || !((p.mask >> id) & 1ull) || (p.ids.size() + 1) * 2 > p.events.size()) return;
        slot = p.ids.size();
        p.ids.push_back(id);
        (void)hipEventRecord(p.events[2 * slot], s);
    }
    ~ProfScope()
    {
        if (slot != SIZE_MAX) (void)hipEventRecord(p.events[2 * slot + 1], s);
    }
};


// What the two steps of the capability order need (Alg. 1's argmax d_g: rank 0 = largest d_g,
// equal d_g by index).  They run as kernels of their own or as extra workgroups of the first two
// kernels of a scoring pass (see launch_score).
struct RankArgs {
    const double* d;        // [M] d_g
    int* rank_acc;          // [M] partial counts, zero before the count and again after the final step
    const ClassCoef* cls;
    const int* inst_class;
    const double* emaP;
    double lam;
    int *rank, *order;
    float2* posK;
    int* out_rank;          // may be null
    int n_inst, m_pad;
};

// status.hip
int status_prepare();
int launch_ranks(gr_fleet* f, int* out_rank, hipStream_t s);
RankArgs rank_args(const gr_fleet* f, int* out_rank);
int launch_status(gr_fleet* f, const StatusIn& in, hipStream_t s);
int launch_commit(gr_fleet* f, int64_t n, const int* inst, const int* ctx0, const int* pred_len, hipStream_t s);
int launch_ema(gr_fleet* f, double w, const float* s_q, const float* s_p, const float* s_d, hipStream_t s);

// score.hip
size_t score_lds_bytes(const gr_fleet* f);
int score_prepare(gr_fleet* f);
int launch_score(gr_fleet* f, const ReqSrc& src, bool migrate, const ScoreOut& out, hipStream_t s,
                 bool small_batch_ok = false);
int static_scratch(int device, unsigned long long** out);
int launch_score_static(gr_fleet* f, const ReqSrc& src, const ScoreOut& out, hipStream_t s);
int launch_hits(gr_fleet* f, const ReqSrc& src, const int* hit_off, const int* hit_inst, const int* hit_len,
                int64_t n_hits, const ScoreOut& out, hipStream_t s);

// ------------------------------------------------------------------ wave helpers
__device__ inline int lane_id() { return threadIdx.x & (kWave - 1); }

template <typename T>
__device__ inline T wave_sum(T v)
{
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

template <typename T>
__device__ inline T wave_incl_scan(T v)
{
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        T o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

// Inclusive prefix sum of a 32-bit value over the wave without going through
// LDS: inside each row of 16 lanes by shifts of 1, 2, 4, 8 (a lane without a
// source adds 0), then lane 15 of rows 0 and 2 onto rows 1 and 3, then lane 31
// onto rows 2 and 3.
__device__ inline int wave_incl_scan_i32(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2, 3
    return v;
}

// rank_g = #{h : d_h > d_g} + #{h < g : d_h = d_g}, counted over tiles of 64 instances x kThreads
// competitors (tile `bx` of the instances, tile `by` of the competitors) and added up with
// atomics.  `comp`: kThreads doubles of LDS.  Every thread of the workgroup must call it.
template <int kThreads>
__device__ inline void rank_count_tile(const RankArgs& a, int bx, int by, double* comp)
{
    const int tid = threadIdx.x;
    const int g = bx * kWave + (tid & (kWave - 1));
    const int h0 = by * kThreads;
    comp[tid] = h0 + tid < a.n_inst ? a.d[h0 + tid] : 0.0;
    __syncthreads();
    if (g >= a.n_inst) return;
    const double dg = a.d[g];
    const int part = tid / kWave;                 // which 64 of the competitors
    const int lim = min(kWave, a.n_inst - h0 - part * kWave);
    int r = 0;
    for (int j = 0; j < lim; ++j) {
        const double dh = comp[part * kWave + j];
        r += (dh > dg) || (dh == dg && h0 + part * kWave + j < g);
    }
    if (r) atomicAdd(&a.rank_acc[g], r);
}

// The counts are complete: rank, order[rank] = g and the prefill coefficients per position.
__device__ inline void rank_final_item(const RankArgs& a, int g)
{
    if (g < a.n_inst) {
        const int r = a.rank_acc[g];
        a.rank_acc[g] = 0;
        if ((unsigned)r >= (unsigned)a.n_inst) return;      // (counts are below n_inst by construction; never index past the tables)
        const ClassCoef cc = a.cls[a.inst_class[g]];
        a.rank[g] = r;
        a.order[r] = g;
        // T = E + c0 * (delta + gamma * L); blended: keep * that + lam * p_g * c0
        const double keep = 1.0 - a.lam;
        a.posK[r] = a.lam != 0.0 ? make_float2((float)(keep * cc.delta + a.lam * a.emaP[g]), (float)(keep * cc.gamma))
                                 : make_float2((float)cc.delta, (float)cc.gamma);
        if (a.out_rank) a.out_rank[g] = r;
    } else if (g < a.m_pad) {
        a.order[g] = -1;     // positions past the last instance
        a.posK[g] = make_float2(0.f, 0.f);
    }
}

}  // namespace gr
