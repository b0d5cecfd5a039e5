// libgoodroute for gfx950: status build, pair scoring and risk scan of
// GoodServe's routing math (Eq. 2, Alg. 1, Sec. 3.4).  The C interface and the
// time model are described in goodroute.h; this file holds the kernels and the
// host entry points.
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
// more batch member with R = L: T(r,g) = q_g + delta*c0 + W_g(L) + beta*L + gamma*(c0*L + tri(L)).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <new>
#include <vector>

#include "goodroute.h"

namespace {

constexpr int kBlock = 256;
constexpr int kWave = 64;
constexpr int kWaves = kBlock / kWave;
constexpr int kMaxEntries = 8192;
constexpr int kMaxClasses = 64;

struct ClassCoef {
    double delta, alpha, beta, gamma;
};

}  // namespace

// Kernel ids for the optional per-kernel timing (gr_profile_*).
enum KernelId { kBuild = 0, kRank, kScoreRoute, kCompact, kScoreMigrate, kNumKernels };
static const char* const kKernelNames[kNumKernels] = {"k_build", "k_rank", "k_score<route>", "k_compact",
                                                      "k_score<migrate>"};

struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> events;  // pairs: start, stop
    std::vector<int> ids;            // kernel id of each recorded pair
};

struct gr_fleet {
    Profiler prof;
    int n_inst = 0, n_class = 0, max_entries = 0, max_len = 0;
    int64_t max_requests = 0;
    int64_t max_active = 0;
    int idx_bits = 0, key_bits = 0;
    int ncap = 0;       // entries the sort buffers hold (multiple of 64)
    int tstride = 0;    // table entries per instance, max_entries + 1
    int device = 0;
    bool has_status = false;
    // device memory
    ClassCoef* cls = nullptr;
    int* inst_class = nullptr;
    int* tabR = nullptr;     // [M][tstride] sorted remaining lengths, entry 0 = 0
    float* tabG = nullptr;   // [M][tstride] beta*Y_k + gamma*X_k
    float* tabS = nullptr;   // [M][tstride] S_{k+1}
    int* hN = nullptr;       // [M] entries per instance
    float* hQ = nullptr;     // [M] q_g
    double* hD = nullptr;    // [M] d_g
    int* rank = nullptr;     // [M]
    int* order = nullptr;    // [M] order[rank[g]] = g
    int* act_inst = nullptr; // [max_active] instance of each active request
    int* sel = nullptr;      // [max_active] indices of flagged requests
    int* counters = nullptr; // [0] flagged count, [1] GR_DEV_* bits
};

namespace {

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

// Lanes of the wave whose 8-bit digit equals this lane's, among `valid` lanes.
__device__ inline unsigned long long match_digit(unsigned digit, bool valid)
{
    unsigned long long m = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const bool bit = (digit >> b) & 1u;
        const unsigned long long bb = __ballot(bit);
        m &= bit ? bb : ~bb;
    }
    return m;
}

// ------------------------------------------------------------------ status build
struct BuildArgs {
    const int *act_off, *act_prompt, *act_gen, *act_rem;
    const int *q_off, *q_prompt, *q_len;
    const float* act_budget;  // null unless flags are wanted
    float *out_act_finish, *out_q_finish;
    double* out_d;
    uint8_t* out_flag;
    const ClassCoef* cls;
    const int* inst_class;
    int* tabR;
    float *tabG, *tabS;
    int* hN;
    float* hQ;
    double* hD;
    int* act_inst;
    int* counters;
    int64_t n_active, n_queued;
    int max_entries, ncap, tstride, idx_bits, key_bits, max_len;
};

// One stable counting pass of the LSD radix sort over an 8-bit digit.  Each
// wave owns a contiguous run of 64-entry chunks, so "wave, then chunk, then
// lane" is the entry order and per-wave digit counters keep the pass stable.
__device__ inline void radix_pass(const uint32_t* src, uint32_t* dst, uint32_t* cnt,
                                  uint32_t* wsum, int n, int shift, int c_begin, int c_end)
{
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) cnt[w * 256 + tid] = 0;
    __syncthreads();
    for (int c = c_begin; c < c_end; ++c) {
        const int i = c * kWave + lane;
        if (i < n) atomicAdd(&cnt[wave * 256 + ((src[i] >> shift) & 0xFFu)], 1u);
    }
    __syncthreads();
    {   // thread t owns digit t: exclusive scan over (digit, wave)
        uint32_t c[kWaves], tot = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) { c[w] = cnt[w * 256 + tid]; tot += c[w]; }
        const uint32_t incl = wave_incl_scan(tot);
        if (lane == kWave - 1) wsum[wave] = incl;
        __syncthreads();
        uint32_t base = incl - tot;
        for (int w = 0; w < wave; ++w) base += wsum[w];
#pragma unroll
        for (int w = 0; w < kWaves; ++w) { cnt[w * 256 + tid] = base; base += c[w]; }
    }
    __syncthreads();
    for (int c = c_begin; c < c_end; ++c) {
        const int i = c * kWave + lane;
        const bool valid = i < n;
        const uint32_t word = valid ? src[i] : 0u;
        const unsigned digit = (word >> shift) & 0xFFu;
        const unsigned long long m = match_digit(digit, valid);
        const unsigned long long below = m & ((1ull << lane) - 1ull);
        uint32_t old = 0;
        if (valid && below == 0ull) old = atomicAdd(&cnt[wave * 256 + digit], (uint32_t)__popcll(m));
        const int leader = valid ? __ffsll((long long)m) - 1 : lane;
        old = __shfl(old, leader, kWave);
        if (valid) dst[old + __popcll(below)] = word;
    }
    __syncthreads();
}

__global__ __launch_bounds__(kBlock) void k_build(BuildArgs a)
{
    extern __shared__ uint32_t smem[];
    uint32_t* keyA = smem;
    uint32_t* keyB = keyA + a.ncap;
    int* ctx = reinterpret_cast<int*>(keyB + a.ncap);
    uint32_t* cnt = reinterpret_cast<uint32_t*>(ctx + a.ncap);  // [kWaves][256]
    __shared__ long long red[kWaves][3];
    __shared__ uint32_t wsum[kWaves];

    const int g = blockIdx.x, tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
    const ClassCoef cc = a.cls[a.inst_class[g]];
    // offsets are clamped into the arrays, so broken CSR data cannot index outside them
    const int a0 = (int)min((int64_t)max(a.act_off[g], 0), a.n_active);
    const int q0 = (int)min((int64_t)max(a.q_off[g], 0), a.n_queued);
    int A = (int)max(min((int64_t)a.act_off[g + 1], a.n_active) - a0, (int64_t)0);
    int Q = (int)max(min((int64_t)a.q_off[g + 1], a.n_queued) - q0, (int64_t)0);
    int status = 0;
    if (A > a.max_entries) { A = a.max_entries; status |= GR_DEV_ENTRIES_DROPPED; }
    if (Q > a.max_entries - A) { Q = a.max_entries - A; status |= GR_DEV_ENTRIES_DROPPED; }
    const int N = A + Q;
    if (g == 0 && tid == 0) a.counters[0] = 0;

    // load: one sort word per entry = (remaining length << idx_bits) | entry index
    long long csum = 0, qsum = 0;
    for (int i = tid; i < N; i += kBlock) {
        int rem, c;
        if (i < A) {
            rem = a.act_rem[a0 + i];
            c = a.act_prompt[a0 + i] + a.act_gen[a0 + i];
            a.act_inst[a0 + i] = g;
        } else {
            rem = a.q_len[q0 + i - A];
            c = a.q_prompt[q0 + i - A];
            qsum += c;
        }
        if (rem < 0 || rem > a.max_len) { rem = min(max(rem, 0), a.max_len); status |= GR_DEV_LEN_CLAMPED; }
        keyA[i] = ((uint32_t)rem << a.idx_bits) | (uint32_t)i;
        ctx[i] = c;
        csum += c;
    }
    if (status) atomicOr(&a.counters[1], status);
    csum = wave_sum(csum);
    qsum = wave_sum(qsum);
    if (lane == 0) { red[wave][0] = csum; red[wave][1] = qsum; }
    __syncthreads();
    long long Ctot = 0, Qtot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) { Ctot += red[w][0]; Qtot += red[w][1]; }
    __syncthreads();

    const int nchunks = (N + kWave - 1) / kWave;
    const int cpw = (nchunks + kWaves - 1) / kWaves;
    const int c_begin = min(wave * cpw, nchunks), c_end = min(c_begin + cpw, nchunks);

    uint32_t *src = keyA, *dst = keyB;
    for (int shift = a.idx_bits; shift < a.idx_bits + a.key_bits; shift += 8) {
        radix_pass(src, dst, cnt, wsum, N, shift, c_begin, c_end);
        uint32_t* t = src; src = dst; dst = t;
    }

    // integer prefix sums over the sorted order: a reduction per wave, then a scan
    const uint32_t idx_mask = (1u << a.idx_bits) - 1u;
    long long sY = 0, sX = 0, sC = 0;
    for (int c = c_begin; c < c_end; ++c) {
        const int pos = c * kWave + lane;
        if (pos < N) {
            const uint32_t word = src[pos];
            const long long R = word >> a.idx_bits, cx = ctx[word & idx_mask];
            sY += R; sX += cx * R + R * (R - 1) / 2; sC += cx;
        }
    }
    sY = wave_sum(sY); sX = wave_sum(sX); sC = wave_sum(sC);
    if (lane == 0) { red[wave][0] = sY; red[wave][1] = sX; red[wave][2] = sC; }
    __syncthreads();
    long long cY = 0, cX = 0, cC = 0;   // carries: totals of the waves before this one
    for (int w = 0; w < wave; ++w) { cY += red[w][0]; cX += red[w][1]; cC += red[w][2]; }

    const double q = cc.delta * (double)Qtot;
    const size_t tb = (size_t)g * a.tstride;
    for (int c = c_begin; c < c_end; ++c) {
        const int pos = c * kWave + lane;
        const bool valid = pos < N;
        long long R = 0, cx = 0;
        uint32_t idx = 0;
        if (valid) {
            const uint32_t word = src[pos];
            R = word >> a.idx_bits; idx = word & idx_mask; cx = ctx[idx];
        }
        const long long triR = R * (R - 1) / 2;
        const long long Y = wave_incl_scan(R) + cY;
        const long long X = wave_incl_scan(cx * R + triR) + cX;
        const long long Pc = wave_incl_scan(cx) + cC;
        cY = __shfl(Y, kWave - 1, kWave); cX = __shfl(X, kWave - 1, kWave); cC = __shfl(Pc, kWave - 1, kWave);
        if (valid) {
            const int k = pos + 1;
            const long long S_next = Ctot - Pc, n_after = N - k;
            a.tabR[tb + k] = (int)R;
            a.tabG[tb + k] = (float)(cc.beta * (double)Y + cc.gamma * (double)X);
            a.tabS[tb + k] = (float)S_next;
            const long long I1 = Y + n_after * R;
            const long long I2 = X + R * S_next + n_after * triR;
            const double fin = q + fma(cc.gamma, (double)I2, fma(cc.beta, (double)I1, cc.alpha * (double)R));
            if (idx < (uint32_t)A) {
                a.out_act_finish[a0 + idx] = (float)fin;
                if (a.act_budget) a.out_flag[a0 + idx] = fin > (double)a.act_budget[a0 + idx];
            } else if (a.out_q_finish) {
                a.out_q_finish[q0 + idx - A] = (float)fin;
            }
        }
    }
    if (tid == 0) {
        a.tabR[tb] = 0; a.tabG[tb] = 0.f; a.tabS[tb] = (float)Ctot;
        a.hN[g] = N;
        a.hQ[g] = (float)q;
        const double d = fma(cc.gamma, (double)Ctot, fma(cc.beta, (double)N, cc.alpha));
        a.hD[g] = d;
        if (a.out_d) a.out_d[g] = d;
    }
}

// Capability order of Alg. 1's argmax d_g: rank 0 = largest d_g, equal d_g by index.
__global__ __launch_bounds__(kBlock) void k_rank(const double* d, int n_inst, int* rank, int* order,
                                                 int* out_rank)
{
    __shared__ double tile[kBlock];
    const int g = blockIdx.x * kBlock + threadIdx.x;
    const double dg = g < n_inst ? d[g] : 0.0;
    int r = 0;
    for (int base = 0; base < n_inst; base += kBlock) {
        const int h = base + threadIdx.x;
        tile[threadIdx.x] = h < n_inst ? d[h] : 0.0;
        __syncthreads();
        const int lim = min(kBlock, n_inst - base);
        for (int j = 0; j < lim; ++j) {
            const double dh = tile[j];
            r += (dh > dg) || (dh == dg && base + j < g);
        }
        __syncthreads();
    }
    if (g < n_inst) {
        rank[g] = r;
        order[r] = g;
        if (out_rank) out_rank[g] = r;
    }
}

// ------------------------------------------------------------------ pair scoring
struct ScoreArgs {
    // request batch (route) ...
    const int *ctx0, *pred_len;
    const float* budget;
    const int* exclude;
    // ... or flagged active requests (migration), through sel[0 .. *n_sel)
    const int *act_prompt, *act_gen, *act_rem, *act_inst, *sel, *n_sel;
    const float* act_budget;
    int64_t n_req;
    int *out_inst;
    float* out_slack;
    uint8_t* out_fallback;
    float* out_T;
    const ClassCoef* cls;
    const int* inst_class;
    const int* tabR;
    const float *tabG, *tabS;
    const int* hN;
    const float* hQ;
    const int *rank, *order;
    int n_inst, tstride, max_len;
};

template <bool kMigrate>
__global__ __launch_bounds__(kBlock) void k_score(ScoreArgs a)
{
    extern __shared__ uint32_t smem[];
    int* sR = reinterpret_cast<int*>(smem);
    float* sG = reinterpret_cast<float*>(sR + a.tstride);
    float* sS = sG + a.tstride;

    const int64_t n = kMigrate ? (int64_t)*a.n_sel : a.n_req;
    const int64_t r0 = (int64_t)blockIdx.x * kBlock;
    if (r0 >= n) return;
    const int64_t r = r0 + threadIdx.x;
    const bool live = r < n;
    int64_t out = r;
    int c0 = 1, L = 1, ex = -1;
    float D = 0.f;
    if (live) {
        if (kMigrate) {
            out = a.sel[r];
            c0 = a.act_prompt[out] + a.act_gen[out];
            L = a.act_rem[out];
            D = a.act_budget[out];
            ex = a.act_inst[out];
        } else {
            c0 = a.ctx0[r]; L = a.pred_len[r]; D = a.budget[r];
            ex = a.exclude ? a.exclude[r] : -1;
        }
    }
    L = min(max(L, 0), a.max_len);
    const float Lf = (float)L, c0f = (float)c0;
    const float triL = 0.5f * Lf * (Lf - 1.f);

    int best_rank = 0x7fffffff, min_g = -1;
    float best_T = 0.f, min_T = __builtin_inff();
    for (int g = 0; g < a.n_inst; ++g) {
        const int N = a.hN[g];
        const size_t tb = (size_t)g * a.tstride;
        __syncthreads();
        for (int k = threadIdx.x; k <= N; k += kBlock) {
            sR[k] = a.tabR[tb + k]; sG[k] = a.tabG[tb + k]; sS[k] = a.tabS[tb + k];
        }
        __syncthreads();
        // k = number of the instance's requests that end within L steps
        int lo = 0, hi = N;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (sR[mid] <= L) lo = mid; else hi = mid - 1;
        }
        const ClassCoef cc = a.cls[a.inst_class[g]];
        const float alpha = (float)cc.alpha, beta = (float)cc.beta, gamma = (float)cc.gamma,
                    delta = (float)cc.delta;
        const float n1 = (float)(N - lo + 1);
        float T = fmaf(Lf, fmaf(gamma, sS[lo] + c0f, beta * n1), sG[lo]);
        T = fmaf(gamma * n1, triL, T);
        T += fmaf(alpha, Lf, a.hQ[g]) + delta * c0f;
        if (a.out_T && live) a.out_T[out * a.n_inst + g] = T;
        if (g != ex) {
            const int rk = a.rank[g];
            if (T <= D && rk < best_rank) { best_rank = rk; best_T = T; }
            if (T < min_T) { min_T = T; min_g = g; }
        }
    }
    if (!live) return;
    const bool feas = best_rank != 0x7fffffff;
    const int pick = feas ? a.order[best_rank] : min_g;
    a.out_inst[out] = pick;
    a.out_slack[out] = pick >= 0 ? D - (feas ? best_T : min_T) : 0.f;
    if (a.out_fallback) a.out_fallback[out] = !feas;
}

// Flagged active requests -> dense index list; everyone else gets "no target".
__global__ __launch_bounds__(kBlock) void k_compact(const uint8_t* flag, int64_t n, int* sel, int* counter,
                                                    int* out_target, float* out_target_slack)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const bool f = i < n && flag[i];
    const unsigned long long m = __ballot(f);
    int base = 0;
    if (lane_id() == 0 && m) base = atomicAdd(counter, (int)__popcll(m));
    base = __shfl(base, 0, kWave);
    if (f) sel[base + __popcll(m & ((1ull << lane_id()) - 1ull))] = (int)i;
    else if (i < n) { out_target[i] = -1; out_target_slack[i] = 0.f; }
}

__global__ void k_copy_count(const int* counter, int* out) { *out = *counter; }

// ------------------------------------------------------------------ host side
// Brackets one kernel launch with a pair of events when timing is switched on.
struct ProfScope {
    Profiler& p;
    hipStream_t s;
    size_t slot = SIZE_MAX;
    ProfScope(gr_fleet* f, int id, hipStream_t stream) : p(f->prof), s(stream)
    {
        if (!p.on || (p.ids.size() + 1) * 2 > p.events.size()) return;
        slot = p.ids.size();
        p.ids.push_back(id);
        (void)hipEventRecord(p.events[2 * slot], s);
    }
    ~ProfScope()
    {
        if (slot != SIZE_MAX) (void)hipEventRecord(p.events[2 * slot + 1], s);
    }
};

int bits_for(int64_t v)
{
    int b = 0;
    while ((int64_t(1) << b) <= v) ++b;
    return b;
}

template <typename T>
bool dev_alloc(T** p, size_t n)
{
    return hipMalloc(reinterpret_cast<void**>(p), (n ? n : 1) * sizeof(T)) == hipSuccess;
}

size_t build_lds_bytes(const gr_fleet* f) { return (size_t)f->ncap * 12 + kWaves * 256 * 4; }

int launch_build(gr_fleet* f, const int32_t* act_off, const int32_t* act_prompt, const int32_t* act_gen,
                 const int32_t* act_rem, const int32_t* q_off, const int32_t* q_prompt, const int32_t* q_len,
                 const float* act_budget, float* out_act_finish, float* out_q_finish, double* out_d,
                 int32_t* out_rank, uint8_t* out_flag, int64_t n_active, int64_t n_queued, hipStream_t s)
{
    BuildArgs b{};
    b.n_active = n_active; b.n_queued = n_queued;
    b.act_off = act_off; b.act_prompt = act_prompt; b.act_gen = act_gen; b.act_rem = act_rem;
    b.q_off = q_off; b.q_prompt = q_prompt; b.q_len = q_len;
    b.act_budget = act_budget;
    b.out_act_finish = out_act_finish; b.out_q_finish = out_q_finish; b.out_d = out_d; b.out_flag = out_flag;
    b.cls = f->cls; b.inst_class = f->inst_class;
    b.tabR = f->tabR; b.tabG = f->tabG; b.tabS = f->tabS;
    b.hN = f->hN; b.hQ = f->hQ; b.hD = f->hD; b.act_inst = f->act_inst; b.counters = f->counters;
    b.max_entries = f->max_entries; b.ncap = f->ncap; b.tstride = f->tstride;
    b.idx_bits = f->idx_bits; b.key_bits = f->key_bits; b.max_len = f->max_len;
    {
        ProfScope ps(f, kBuild, s);
        hipLaunchKernelGGL(k_build, dim3(f->n_inst), dim3(kBlock), build_lds_bytes(f), s, b);
    }
    {
        ProfScope ps(f, kRank, s);
        hipLaunchKernelGGL(k_rank, dim3((f->n_inst + kBlock - 1) / kBlock), dim3(kBlock), 0, s,
                           f->hD, f->n_inst, f->rank, f->order, out_rank);
    }
    if (hipGetLastError() != hipSuccess) return GR_ERR_HIP;
    f->has_status = true;
    return GR_OK;
}

void fill_score_tables(const gr_fleet* f, ScoreArgs& a)
{
    a.cls = f->cls; a.inst_class = f->inst_class;
    a.tabR = f->tabR; a.tabG = f->tabG; a.tabS = f->tabS;
    a.hN = f->hN; a.hQ = f->hQ; a.rank = f->rank; a.order = f->order;
    a.n_inst = f->n_inst; a.tstride = f->tstride; a.max_len = f->max_len;
}

bool check_sizes(const gr_fleet* f, int64_t n_active, int64_t n_queued)
{
    return n_active <= f->max_active && n_queued <= f->max_active;
}

}  // namespace

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
    if (n_class > kMaxClasses || max_entries_per_inst > kMaxEntries) return GR_ERR_TOO_LARGE;
    for (int c = 0; c < n_class; ++c)
        if (!(delta[c] >= 0) || !(alpha[c] >= 0) || !(beta[c] >= 0) || !(gamma[c] >= 0))
            return GR_ERR_INVALID_ARG;
    for (int g = 0; g < n_inst; ++g)
        if (inst_class[g] < 0 || inst_class[g] >= n_class) return GR_ERR_INVALID_ARG;
    const int idx_bits = bits_for(max_entries_per_inst > 0 ? max_entries_per_inst - 1 : 0);
    const int key_bits = bits_for(max_len);
    if (idx_bits + key_bits > 32) return GR_ERR_TOO_LARGE;

    gr_fleet* f = new (std::nothrow) gr_fleet;
    if (!f) return GR_ERR_NOMEM;
    f->n_inst = n_inst; f->n_class = n_class;
    f->max_entries = max_entries_per_inst; f->max_len = max_len; f->max_requests = max_requests;
    f->max_active = (int64_t)n_inst * max_entries_per_inst;
    f->idx_bits = idx_bits > 0 ? idx_bits : 1; f->key_bits = key_bits;
    f->ncap = ((max_entries_per_inst + kWave - 1) / kWave) * kWave;
    if (f->ncap == 0) f->ncap = kWave;
    f->tstride = max_entries_per_inst + 1;
    if (hipGetDevice(&f->device) != hipSuccess) { delete f; return GR_ERR_HIP; }

    const size_t tab = (size_t)n_inst * f->tstride;
    bool ok = dev_alloc(&f->cls, n_class) && dev_alloc(&f->inst_class, n_inst) &&
              dev_alloc(&f->tabR, tab) && dev_alloc(&f->tabG, tab) && dev_alloc(&f->tabS, tab) &&
              dev_alloc(&f->hN, n_inst) && dev_alloc(&f->hQ, n_inst) && dev_alloc(&f->hD, n_inst) &&
              dev_alloc(&f->rank, n_inst) && dev_alloc(&f->order, n_inst) &&
              dev_alloc(&f->act_inst, f->max_active) && dev_alloc(&f->sel, f->max_active) &&
              dev_alloc(&f->counters, 2);
    if (!ok) { gr_destroy(f); return GR_ERR_NOMEM; }

    ClassCoef* host = static_cast<ClassCoef*>(malloc(sizeof(ClassCoef) * n_class));
    if (!host) { gr_destroy(f); return GR_ERR_NOMEM; }
    for (int c = 0; c < n_class; ++c) host[c] = ClassCoef{delta[c], alpha[c], beta[c], gamma[c]};
    hipError_t e1 = hipMemcpy(f->cls, host, sizeof(ClassCoef) * n_class, hipMemcpyHostToDevice);
    hipError_t e2 = hipMemcpy(f->inst_class, inst_class, sizeof(int) * n_inst, hipMemcpyHostToDevice);
    hipError_t e3 = hipMemset(f->counters, 0, 2 * sizeof(int));
    free(host);
    if (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess) { gr_destroy(f); return GR_ERR_HIP; }

    const size_t lds = build_lds_bytes(f) > (size_t)f->tstride * 12 ? build_lds_bytes(f) : (size_t)f->tstride * 12;
    if (lds > 160 * 1024) { gr_destroy(f); return GR_ERR_TOO_LARGE; }
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_build),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)build_lds_bytes(f)) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void*>(k_score<false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, f->tstride * 12) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void*>(k_score<true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, f->tstride * 12) != hipSuccess) {
        gr_destroy(f);
        return GR_ERR_HIP;
    }
    *out = f;
    return GR_OK;
}

int gr_destroy(gr_fleet* f)
{
    if (!f) return GR_OK;
    (void)hipDeviceSynchronize();
    void* ptrs[] = {f->cls, f->inst_class, f->tabR, f->tabG, f->tabS, f->hN, f->hQ, f->hD,
                    f->rank, f->order, f->act_inst, f->sel, f->counters};
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
    if (!f || !act_off || !q_off || n_active < 0 || n_queued < 0) return GR_ERR_INVALID_ARG;
    if (n_active > 0 && (!act_prompt || !act_gen || !act_rem || !out_act_finish)) return GR_ERR_INVALID_ARG;
    if (n_queued > 0 && (!q_prompt || !q_len)) return GR_ERR_INVALID_ARG;
    if (!check_sizes(f, n_active, n_queued)) return GR_ERR_TOO_LARGE;
    return launch_build(f, act_off, act_prompt, act_gen, act_rem, q_off, q_prompt, q_len, nullptr,
                        out_act_finish, out_q_finish, out_d, out_rank, nullptr, n_active, n_queued,
                        static_cast<hipStream_t>(hip_stream));
}

int gr_score_route(gr_fleet* f, int64_t n_req, const int32_t* ctx0, const int32_t* pred_len,
                   const float* budget, const int32_t* exclude_inst, int32_t* out_inst,
                   float* out_slack, uint8_t* out_fallback, float* out_T, void* hip_stream)
{
    if (!f || n_req < 0) return GR_ERR_INVALID_ARG;
    if (!f->has_status) return GR_ERR_NO_STATUS;
    if (n_req == 0) return GR_OK;
    if (!ctx0 || !pred_len || !budget || !out_inst || !out_slack) return GR_ERR_INVALID_ARG;
    if (n_req > f->max_requests) return GR_ERR_TOO_LARGE;
    ScoreArgs a{};
    a.ctx0 = ctx0; a.pred_len = pred_len; a.budget = budget; a.exclude = exclude_inst;
    a.n_req = n_req;
    a.out_inst = out_inst; a.out_slack = out_slack; a.out_fallback = out_fallback; a.out_T = out_T;
    fill_score_tables(f, a);
    {
        ProfScope ps(f, kScoreRoute, static_cast<hipStream_t>(hip_stream));
        hipLaunchKernelGGL(k_score<false>, dim3((unsigned)((n_req + kBlock - 1) / kBlock)), dim3(kBlock),
                           (size_t)f->tstride * 12, static_cast<hipStream_t>(hip_stream), a);
    }
    return hipGetLastError() == hipSuccess ? GR_OK : GR_ERR_HIP;
}

int gr_risk_scan(gr_fleet* f, const int32_t* act_off, const int32_t* act_prompt,
                 const int32_t* act_gen, const int32_t* act_rem_refreshed, int64_t n_active,
                 const int32_t* q_off, const int32_t* q_prompt, const int32_t* q_len,
                 int64_t n_queued, const float* act_budget, uint8_t* out_flag, float* out_finish,
                 int32_t* out_target, float* out_target_slack, int32_t* out_n_flagged,
                 void* hip_stream)
{
    if (!f || !act_off || !q_off || n_active < 0 || n_queued < 0) return GR_ERR_INVALID_ARG;
    if (n_active > 0 && (!act_prompt || !act_gen || !act_rem_refreshed || !act_budget || !out_flag ||
                         !out_finish || !out_target || !out_target_slack))
        return GR_ERR_INVALID_ARG;
    if (n_queued > 0 && (!q_prompt || !q_len)) return GR_ERR_INVALID_ARG;
    if (!check_sizes(f, n_active, n_queued)) return GR_ERR_TOO_LARGE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int rc = launch_build(f, act_off, act_prompt, act_gen, act_rem_refreshed, q_off, q_prompt, q_len,
                          act_budget, out_finish, nullptr, nullptr, nullptr, out_flag, n_active, n_queued, s);
    if (rc != GR_OK) return rc;
    if (n_active > 0) {
        const unsigned blocks = (unsigned)((n_active + kBlock - 1) / kBlock);
        {
            ProfScope ps(f, kCompact, s);
            hipLaunchKernelGGL(k_compact, dim3(blocks), dim3(kBlock), 0, s, out_flag, n_active, f->sel,
                               f->counters, out_target, out_target_slack);
        }
        ScoreArgs a{};
        a.act_prompt = act_prompt; a.act_gen = act_gen; a.act_rem = act_rem_refreshed;
        a.act_inst = f->act_inst; a.sel = f->sel; a.n_sel = f->counters; a.act_budget = act_budget;
        a.out_inst = out_target; a.out_slack = out_target_slack;
        fill_score_tables(f, a);
        ProfScope ps(f, kScoreMigrate, s);
        hipLaunchKernelGGL(k_score<true>, dim3(blocks), dim3(kBlock), (size_t)f->tstride * 12, s, a);
    }
    if (out_n_flagged) hipLaunchKernelGGL(k_copy_count, dim3(1), dim3(1), 0, s, f->counters, out_n_flagged);
    return hipGetLastError() == hipSuccess ? GR_OK : GR_ERR_HIP;
}

int gr_device_status(gr_fleet* f, int32_t* out_bits)
{
    if (!f || !out_bits) return GR_ERR_INVALID_ARG;
    if (hipDeviceSynchronize() != hipSuccess) return GR_ERR_HIP;
    int v = 0;
    if (hipMemcpy(&v, f->counters + 1, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return GR_ERR_HIP;
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
        case GR_ERR_NO_STATUS: return "no status built yet: call gr_build_status or gr_risk_scan first";
        case GR_ERR_NOMEM: return "out of memory";
        default: return "unknown error";
    }
}

}  // extern "C"
