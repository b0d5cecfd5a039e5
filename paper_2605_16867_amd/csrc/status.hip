// Status build (step 1 of the path): per instance, an LDS radix sort of the
// remaining lengths, three integer prefix sums over the sorted order, and from
// them the finish time of every held request (Sec. 3.4's "expected finish
// time"), q_g and d_g of Eq. 2, and the instance table used for scoring; then
// the capability order of Alg. 1's argmax d_g.
#include "common.h"

namespace gr {
namespace {

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
    double* hQ;
    double* hD;
    int* act_inst;
    int* rank_acc;
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
    if (status) atomicOr(&a.counters[0], status);
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
        a.hQ[g] = q;
        a.rank_acc[g] = 0;
        const double d = fma(cc.gamma, (double)Ctot, fma(cc.beta, (double)N, cc.alpha));
        a.hD[g] = d;
        if (a.out_d) a.out_d[g] = d;
    }
}

// Capability order of Alg. 1's argmax d_g: rank 0 = largest d_g, equal d_g by
// index.  rank_g = #{h : d_h > d_g} + #{h < g : d_h = d_g}, counted over tiles of
// 64 instances x 256 competitors and added up with atomics.
__global__ __launch_bounds__(kBlock) void k_rank_count(const double* __restrict__ d, int n_inst,
                                                       int* __restrict__ rank_acc)
{
    __shared__ double comp[kBlock];
    const int tid = threadIdx.x;
    const int g = blockIdx.x * kWave + (tid & (kWave - 1));
    const int h0 = blockIdx.y * kBlock;
    comp[tid] = h0 + tid < n_inst ? d[h0 + tid] : 0.0;
    __syncthreads();
    if (g >= n_inst) return;
    const double dg = d[g];
    const int part = tid / kWave;                 // which 64 of the 256 competitors
    const int lim = min(kWave, n_inst - h0 - part * kWave);
    int r = 0;
    for (int j = 0; j < lim; ++j) {
        const double dh = comp[part * kWave + j];
        r += (dh > dg) || (dh == dg && h0 + part * kWave + j < g);
    }
    if (r) atomicAdd(&rank_acc[g], r);
}

__global__ __launch_bounds__(kBlock) void k_rank_final(const int* __restrict__ rank_acc, int n_inst, int m_pad,
                                                       const ClassCoef* __restrict__ cls,
                                                       const int* __restrict__ inst_class,
                                                       int* __restrict__ rank, int* __restrict__ order,
                                                       float2* __restrict__ posK, int* __restrict__ out_rank)
{
    const int g = blockIdx.x * kBlock + threadIdx.x;
    if (g < n_inst) {
        const int r = rank_acc[g];
        const ClassCoef cc = cls[inst_class[g]];
        rank[g] = r;
        order[r] = g;
        posK[r] = make_float2((float)cc.delta, (float)cc.gamma);
        if (out_rank) out_rank[g] = r;
    } else if (g < m_pad) {
        order[g] = -1;     // positions past the last instance
        posK[g] = make_float2(0.f, 0.f);
    }
}

}  // namespace

size_t status_lds_bytes(const gr_fleet* f) { return (size_t)f->ncap * 12 + kWaves * 256 * 4; }

int status_prepare(gr_fleet* f)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(k_build),
                               hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)status_lds_bytes(f)) == hipSuccess ? GR_OK : GR_ERR_HIP;
}

int launch_status(gr_fleet* f, const StatusIn& in, hipStream_t s)
{
    BuildArgs b{};
    b.act_off = in.act_off; b.act_prompt = in.act_prompt; b.act_gen = in.act_gen; b.act_rem = in.act_rem;
    b.q_off = in.q_off; b.q_prompt = in.q_prompt; b.q_len = in.q_len;
    b.act_budget = in.act_budget;
    b.out_act_finish = in.out_act_finish; b.out_q_finish = in.out_q_finish;
    b.out_d = in.out_d; b.out_flag = in.out_flag;
    b.cls = f->cls; b.inst_class = f->inst_class;
    b.tabR = f->tabR; b.tabG = f->tabG; b.tabS = f->tabS;
    b.hN = f->hN; b.hQ = f->hQ; b.hD = f->hD; b.act_inst = f->act_inst;
    b.rank_acc = f->rank_acc; b.counters = f->counters;
    b.n_active = in.n_active; b.n_queued = in.n_queued;
    b.max_entries = f->max_entries; b.ncap = f->ncap; b.tstride = f->tstride;
    b.idx_bits = f->idx_bits; b.key_bits = f->key_bits; b.max_len = f->max_len;
    const int M = f->n_inst;
    {
        ProfScope ps(f, kBuild, s);
        hipLaunchKernelGGL(k_build, dim3(M), dim3(kBlock), status_lds_bytes(f), s, b);
    }
    {
        ProfScope ps(f, kRankCount, s);
        hipLaunchKernelGGL(k_rank_count, dim3((M + kWave - 1) / kWave, (M + kBlock - 1) / kBlock),
                           dim3(kBlock), 0, s, f->hD, M, f->rank_acc);
    }
    {
        ProfScope ps(f, kRankFinal, s);
        hipLaunchKernelGGL(k_rank_final, dim3((f->m_pad + kBlock - 1) / kBlock), dim3(kBlock), 0, s,
                           f->rank_acc, M, f->m_pad, f->cls, f->inst_class, f->rank, f->order, f->posK,
                           in.out_rank);
    }
    if (hipGetLastError() != hipSuccess) return GR_ERR_HIP;
    f->has_status = true;
    return GR_OK;
}

}  // namespace gr
