// Status build (step 1 of the path): per instance, a sort of the remaining
// lengths, three exact prefix sums over the sorted order, and from them the
// finish time of every held request (Sec. 3.4's "expected finish time"), q_g
// and d_g of Eq. 2, and the instance table used for scoring; then the
// capability order of Alg. 1's argmax d_g.
//
// One wave per instance (two or four when the fleet has fewer instances than
// the chip takes waves), everything in registers: a wave holds 64 * kEPL sort
// words (remaining length in the high bits, entry index in the low bits, so
// all words differ and the order is stable), kEPL consecutive positions of the
// sorted order per lane.  A bitonic network sorts them: exchanges inside a lane
// are a min/max pair, exchanges between lanes fetch the partner's word (a DPP
// move inside a row of 16 lanes where a pattern exists, else the LDS crossbar)
// and keep the smaller or the larger of the two with one median-of-three
// against 0 or 0xFFFFFFFF.  No atomics; barriers only between the waves that
// share an instance.
#include "common.h"

namespace gr {
namespace {

struct BuildArgs {
    const int *act_off, *act_prompt, *act_gen, *act_rem;
    const int *q_off, *q_prompt, *q_len;
    const float* act_budget;  // null unless flags are wanted
    float *out_act_finish, *out_q_finish;
    double* out_d;
    uint8_t* out_flag;
    const ClassCoef* cls;
    const int* inst_class;
    uint16_t* tabR;
    float2* tabGH;
    float2* headGH;
    int* hN;
    double* hD;
    int* act_inst;
    int* rank_acc;
    int* counters;
    int64_t n_active, n_queued;
    int n_inst, max_entries, max_len;
    // requests routed since the caller's status (feedback routing): per instance, queued behind the queue
    int* pend_cnt;
    const int *pend_prompt, *pend_len;
    int use_pending;     // 0: a fresh status from the caller, the lists are emptied
    int* pend_touched;   // 1: given requests since its table was built
    int only_touched;    // leave the instances with a 0 there as they are
    const int* batch_cap;   // per instance: requests that may decode together; null = no bound
    // blend with the smoothed black-box status (Sec. 3.3): weight lam on it, 0 = none
    double lam;
    const double *emaQ, *emaP, *emaD;
};

// Median of three; the compiler turns this shape into one v_med3_u32.
__device__ __forceinline__ uint32_t med3_u32(uint32_t a, uint32_t b, uint32_t c)
{
    return min(max(a, b), max(min(a, b), c));
}

template <int kCtrl>
__device__ __forceinline__ uint32_t dpp_move(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, kCtrl, 0xf, 0xf, false);
}

// The copy of x held by lane (lane ^ mask); lane4 = 4 * lane.  Partners inside a
// row of 16 lanes that a DPP pattern reaches come straight from the register
// file; the others through the LDS crossbar.
__device__ __forceinline__ uint32_t fetch_xor(uint32_t x, int mask, int lane4)
{
    switch (mask) {
        case 1: return dpp_move<0xB1>(x);      // quad_perm [1,0,3,2]
        case 2: return dpp_move<0x4E>(x);      // quad_perm [2,3,0,1]
        case 3: return dpp_move<0x1B>(x);      // quad_perm [3,2,1,0]
        case 7: return dpp_move<0x141>(x);     // row_half_mirror
        case 15: return dpp_move<0x140>(x);    // row_mirror
        default: return (uint32_t)__builtin_amdgcn_ds_bpermute(lane4 ^ (mask << 2), (int)x);
    }
}

__device__ __forceinline__ void order2(uint32_t& lo, uint32_t& hi)
{
    const uint32_t a = lo, b = hi;
    lo = a < b ? a : b;
    hi = a < b ? b : a;
}

// Ascending bitonic sort of 64 * kEPL words, word v = lane * kEPL + r in key[r].
// Level K merges sorted runs of K/2 into runs of K: first v against its mirror
// image v ^ (K-1) in the run, then distances K/4, K/8, .. 1; the lower position
// always keeps the smaller word.  Levels and distances are template parameters
// (the network is straight-line code with every register named at compile
// time; as loops over K and the distance the larger sizes were left rolled,
// with registers addressed indirectly).
template <int kEPL, int K>
__device__ __forceinline__ void bitonic_mirror(uint32_t (&key)[kEPL], int lane, int lane4)
{
    if constexpr (K <= kEPL) {
#pragma unroll
        for (int r = 0; r < kEPL; ++r)
            if (r < (r ^ (K - 1))) order2(key[r], key[r ^ (K - 1)]);
    } else {
        constexpr int lm = K / kEPL - 1;
        const uint32_t bound = (lane & (K / kEPL / 2)) ? 0xFFFFFFFFu : 0u;   // upper partner keeps the larger
        uint32_t p[kEPL];
#pragma unroll
        for (int r = 0; r < kEPL; ++r) p[r] = fetch_xor(key[kEPL - 1 - r], lm, lane4);
#pragma unroll
        for (int r = 0; r < kEPL; ++r) key[r] = med3_u32(key[r], p[r], bound);
    }
}

template <int kEPL, int J>
__device__ __forceinline__ void bitonic_distances(uint32_t (&key)[kEPL], int lane, int lane4)
{
    if constexpr (J >= 1) {
        if constexpr (J < kEPL) {
#pragma unroll
            for (int r = 0; r < kEPL; ++r)
                if ((r & J) == 0) order2(key[r], key[r | J]);
        } else {
            constexpr int lm = J / kEPL;
            const uint32_t bound = (lane & lm) ? 0xFFFFFFFFu : 0u;
#pragma unroll
            for (int r = 0; r < kEPL; ++r) key[r] = med3_u32(key[r], fetch_xor(key[r], lm, lane4), bound);
        }
        bitonic_distances<kEPL, J / 2>(key, lane, lane4);
    }
}

template <int kEPL, int K>
__device__ __forceinline__ void bitonic_levels(uint32_t (&key)[kEPL], int lane, int lane4)
{
    if constexpr (K <= kWave * kEPL) {
        bitonic_mirror<kEPL, K>(key, lane, lane4);
        bitonic_distances<kEPL, K / 4>(key, lane, lane4);
        bitonic_levels<kEPL, 2 * K>(key, lane, lane4);
    }
}

template <int kEPL>
__device__ __forceinline__ void bitonic_sort(uint32_t (&key)[kEPL], int lane)
{
    bitonic_levels<kEPL, 2>(key, lane, lane << 2);
}

// The same network over the kSplit waves that share an instance (word v = (part * 64 + lane) *
// kEPL + r): each wave sorts its own words as above, and the levels that span waves fetch the
// partner's words through LDS -- word r of lane l of wave w sits at buf[(w * kEPL + r) * 64 + l],
// so every access is consecutive over the lanes, mirrored or not.  One workgroup barrier per
// exchange: consecutive exchanges alternate between two buffers, and a wave reaches the barrier
// of the next exchange only after it has read what it needed of this one.
template <int kEPL, bool kMirrored>
__device__ __forceinline__ void bitonic_exchange(uint32_t (&key)[kEPL], int lane, int part, int partner, bool upper,
                                                 uint32_t* buf)
{
#pragma unroll
    for (int r = 0; r < kEPL; ++r) buf[(part * kEPL + r) * kWave + lane] = key[r];
    __syncthreads();
    const uint32_t bound = upper ? 0xFFFFFFFFu : 0u;      // the upper partner keeps the larger word
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
        const uint32_t p = kMirrored ? buf[(partner * kEPL + (kEPL - 1 - r)) * kWave + (kWave - 1 - lane)]
                                     : buf[(partner * kEPL + r) * kWave + lane];
        key[r] = med3_u32(key[r], p, bound);
    }
}

template <int kEPL, int kSplit>
__device__ __forceinline__ void bitonic_sort_split(uint32_t (&key)[kEPL], int lane, int part, uint32_t* xch)
{
    static_assert(kSplit >= 2 && (kSplit & (kSplit - 1)) == 0, "a power of two of waves per instance");
    constexpr int kWords = kWave * kEPL, kCap = kWords * kSplit;
    const int lane4 = lane << 2;
    bitonic_levels<kEPL, 2>(key, lane, lane4);
    int flip = 0;
#pragma unroll
    for (int span = 2; span <= kSplit; span *= 2) {
        // runs of `span` waves: the mirror image across the run, then the same position span/4, .. 1
        // waves away, then the distances inside the wave
        bitonic_exchange<kEPL, true>(key, lane, part, part ^ (span - 1), part & (span / 2), xch + flip * kCap);
        flip ^= 1;
#pragma unroll
        for (int d = span / 4; d >= 1; d /= 2) {
            bitonic_exchange<kEPL, false>(key, lane, part, part ^ d, part & d, xch + flip * kCap);
            flip ^= 1;
        }
        bitonic_distances<kEPL, kWords / 2>(key, lane, lane4);
    }
}

// Exclusive prefix over the lanes of a wave, and the total.
__device__ __forceinline__ long long wave_excl_scan(long long v, long long& total)
{
    const long long incl = wave_incl_scan(v);
    total = __shfl(incl, kWave - 1, kWave);
    return incl - v;
}

constexpr int kBuildWaves = kBlock / kWave;

constexpr int log2_of(int v) { return v <= 1 ? 0 : 1 + log2_of(v / 2); }

// The build under batch caps (a kernel of its own: the event loop's registers would cost the
// plain build, k_build_lean below, a wave per SIMD).
template <int kEPL>
__global__ __launch_bounds__(kBlock, 1) void k_build_capped(BuildArgs a)
{
    extern __shared__ uint32_t smem[];
    constexpr int kCap = kWave * kEPL;
    constexpr int kIdxBits = log2_of(kCap);
    constexpr uint32_t kIdxMask = (1u << kIdxBits) - 1u;
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int g = blockIdx.x * kBuildWaves + wave;
    if (g >= a.n_inst) return;
    {   // feedback routing: an instance that has been given nothing since its table was built keeps it
        const bool touched = a.pend_touched[g] != 0;
        if (lane == 0 && touched) a.pend_touched[g] = 0;
        if (a.only_touched && !touched) {
            if (lane == 0) a.rank_acc[g] = 0;
            return;
        }
    }
    int* ctx = reinterpret_cast<int*>(smem) + wave * 3 * kCap;  // this wave's contexts, by entry index
    int* olen = ctx + kCap;    // under a batch cap: length and context as given (ctx then holds them
    int* octx = olen + kCap;   // as they are when a newcomer would be admitted)

    const ClassCoef cc = a.cls[a.inst_class[g]];
    // offsets are clamped into the arrays, so broken CSR data cannot index outside them
    const int a0 = (int)min((int64_t)max(a.act_off[g], 0), a.n_active);
    const int q0 = (int)min((int64_t)max(a.q_off[g], 0), a.n_queued);
    int A = (int)max(min((int64_t)a.act_off[g + 1], a.n_active) - a0, (int64_t)0);
    int Q = (int)max(min((int64_t)a.q_off[g + 1], a.n_queued) - q0, (int64_t)0);
    int status = 0;
    if (A > a.max_entries) { A = a.max_entries; status |= GR_DEV_ENTRIES_DROPPED; }
    if (Q > a.max_entries - A) { Q = a.max_entries - A; status |= GR_DEV_ENTRIES_DROPPED; }
    int P = a.use_pending ? min(a.pend_cnt[g], kCap) : 0;
    if (P > a.max_entries - A - Q) { P = a.max_entries - A - Q; status |= GR_DEV_ENTRIES_DROPPED; }
    const int N = A + Q + P;
    const int* pp = a.pend_prompt + (size_t)g * kCap;
    const int* pl = a.pend_len + (size_t)g * kCap;

    // load, entry i = 64 r + lane.  First every entry's three words, from wherever its kind keeps
    // them (running, queued, routed since the status), so that all loads are in flight together;
    // then one sort word per entry = (remaining length << kIdxBits) | i.
    int rem_in[kEPL], c_in[kEPL], gen_in[kEPL];
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
        const int i = r * kWave + lane;
        const int* p_rem = a.act_rem + a0 + i;
        const int* p_ctx = a.act_prompt + a0 + i;
        if (i >= A + Q) { p_rem = pl + (i - A - Q); p_ctx = pp + (i - A - Q); }
        else if (i >= A) { p_rem = a.q_len + q0 + (i - A); p_ctx = a.q_prompt + q0 + (i - A); }
        rem_in[r] = i < N ? *p_rem : 0;
        c_in[r] = i < N ? *p_ctx : 0;
        gen_in[r] = i < A ? a.act_gen[a0 + i] : 0;
    }
    uint32_t key[kEPL];
    long long qsum = 0;
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
        const int i = r * kWave + lane;
        uint32_t word = 0xFFFFFFFFu;        // past the last entry: sorts to the end
        if (i < N) {
            int rem = rem_in[r];
            const int c = c_in[r] + gen_in[r];
            if (i >= A) qsum += c;
            if (rem < 0 || rem > a.max_len) { rem = min(max(rem, 0), a.max_len); status |= GR_DEV_LEN_CLAMPED; }
            word = ((uint32_t)rem << kIdxBits) | (uint32_t)i;
            ctx[i] = c;
        }
        key[r] = word;
    }
    // (stores on their own: a store between two uses of loaded words would make the second wait for it)
#pragma unroll
    for (int r = 0; r < kEPL; ++r)
        if (r * kWave + lane < A) a.act_inst[a0 + r * kWave + lane] = g;
    if (status) atomicOr(&a.counters[0], status);
    if (Q + P > 0) qsum = wave_sum(qsum);   // Q and P are the same in every lane
    double q = cc.delta * (double)qsum;

    // with a blend, every estimate below is keep * (white-box value) + lam * (Eq. 2 with the smoothed status)
    const bool blended = a.lam != 0.0;
    const double keep = 1.0 - a.lam;
    const double bq = blended ? a.emaQ[g] : 0.0, bp = blended ? a.emaP[g] : 0.0, bd = blended ? a.emaD[g] : 0.0;
    // what a request of the instance is told: entry i, white-box finish time, its length and context as given
    auto report = [&](int i, double fin, double len0, double ctx0) {
        if (blended)   // black-box finish: d per remaining token; a queued request also waits and prefills
            fin = keep * fin + a.lam * (i < A ? bd * len0 : (bq + bp * ctx0) + bd * len0);
        if (i < A) {
            a.out_act_finish[a0 + i] = (float)fin;
            if (a.act_budget) a.out_flag[a0 + i] = fin > (double)a.act_budget[a0 + i];
        } else if (a.out_q_finish && i < A + Q) {
            a.out_q_finish[q0 + i - A] = (float)fin;
        }
    };

    // ---- batch cap (Sec. 3.1: concurrency bounded by memory).  With room for everybody and a
    // newcomer nothing changes.  Otherwise, while there is a queue, the instance is played forward
    // event by event (the queue's head is admitted whenever the batch has room; between two
    // departures the batch is fixed and its time is a closed form); requests that leave meanwhile
    // get their finish time here.  Once the queue is empty only departures are left: if the batch
    // has room now, a newcomer is admitted now (q_g = now, and the closed form below is built on
    // what is running); if not, it is admitted after the departure that makes room, which the
    // closed form itself gives (further down).
    const int cap_g = max(a.batch_cap[g], 1);
    const bool capped = cap_g <= N;
    int Nrun = N;
    double d_first = -1.0;
    if (capped) {
        int fstep[kEPL], cbase[kEPL];     // decode step at which the entry leaves; its context minus the step count
#pragma unroll
        for (int r = 0; r < kEPL; ++r) {
            const int i = r * kWave + lane;
            const int len0 = i < N ? (int)(key[r] >> kIdxBits) : 0, c0 = i < N ? ctx[i] : 0;
            fstep[r] = i < A ? len0 : (i < N ? 0x7fffffff : 0);     // queued: not in yet; none: gone
            cbase[r] = c0;
            if (i < N) { olen[i] = len0; octx[i] = c0; }
        }
        long long C = 0;
#pragma unroll
        for (int r = 0; r < kEPL; ++r) C += r * kWave + lane < A ? cbase[r] : 0;
        C = wave_sum(C);
        int n = A, s = 0, next_q = A;     // batch size, steps done, next entry of the queue
        double t = 0.0;
        for (int guard = 0; guard <= 2 * N + 2; ++guard) {
            const int k = min(cap_g - n, N - next_q);
            if (k > 0) {                   // admit entries next_q .. next_q + k - 1: prefill, then into the batch
                long long sumP = 0;
#pragma unroll
                for (int r = 0; r < kEPL; ++r) {
                    const int i = r * kWave + lane;
                    if (i >= next_q && i < next_q + k) {
                        fstep[r] = s + (int)(key[r] >> kIdxBits);
                        sumP += cbase[r];
                        cbase[r] -= s;
                    }
                }
                sumP = wave_sum(sumP);
                t += cc.delta * (double)sumP;
                n += k; C += sumP; next_q += k;
            }
            if (next_q == N) break;        // the queue is empty: what follows is departures only (below)
            // next departure
            int smin = 0x7fffffff;
#pragma unroll
            for (int r = 0; r < kEPL; ++r) smin = min(smin, fstep[r] > s ? fstep[r] : 0x7fffffff);
#pragma unroll
            for (int dlt = kWave / 2; dlt > 0; dlt >>= 1) smin = min(smin, __shfl_xor(smin, dlt, kWave));
            if (smin == 0x7fffffff) break;            // (nobody is running: cannot be, the batch has room then)
            const double step_now = fma(cc.gamma, (double)C, fma(cc.beta, (double)n, cc.alpha));
            if (d_first < 0.0) d_first = step_now;
            const long long ks = smin - s;
            // ks steps of a fixed batch: contexts grow by one per member and step
            t += (double)ks * step_now + cc.gamma * ((double)n * (double)(ks * (ks - 1) / 2));
            C += (long long)n * ks;
            s = smin;
            int gone = 0;
            long long goneC = 0;
#pragma unroll
            for (int r = 0; r < kEPL; ++r) {
                if (fstep[r] == s) {
                    const int i = r * kWave + lane;
                    ++gone;
                    goneC += cbase[r] + s;
                    report(i, t, (double)olen[i], (double)octx[i]);
                }
            }
            n -= wave_sum(gone);
            C -= wave_sum(goneC);
        }
        // what is left, as of now: the sort words and contexts the closed form is built from
        q = t;
        Nrun = n;
#pragma unroll
        for (int r = 0; r < kEPL; ++r) {
            const int i = r * kWave + lane;
            const bool running = fstep[r] > s && fstep[r] != 0x7fffffff;
            key[r] = running ? ((uint32_t)(fstep[r] - s) << kIdxBits) | (uint32_t)i : 0xFFFFFFFFu;
            if (running) ctx[i] = cbase[r] + s;
        }
    }

    bitonic_sort<kEPL>(key, lane);

    // the wave's own LDS writes above must be visible to its reads below
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // sorted position v = lane * kEPL + r; entries first, in order of remaining length
    int R[kEPL], cx[kEPL], idx[kEPL];
    long long yl = 0, xl = 0, cl = 0;       // this lane's sums of R, c*R + tri(R), c
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
        const bool valid = lane * kEPL + r < Nrun;
        idx[r] = (int)(key[r] & kIdxMask);
        R[r] = valid ? (int)(key[r] >> kIdxBits) : 0;
        cx[r] = valid ? ctx[idx[r]] : 0;
        yl += R[r];
        xl += (long long)cx[r] * R[r] + (long long)(R[r] * (R[r] - 1) / 2);
        cl += cx[r];
    }
    long long Ytot, Xtot, Ctot;
    long long Y = wave_excl_scan(yl, Ytot), X = wave_excl_scan(xl, Xtot), Pc = wave_excl_scan(cl, Ctot);

    // ---- a full batch with an empty queue: a newcomer is admitted when the kstar-th of the running
    // requests has left.  Until then nobody joins, so everybody's finish time is the closed form
    // as it stands, the admission time q_g is the finish time of that request (s steps from now),
    // and the table describes the others as they are then: s steps shorter, contexts s longer.
    // With R' = R - s, c' = c + s over the survivors (positions vstar.. of the sorted order):
    //   sum R' = sum R - m s,   sum (c' R' + tri(R')) = sum (c R + tri(R)) - s sum c - m tri(s),
    //   sum c' = sum c + m s    (m terms each; all integers, exact)
    {
        if (capped && Nrun >= cap_g) {
            const int kstar = Nrun - cap_g + 1;
            long long Y1 = Y, X1 = X, P1 = Pc;
            double q_adm = 0.0;
            int sstar = 0;
#pragma unroll
            for (int r = 0; r < kEPL; ++r) {
                const int v = lane * kEPL + r;
                const long long Rr = R[r], triR = (long long)(R[r] * (R[r] - 1) / 2);
                Y1 += Rr; X1 += (long long)cx[r] * Rr + triR; P1 += cx[r];
                if (v < Nrun) {
                    const double n_after = (double)(Nrun - v - 1), S_next = (double)(Ctot - P1), Rd = (double)Rr;
                    const double I1 = (double)Y1 + n_after * Rd;
                    const double I2 = (double)X1 + Rd * S_next + n_after * (double)triR;
                    const double fin = q + fma(cc.gamma, I2, fma(cc.beta, I1, cc.alpha * Rd));
                    report(idx[r], fin, (double)olen[idx[r]], (double)octx[idx[r]]);
                    if (v == kstar - 1) { q_adm = fin; sstar = R[r]; }
                }
            }
            const int owner = (kstar - 1) / kEPL;
            q_adm = __shfl(q_adm, owner, kWave);
            sstar = __shfl(sstar, owner, kWave);
            // those that have left by then (equal lengths leave together)
            long long gone = 0, yg = 0, xg = 0, cg = 0;
#pragma unroll
            for (int r = 0; r < kEPL; ++r)
                if (lane * kEPL + r < Nrun && R[r] <= sstar) {
                    ++gone; yg += R[r]; cg += cx[r];
                    xg += (long long)cx[r] * R[r] + (long long)(R[r] * (R[r] - 1) / 2);
                }
            const int vstar = (int)wave_sum(gone);
            const long long Ystar = wave_sum(yg), Xstar = wave_sum(xg), Pstar = wave_sum(cg);
            const int Nleft = Nrun - vstar;
            const long long s64 = sstar, tri_s = s64 * (s64 - 1) / 2;
            Y1 = Y; X1 = X; P1 = Pc;
            uint16_t* dstR = a.tabR + (size_t)g * kCap;
            float2* dstGH = a.tabGH + (size_t)g * kCap;
#pragma unroll
            for (int r = 0; r < kEPL; ++r) {
                const int v = lane * kEPL + r;
                const long long Rr = R[r];
                Y1 += Rr; X1 += (long long)cx[r] * Rr + (long long)(R[r] * (R[r] - 1) / 2); P1 += cx[r];
                if (v >= vstar && v < Nrun) {
                    const int w = v - vstar;                      // position among the survivors
                    const long long m = w + 1;
                    const double Ys = (double)((Y1 - Ystar) - m * s64);
                    const double Xs = (double)((X1 - Xstar) - s64 * (P1 - Pstar) - m * tri_s);
                    const double n_after = (double)(Nleft - w - 1);
                    const double S_next = (double)((Ctot - P1) + (long long)(Nleft - w - 1) * s64);
                    double Gq = q_adm + (cc.beta * Ys + cc.gamma * Xs);
                    double Hs = cc.alpha + (cc.beta * (n_after + 1.0) + cc.gamma * S_next);
                    if (blended) { Gq = keep * Gq + a.lam * bq; Hs = keep * Hs + a.lam * bd; }
                    dstR[w] = (uint16_t)(R[r] - sstar);
                    dstGH[w] = make_float2((float)Gq, (float)Hs);
                } else {                                          // the slots behind the survivors
                    const int slot = v < Nrun ? Nleft + v : v;
                    dstR[slot] = (uint16_t)0xFFFFu;
                    dstGH[slot] = make_float2(0.f, 0.f);
                }
            }
            if (lane == 0) {
                const double Cd = (double)((Ctot - Pstar) + (long long)Nleft * s64);
                double Gq0 = q_adm, H0 = cc.alpha + (cc.beta * (double)(Nleft + 1) + cc.gamma * Cd);
                if (blended) { Gq0 = keep * Gq0 + a.lam * bq; H0 = keep * H0 + a.lam * bd; }
                a.headGH[g] = make_float2((float)Gq0, (float)H0);
                a.hN[g] = Nleft;
                a.rank_acc[g] = 0;
                if (!a.use_pending) a.pend_cnt[g] = 0;
                // the next decode step that runs: the first one played above, else the batch as it stands
                double d = d_first >= 0.0 ? d_first
                                          : fma(cc.gamma, (double)Ctot, fma(cc.beta, (double)Nrun, cc.alpha));
                if (blended) d = keep * d + a.lam * bd;
                a.hD[g] = d;
                if (a.out_d) a.out_d[g] = d;
            }
            return;
        }
    }

    // table entry v describes the segment after the v+1 shortest requests, n of them still running:
    //   E_g(L) = Gq + L * H + tri(L) * gamma * (n + 1)
    //   Gq = q + beta * Y + gamma * X,   H = alpha + beta * (n + 1) + gamma * S
    uint16_t tR[kEPL];
    float2 tGH[kEPL];
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
        const int v = lane * kEPL + r;
        const bool valid = v < Nrun;
        const long long Rr = R[r], triR = (long long)(R[r] * (R[r] - 1) / 2);
        Y += Rr;
        X += (long long)cx[r] * Rr + triR;
        Pc += cx[r];
        const double n_after = (double)(Nrun - v - 1), S_next = (double)(Ctot - Pc);
        const double Yd = (double)Y, Xd = (double)X, Rd = (double)Rr;
        tR[r] = valid ? (uint16_t)R[r] : (uint16_t)0xFFFFu;
        double Gq = q + (cc.beta * Yd + cc.gamma * Xd);
        double Hs = cc.alpha + (cc.beta * (n_after + 1.0) + cc.gamma * S_next);
        if (blended) { Gq = keep * Gq + a.lam * bq; Hs = keep * Hs + a.lam * bd; }
        tGH[r] = make_float2((float)Gq, (float)Hs);
        if (valid) {
            // every product below is an integer below 2^53: exact
            const double I1 = Yd + n_after * Rd;
            const double I2 = Xd + Rd * S_next + n_after * (double)triR;
            const double fin = q + fma(cc.gamma, I2, fma(cc.beta, I1, cc.alpha * Rd));
            report(idx[r], fin, capped ? (double)olen[idx[r]] : Rd, capped ? (double)octx[idx[r]] : (double)cx[r]);
        }
    }
    {
        uint16_t* dstR = a.tabR + (size_t)g * kCap + lane * kEPL;
        float2* dstGH = a.tabGH + (size_t)g * kCap + lane * kEPL;
        if constexpr (kEPL >= 8) {
#pragma unroll
            for (int r = 0; r < kEPL; r += 8) {
                uint4 w;
                w.x = tR[r] | ((uint32_t)tR[r + 1] << 16); w.y = tR[r + 2] | ((uint32_t)tR[r + 3] << 16);
                w.z = tR[r + 4] | ((uint32_t)tR[r + 5] << 16); w.w = tR[r + 6] | ((uint32_t)tR[r + 7] << 16);
                *reinterpret_cast<uint4*>(dstR + r) = w;
            }
        } else {
#pragma unroll
            for (int r = 0; r < kEPL; ++r) dstR[r] = tR[r];
        }
        if constexpr (kEPL >= 2) {
#pragma unroll
            for (int r = 0; r < kEPL; r += 2)
                *reinterpret_cast<float4*>(dstGH + r) = make_float4(tGH[r].x, tGH[r].y, tGH[r + 1].x, tGH[r + 1].y);
        } else {
            dstGH[0] = tGH[0];
        }
    }
    if (lane == 0) {
        const double Cd = (double)Ctot;
        double Gq0 = q, H0 = cc.alpha + (cc.beta * (double)(Nrun + 1) + cc.gamma * Cd);
        if (blended) { Gq0 = keep * Gq0 + a.lam * bq; H0 = keep * H0 + a.lam * bd; }
        a.headGH[g] = make_float2((float)Gq0, (float)H0);
        a.hN[g] = Nrun;
        a.rank_acc[g] = 0;
        if (!a.use_pending) a.pend_cnt[g] = 0;
        // the next decode step that runs: the first one played above, else the batch as it stands
        double d = d_first >= 0.0 ? d_first : fma(cc.gamma, Cd, fma(cc.beta, (double)Nrun, cc.alpha));
        if (blended) d = keep * d + a.lam * bd;
        a.hD[g] = d;
        if (a.out_d) a.out_d[g] = d;
    }
}

// ---- the build without batch caps: the same results from fewer instructions.
//
// The instance's running requests are read and their results written through buffer
// descriptors that span exactly the instance's slice of the caller's arrays: an offset past
// the slice reads zero and stores nothing, so there is no address arithmetic and no branch per
// entry.  The three prefix sums run in double precision (every term and every sum is an
// integer below 2^53, so they are exact), first along the lane's own consecutive positions,
// then across the lanes by DPP shifts, and the table and finish times come out of them with
// fused multiply-adds, without any integer-to-double conversion of a 64-bit sum.

// x of the lane `ctrl` names (0.0 where there is none or the row is masked out), both halves
template <int kCtrl, int kRowMask>
__device__ __forceinline__ double dpp_or_zero(double x)
{
    const long long b = __builtin_bit_cast(long long, x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)b, kCtrl, kRowMask, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), kCtrl, kRowMask, 0xf, false);
    return __builtin_bit_cast(double, ((long long)hi << 32) | (unsigned)lo);
}

// Inclusive prefix sum over the lanes of a wave (see wave_incl_scan_i32 for the pattern).
__device__ __forceinline__ double wave_incl_scan_f64(double v)
{
    v += dpp_or_zero<0x111, 0xf>(v);   // row_shr:1
    v += dpp_or_zero<0x112, 0xf>(v);   // row_shr:2
    v += dpp_or_zero<0x114, 0xf>(v);   // row_shr:4
    v += dpp_or_zero<0x118, 0xf>(v);   // row_shr:8
    v += dpp_or_zero<0x142, 0xa>(v);   // row_bcast:15 into rows 1, 3
    v += dpp_or_zero<0x143, 0xc>(v);   // row_bcast:31 into rows 2, 3
    return v;
}

__device__ __forceinline__ double readlane_f64(double v, int lane)
{
    const long long b = __builtin_bit_cast(long long, v);
    const int lo = __builtin_amdgcn_readlane((int)b, lane), hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
    return __builtin_bit_cast(double, ((long long)hi << 32) | (unsigned)lo);
}

constexpr int kBufferDwords = 0x00020000;   // descriptor word 3: raw buffer of 32-bit elements

// 32-bit words of LDS per instance of the plain build: contexts, budgets / finish times, flag bytes
constexpr int lean_inst_words(int cap) { return 2 * cap + cap / 4; }

// kEPL sort words per lane; kSplit waves share an instance (kSplit = 1: a workgroup is four instances, a wave each; 2 or 4:
// a workgroup is one instance): wave `part` reads entries part * 64 * kEPL onwards, the sort's
// last levels and the totals of the prefix sums cross the waves through LDS, and the wave ends
// up with sorted positions part * 64 * kEPL onwards.  The results are the same bit for bit (the
// sums are exact); a fleet with fewer instances than the chip has SIMDs gets shorter dependent
// chains and more waves to overlap them.
template <int kEPL, int kSplit>
__global__ __launch_bounds__(kSplit == 1 ? kBlock : kWave * kSplit, (kEPL <= 8 ? 4 : 1)) void k_build_lean(BuildArgs a)
{
    extern __shared__ uint32_t smem[];
    constexpr int kWords = kWave * kEPL;         // sort words of a wave
    constexpr int kCap = kWords * kSplit;        // of an instance
    constexpr int kIdxBits = log2_of(kCap);
    constexpr uint32_t kIdxMask = (1u << kIdxBits) - 1u;
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int g = kSplit == 1 ? blockIdx.x * kBuildWaves + wave : blockIdx.x;   // wave-uniform: what follows is scalar
    const int part = kSplit == 1 ? 0 : wave;
    const int first = part * kWords;             // this wave's first entry, and its first sorted position
    if (g >= a.n_inst) return;
    // feedback routing: an instance that has been given nothing since its table was built keeps it
    // (the mark is cleared at the very end, when every wave of the instance has read it)
    if (a.only_touched && a.pend_touched[g] == 0) {
        if (lane == 0 && part == 0) a.rank_acc[g] = 0;
        return;
    }
    // LDS of an instance, all by entry index: contexts; budgets on the way in and finish times on the
    // way out (the caller's arrays are read and written in their own order, 64 consecutive entries
    // per instruction; the sorted order reaches them through LDS); flags, a byte each
    constexpr int kInstWords = lean_inst_words(kCap);
    uint32_t* const mine_lds = smem + (kSplit == 1 ? wave * kInstWords : 0);
    int* ctx = reinterpret_cast<int*>(mine_lds);
    float* stage = reinterpret_cast<float*>(mine_lds + kCap);
    uint8_t* flag_lds = reinterpret_cast<uint8_t*>(mine_lds + 2 * kCap);
    uint32_t* xch = smem + kInstWords;                                              // (split) two exchange buffers
    double* sums = reinterpret_cast<double*>(smem + kInstWords + 2 * kCap);         // (split) four totals per wave

    const ClassCoef cc = a.cls[a.inst_class[g]];
    // offsets are clamped into the arrays, so broken CSR data cannot index outside them
    const int a0 = (int)min((int64_t)max(a.act_off[g], 0), a.n_active);
    const int q0 = (int)min((int64_t)max(a.q_off[g], 0), a.n_queued);
    int A = (int)max(min((int64_t)a.act_off[g + 1], a.n_active) - a0, (int64_t)0);
    int Q = (int)max(min((int64_t)a.q_off[g + 1], a.n_queued) - q0, (int64_t)0);
    int status = 0;
    if (A > a.max_entries) { A = a.max_entries; status |= GR_DEV_ENTRIES_DROPPED; }
    if (Q > a.max_entries - A) { Q = a.max_entries - A; status |= GR_DEV_ENTRIES_DROPPED; }
    int P = a.use_pending ? min(a.pend_cnt[g], kCap) : 0;
    if (P > a.max_entries - A - Q) { P = a.max_entries - A - Q; status |= GR_DEV_ENTRIES_DROPPED; }
    const int N = A + Q + P;

    // the instance's slice of each array of running requests (A entries from a0 on)
    const auto slice = [&](const void* base, size_t elem) {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(static_cast<const char*>(base)) + (size_t)a0 * elem,
                                                 0, A * (int)elem, kBufferDwords);
    };
    const __amdgpu_buffer_rsrc_t b_rem = slice(a.act_rem, 4), b_prompt = slice(a.act_prompt, 4),
                                 b_gen = slice(a.act_gen, 4), b_fin = slice(a.out_act_finish, 4);
    __amdgpu_buffer_rsrc_t b_bud = b_fin, b_flag = b_fin;
    if (a.act_budget) { b_bud = slice(a.act_budget, 4); b_flag = slice(a.out_flag, 1); }

    // load, entry i = first + 64 r + lane: all loads in flight together
    const int lane4 = lane * 4;
    int rem_in[kEPL], c_in[kEPL], gen_in[kEPL], bud_in[kEPL];
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
        rem_in[r] = __builtin_amdgcn_raw_buffer_load_b32(b_rem, lane4, (first + r * kWave) * 4, 0);
        c_in[r] = __builtin_amdgcn_raw_buffer_load_b32(b_prompt, lane4, (first + r * kWave) * 4, 0);
        gen_in[r] = __builtin_amdgcn_raw_buffer_load_b32(b_gen, lane4, (first + r * kWave) * 4, 0);
    }
    if (a.act_budget) {
#pragma unroll
        for (int r = 0; r < kEPL; ++r)
            bud_in[r] = __builtin_amdgcn_raw_buffer_load_b32(b_bud, lane4, (first + r * kWave) * 4, 0);
    }
    long long qsum = 0;
    if (Q + P > 0) {     // queued requests, and those routed since the status (feedback routing)
        const int* pp = a.pend_prompt + (size_t)g * kCap;
        const int* pl = a.pend_len + (size_t)g * kCap;
#pragma unroll
        for (int r = 0; r < kEPL; ++r) {
            const int i = first + r * kWave + lane;
            if (i >= A && i < N) {
                const bool queued = i < A + Q;
                rem_in[r] = queued ? a.q_len[q0 + i - A] : pl[i - A - Q];
                c_in[r] = queued ? a.q_prompt[q0 + i - A] : pp[i - A - Q];
                qsum += c_in[r];
            }
        }
        qsum = wave_sum(qsum);
    }

    // one sort word per entry = (remaining length << kIdxBits) | i; past the last entry all ones
    uint32_t key[kEPL];
    bool bad = false;
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
        const int i = first + r * kWave + lane;
        const int rem = min(max(rem_in[r], 0), a.max_len);
        bad |= rem != rem_in[r];
        key[r] = i < N ? ((uint32_t)rem << kIdxBits) | (uint32_t)i : 0xFFFFFFFFu;
        ctx[i] = c_in[r] + gen_in[r];          // (zero past the last entry: the loads returned zeros)
    }
    if (a.act_budget) {
#pragma unroll
        for (int r = 0; r < kEPL; ++r) stage[first + r * kWave + lane] = __int_as_float(bud_in[r]);
    }
    if (__ballot(bad)) status |= GR_DEV_LEN_CLAMPED;
    if (status && lane == 0) atomicOr(&a.counters[0], status);
    if (a.act_budget) {      // the instance of each running request, for the migration pass of a risk scan
        const __amdgpu_buffer_rsrc_t b_inst = slice(a.act_inst, 4);
#pragma unroll
        for (int r = 0; r < kEPL; ++r) __builtin_amdgcn_raw_buffer_store_b32(g, b_inst, lane4, (first + r * kWave) * 4, 0);
    }

    if constexpr (kSplit == 1) {
        bitonic_sort<kEPL>(key, lane);
        // the wave's own LDS writes above must be visible to its reads below
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
        bitonic_sort_split<kEPL, kSplit>(key, lane, part, xch);     // (its barriers also publish the contexts)
    }

    // sorted position v = first + lane * kEPL + r; per lane the sums of R, c*R + tri(R), c
    int idx[kEPL], Ri[kEPL], ci[kEPL];
    const int mine = N - first - lane * kEPL;    // positions of this lane that hold an entry
    // an entry's terms of the three sums, as doubles (formed twice, here and below, rather than kept)
    const auto terms = [&](int r, double& Rd, double& cd, double& td, double& xe) {
        Rd = (double)Ri[r];
        cd = (double)ci[r];
        td = (double)(Ri[r] * (Ri[r] - 1) / 2);
        xe = fma(cd, Rd, td);
    };
    double yl = 0.0, xl = 0.0, cl = 0.0;
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
        idx[r] = (int)(key[r] & kIdxMask);
        Ri[r] = r < mine ? (int)(key[r] >> kIdxBits) : 0;
        // (a position without an entry carries index kCap - 1, an entry that does not exist either: zero)
        ci[r] = ctx[idx[r]];
    }
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
        double Rd, cd, td, xe;
        terms(r, Rd, cd, td, xe);
        yl += Rd; xl += xe; cl += cd;
    }
#pragma unroll
    for (int r = 0; r < kEPL; ++r) asm volatile("" : "+v"(Ri[r]), "+v"(ci[r]));   // (so that the terms are not kept in registers)
    const double yi = wave_incl_scan_f64(yl), xi = wave_incl_scan_f64(xl), pi = wave_incl_scan_f64(cl);
    double Ctot = readlane_f64(pi, kWave - 1);
    double Y = yi - yl, X = xi - xl, Pc = pi - cl;
    double qtot = (double)qsum;
    if constexpr (kSplit > 1) {      // the waves before this one, and everybody's total
        if (lane == kWave - 1) {
            sums[part * 4 + 0] = yi; sums[part * 4 + 1] = xi; sums[part * 4 + 2] = pi; sums[part * 4 + 3] = qtot;
        }
        __syncthreads();
        Ctot = 0.0; qtot = 0.0;
#pragma unroll
        for (int w = 0; w < kSplit; ++w) {
            const double yw = sums[w * 4 + 0], xw = sums[w * 4 + 1], pw = sums[w * 4 + 2];
            if (w < part) { Y += yw; X += xw; Pc += pw; }
            Ctot += pw;
            qtot += sums[w * 4 + 3];
        }
    }
    const double q = cc.delta * qtot;

    // with a blend, every estimate below is keep * (white-box value) + lam * (Eq. 2 with the smoothed status)
    const bool blended = a.lam != 0.0;
    const double keep = 1.0 - a.lam;
    const double bq = blended ? a.emaQ[g] : 0.0, bp = blended ? a.emaP[g] : 0.0, bd = blended ? a.emaD[g] : 0.0;

    // table entry v describes the segment after the v+1 shortest requests, n of them still running:
    //   E_g(L) = Gq + L * H + tri(L) * gamma * (n + 1)
    //   Gq = q + beta * Y + gamma * X,   H = alpha + beta * (n + 1) + gamma * S
    // and the request at position v finishes at q + alpha R + beta (Y + n R) + gamma (X + R S + n tri(R)).
    uint16_t tR[kEPL];
    float2 tGH[kEPL];
    float fin32[kEPL], bud[kEPL];
    unsigned late = 0;                           // bit r: the request at position r finishes after its budget
    if (a.act_budget) {
#pragma unroll
        for (int r = 0; r < kEPL; ++r) bud[r] = stage[idx[r]];
    }
    double n_here = (double)mine;                // requests still running from this position on, itself included
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
        double Rd, cd, td, xe;
        terms(r, Rd, cd, td, xe);
        Y += Rd; X += xe; Pc += cd;
        const double n_after = n_here - 1.0, S_next = Ctot - Pc;
        double Gq = fma(cc.gamma, X, fma(cc.beta, Y, q));
        double Hs = fma(cc.gamma, S_next, fma(cc.beta, n_here, cc.alpha));
        double fin = fma(cc.gamma, fma(n_after, td, fma(Rd, S_next, X)),
                         fma(cc.beta, fma(n_after, Rd, Y), fma(cc.alpha, Rd, q)));
        n_here = n_after;
        if (blended) {
            Gq = keep * Gq + a.lam * bq;
            Hs = keep * Hs + a.lam * bd;
            // black-box finish: d per remaining token; a queued request also waits and prefills
            fin = keep * fin + a.lam * (idx[r] < A ? bd * Rd : (bq + bp * cd) + bd * Rd);
        }
        fin32[r] = (float)fin;
        if (a.act_budget) late |= (unsigned)(fin > (double)bud[r]) << r;     // decided in double precision
        tR[r] = r < mine ? (uint16_t)Ri[r] : (uint16_t)0xFFFFu;
        tGH[r] = make_float2((float)Gq, (float)Hs);
    }
    // Finish times and flags go back to entry order through LDS: the lane that read an entry's budget
    // from its slot is the one that writes its finish time there.  (A position without an entry
    // carries index kCap - 1 >= N: a slot past the slice, of which nothing is stored.)
#pragma unroll
    for (int r = 0; r < kEPL; ++r) stage[idx[r]] = fin32[r];
    if (a.act_budget) {
#pragma unroll
        for (int r = 0; r < kEPL; ++r) flag_lds[idx[r]] = (uint8_t)((late >> r) & 1u);
    }
    if constexpr (kSplit == 1) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < kEPL; ++r)
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_int(stage[first + r * kWave + lane]), b_fin, lane4,
                                              (first + r * kWave) * 4, 0);
    if (a.act_budget) {
#pragma unroll
        for (int r = 0; r < kEPL; ++r)
            __builtin_amdgcn_raw_buffer_store_b8(flag_lds[first + r * kWave + lane], b_flag, lane, first + r * kWave, 0);
    }
    if (Q > 0 && a.out_q_finish) {
#pragma unroll
        for (int r = 0; r < kEPL; ++r)
            if (r < mine && idx[r] >= A && idx[r] < A + Q) a.out_q_finish[q0 + idx[r] - A] = fin32[r];
    }
    {
        uint16_t* dstR = a.tabR + (size_t)g * kCap + first + lane * kEPL;
        float2* dstGH = a.tabGH + (size_t)g * kCap + first + lane * kEPL;
        if constexpr (kEPL >= 8) {
#pragma unroll
            for (int r = 0; r < kEPL; r += 8) {
                uint4 w;
                w.x = tR[r] | ((uint32_t)tR[r + 1] << 16); w.y = tR[r + 2] | ((uint32_t)tR[r + 3] << 16);
                w.z = tR[r + 4] | ((uint32_t)tR[r + 5] << 16); w.w = tR[r + 6] | ((uint32_t)tR[r + 7] << 16);
                *reinterpret_cast<uint4*>(dstR + r) = w;
            }
        } else {
#pragma unroll
            for (int r = 0; r < kEPL; ++r) dstR[r] = tR[r];
        }
        if constexpr (kEPL >= 2) {
#pragma unroll
            for (int r = 0; r < kEPL; r += 2)
                *reinterpret_cast<float4*>(dstGH + r) = make_float4(tGH[r].x, tGH[r].y, tGH[r + 1].x, tGH[r + 1].y);
        } else {
            dstGH[0] = tGH[0];
        }
    }
    if (lane == 0 && part == 0) {
        double Gq0 = q, H0 = fma(cc.gamma, Ctot, fma(cc.beta, (double)(N + 1), cc.alpha));
        if (blended) { Gq0 = keep * Gq0 + a.lam * bq; H0 = keep * H0 + a.lam * bd; }
        a.headGH[g] = make_float2((float)Gq0, (float)H0);
        a.hN[g] = N;
        a.rank_acc[g] = 0;
        a.pend_touched[g] = 0;
        if (!a.use_pending) a.pend_cnt[g] = 0;
        double d = fma(cc.gamma, Ctot, fma(cc.beta, (double)N, cc.alpha));     // the next decode step
        if (blended) d = keep * d + a.lam * bd;
        a.hD[g] = d;
        if (a.out_d) a.out_d[g] = d;
    }
}

// Capability order of Alg. 1's argmax d_g as two kernels of their own (see common.h for the
// steps; a scoring pass normally runs them as extra workgroups of its first two kernels).
__global__ __launch_bounds__(kBlock) void k_rank_count(RankArgs a)
{
    __shared__ double comp[kBlock];
    rank_count_tile<kBlock>(a, blockIdx.x, blockIdx.y, comp);
}

__global__ __launch_bounds__(kBlock) void k_rank_final(RankArgs a)
{
    rank_final_item(a, blockIdx.x * kBlock + threadIdx.x);
}

// One step of the exponential moving average of Alg. 1, q <- w * sample + (1 - w) * q, for
// each of the three status terms that has a new sample; a term's first sample is its estimate.
__global__ __launch_bounds__(kBlock) void k_ema(int n_inst, double w, const float* __restrict__ s_q,
                                                const float* __restrict__ s_p, const float* __restrict__ s_d,
                                                int first_q, int first_p, int first_d,
                                                double* __restrict__ q, double* __restrict__ p, double* __restrict__ d)
{
    const int g = blockIdx.x * kBlock + threadIdx.x;
    if (g >= n_inst) return;
    if (s_q) q[g] = first_q ? (double)s_q[g] : w * (double)s_q[g] + (1.0 - w) * q[g];
    if (s_p) p[g] = first_p ? (double)s_p[g] : w * (double)s_p[g] + (1.0 - w) * p[g];
    if (s_d) d[g] = first_d ? (double)s_d[g] : w * (double)s_d[g] + (1.0 - w) * d[g];
}

// Requests that were routed join the queue of their instance (feedback routing), in the order of
// the batch: the slot of a request is the number of requests already queued there plus the number
// of earlier requests of the chunk that were sent to the same instance.  That order matters under
// batch caps (admission is first come, first served), so it must not depend on how the hardware
// schedules waves.  A chunk that fits one wave is placed by that wave (lanes are in request
// order).  A larger chunk under caps takes two kernels: the first marks the instances that were
// chosen at all, the second gives every marked instance a wave that walks the chunk in order.
// Without caps the order of a queue shows in no output (the requests behind it wait for all of
// them either way; sums and sorted lengths do not depend on it), and a larger chunk is placed by
// one kernel that hands out slots with one atomic per wave and instance.
__global__ __launch_bounds__(kWave) void k_commit_wave(int n, const int* __restrict__ inst,
                                                       const int* __restrict__ ctx0, const int* __restrict__ pred_len,
                                                       int* __restrict__ pend_cnt, int* __restrict__ pend_prompt,
                                                       int* __restrict__ pend_len, int* __restrict__ pend_touched,
                                                       int cap, int n_inst, int* __restrict__ counters)
{
    const int lane = lane_id();
    int g = lane < n ? inst[lane] : -1;
    if (g >= n_inst) g = -1;
    const bool act = g >= 0;
    unsigned long long todo = __ballot(act);
    int slot = 0;
    while (todo) {
        const int leader = __ffsll((long long)todo) - 1;
        const int gl = __builtin_amdgcn_readlane(g, leader);
        const unsigned long long same = __ballot(act && g == gl);
        int base = 0;
        if (lane == leader) {
            base = pend_cnt[gl];
            pend_cnt[gl] = base + __popcll(same);
            pend_touched[gl] = 1;
        }
        base = __builtin_amdgcn_readlane(base, leader);
        if (act && g == gl) slot = base + __popcll(same & ((1ull << lane) - 1ull));
        todo &= ~same;
    }
    if (act) {
        if (slot < cap) {
            pend_prompt[(size_t)g * cap + slot] = ctx0[lane];
            pend_len[(size_t)g * cap + slot] = pred_len[lane];
        } else {
            atomicOr(&counters[0], GR_DEV_ENTRIES_DROPPED);
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_commit_any_order(int64_t n, const int* __restrict__ inst,
                                                             const int* __restrict__ ctx0, const int* __restrict__ pred_len,
                                                             int* __restrict__ pend_cnt, int* __restrict__ pend_prompt,
                                                             int* __restrict__ pend_len, int* __restrict__ pend_touched,
                                                             int cap, int n_inst, int* __restrict__ counters)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int lane = lane_id();
    int g = i < n ? inst[i] : -1;
    if (g >= n_inst) g = -1;
    const bool act = g >= 0;
    unsigned long long todo = __ballot(act);
    int slot = 0;
    while (todo) {      // many requests of a chunk go to the same instance: one atomic for all of a wave's
        const int leader = __ffsll((long long)todo) - 1;
        const int gl = __builtin_amdgcn_readlane(g, leader);
        const unsigned long long same = __ballot(act && g == gl);
        int base = 0;
        if (lane == leader) {
            base = atomicAdd(&pend_cnt[gl], __popcll(same));
            pend_touched[gl] = 1;
        }
        base = __builtin_amdgcn_readlane(base, leader);
        if (act && g == gl) slot = base + __popcll(same & ((1ull << lane) - 1ull));
        todo &= ~same;
    }
    if (act) {
        if (slot < cap) {
            pend_prompt[(size_t)g * cap + slot] = ctx0[i];
            pend_len[(size_t)g * cap + slot] = pred_len[i];
        } else {
            atomicOr(&counters[0], GR_DEV_ENTRIES_DROPPED);
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_commit_mark(int64_t n, const int* __restrict__ inst, int n_inst,
                                                        int* __restrict__ mark)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const int g = inst[i];
    if (g >= 0 && g < n_inst) mark[g] = 1;
}

__global__ __launch_bounds__(kBlock) void k_commit_place(int64_t n, const int* __restrict__ inst,
                                                         const int* __restrict__ ctx0, const int* __restrict__ pred_len,
                                                         int* __restrict__ mark, int* __restrict__ pend_cnt,
                                                         int* __restrict__ pend_prompt, int* __restrict__ pend_len,
                                                         int* __restrict__ pend_touched, int cap, int n_inst,
                                                         int* __restrict__ counters)
{
    const int lane = lane_id();
    const int g = blockIdx.x * kBuildWaves + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    if (g >= n_inst || !mark[g]) return;
    int base = pend_cnt[g];
    bool dropped = false;
    constexpr int kStep = 4;      // blocks of 64 requests in flight together
    for (int64_t i0 = 0; i0 < n; i0 += kStep * kWave) {
        int gi[kStep];
#pragma unroll
        for (int k = 0; k < kStep; ++k) {
            const int64_t i = i0 + k * kWave + lane;
            gi[k] = i < n ? inst[i] : -1;
        }
#pragma unroll
        for (int k = 0; k < kStep; ++k) {
            const unsigned long long m = __ballot(gi[k] == g);
            if (!m) continue;
            if (gi[k] == g) {
                const int64_t i = i0 + k * kWave + lane;
                const int slot = base + __popcll(m & ((1ull << lane) - 1ull));
                if (slot < cap) {
                    pend_prompt[(size_t)g * cap + slot] = ctx0[i];
                    pend_len[(size_t)g * cap + slot] = pred_len[i];
                } else {
                    dropped = true;
                }
            }
            base += __popcll(m);
        }
    }
    if (__ballot(dropped) && lane == 0) atomicOr(&counters[0], GR_DEV_ENTRIES_DROPPED);
    if (lane == 0) {
        pend_cnt[g] = base;
        pend_touched[g] = 1;
        mark[g] = 0;
    }
}

// LDS of a build that shares an instance between kSplit waves: contexts, two exchange buffers, totals
template <int kEPL, int kSplit>
constexpr size_t split_lds()
{
    return (size_t)(lean_inst_words(kWave * kEPL) + 2 * kWave * kEPL) * sizeof(int) + kSplit * 4 * sizeof(double);
}

template <int kEPL>
constexpr size_t lean_lds() { return (size_t)kBuildWaves * lean_inst_words(kWave * kEPL) * sizeof(int); }

constexpr int kSimds = 1024;      // 256 compute units of four

template <int kEPL, int kSplit>
void launch_build_split(const BuildArgs& b, int M, hipStream_t s)
{
    constexpr size_t lds = split_lds<kEPL, kSplit>();
    hipLaunchKernelGGL((k_build_lean<kEPL / kSplit, kSplit>), dim3(M), dim3(kSplit * kWave), lds, s, b);
}

// kEPL: sort words per lane if one wave takes an instance
template <int kEPL>
void launch_build(const BuildArgs& b, int M, hipStream_t s)
{
    const dim3 grid((M + kBuildWaves - 1) / kBuildWaves);
    const size_t lds = (size_t)kBuildWaves * kWave * kEPL * sizeof(int);
    if (b.batch_cap) {
        hipLaunchKernelGGL((k_build_capped<kEPL>), grid, dim3(kBlock), 3 * lds, s, b);
        return;
    }
    // fewer instances than the chip takes waves at four per SIMD: several waves per instance
    // (measured on 1 024 instances x 1 000 requests: 19.8 us with one wave each, 17.7 with two, 16.0 with
    // four, 18.0 with eight, 29 with sixteen; on 256 x 512: 9.2, 8.5, 7.7-8.2, 8.1)
    const int room = 4 * kSimds / M;
    if constexpr (kEPL >= 4) if (room >= 4) return launch_build_split<kEPL, 4>(b, M, s);
    if constexpr (kEPL >= 2) if (room >= 2) return launch_build_split<kEPL, 2>(b, M, s);
    hipLaunchKernelGGL((k_build_lean<kEPL, 1>), grid, dim3(kBlock), lean_lds<kEPL>(), s, b);
}

}  // namespace

int launch_commit(gr_fleet* f, int64_t n, const int* inst, const int* ctx0, const int* pred_len, hipStream_t s)
{
    if (n == 0) return GR_OK;
    if (n <= kWave) {
        hipLaunchKernelGGL(k_commit_wave, dim3(1), dim3(kWave), 0, s, (int)n, inst, ctx0, pred_len, f->pend_cnt,
                           f->pend_prompt, f->pend_len, f->pend_touched, f->cap, f->n_inst, f->counters);
    } else if (!f->has_cap) {
        hipLaunchKernelGGL(k_commit_any_order, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, n, inst,
                           ctx0, pred_len, f->pend_cnt, f->pend_prompt, f->pend_len, f->pend_touched, f->cap, f->n_inst,
                           f->counters);
    } else {
        hipLaunchKernelGGL(k_commit_mark, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, n, inst,
                           f->n_inst, f->commit_mark);
        hipLaunchKernelGGL(k_commit_place, dim3((f->n_inst + kBuildWaves - 1) / kBuildWaves), dim3(kBlock), 0, s, n, inst,
                           ctx0, pred_len, f->commit_mark, f->pend_cnt, f->pend_prompt, f->pend_len, f->pend_touched,
                           f->cap, f->n_inst, f->counters);
    }
    return hipGetLastError() == hipSuccess ? GR_OK : GR_ERR_HIP;
}

int launch_ema(gr_fleet* f, double w, const float* s_q, const float* s_p, const float* s_d, hipStream_t s)
{
    hipLaunchKernelGGL(k_ema, dim3((f->n_inst + kBlock - 1) / kBlock), dim3(kBlock), 0, s, f->n_inst, w, s_q, s_p, s_d,
                       !f->have_q, !f->have_p, !f->have_d, f->emaQ, f->emaP, f->emaD);
    if (hipGetLastError() != hipSuccess) return GR_ERR_HIP;
    f->have_q |= s_q != nullptr; f->have_p |= s_p != nullptr; f->have_d |= s_d != nullptr;
    return GR_OK;
}

// Dynamic LDS limits of the build kernels, set to what each needs at most (see score_prepare).
int status_prepare()
{
    bool ok = true;
    const auto set = [&](auto kernel, size_t bytes) {
        ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)bytes) == hipSuccess;
    };
    constexpr size_t word = kBuildWaves * kWave * sizeof(int);     // per sort word per lane
    set(k_build_lean<1, 1>, lean_lds<1>()); set(k_build_lean<2, 1>, lean_lds<2>()); set(k_build_lean<4, 1>, lean_lds<4>());
    set(k_build_lean<8, 1>, lean_lds<8>()); set(k_build_lean<16, 1>, lean_lds<16>()); set(k_build_lean<32, 1>, lean_lds<32>());
    set(k_build_lean<1, 2>, split_lds<2, 2>()); set(k_build_lean<2, 2>, split_lds<4, 2>());
    set(k_build_lean<4, 2>, split_lds<8, 2>()); set(k_build_lean<8, 2>, split_lds<16, 2>());
    set(k_build_lean<16, 2>, split_lds<32, 2>());
    set(k_build_lean<1, 4>, split_lds<4, 4>()); set(k_build_lean<2, 4>, split_lds<8, 4>());
    set(k_build_lean<4, 4>, split_lds<16, 4>()); set(k_build_lean<8, 4>, split_lds<32, 4>());
    set(k_build_capped<1>, 3 * word * 1); set(k_build_capped<2>, 3 * word * 2); set(k_build_capped<4>, 3 * word * 4);
    set(k_build_capped<8>, 3 * word * 8); set(k_build_capped<16>, 3 * word * 16); set(k_build_capped<32>, 3 * word * 32);
    return ok ? GR_OK : GR_ERR_HIP;
}

RankArgs rank_args(const gr_fleet* f, int* out_rank)
{
    RankArgs r{};
    r.d = f->hD; r.rank_acc = f->rank_acc; r.cls = f->cls; r.inst_class = f->inst_class;
    r.emaP = f->emaP; r.lam = f->lam_built;
    r.rank = f->rank; r.order = f->order; r.posK = f->posK; r.out_rank = out_rank;
    r.n_inst = f->n_inst; r.m_pad = f->m_pad;
    return r;
}

int launch_ranks(gr_fleet* f, int* out_rank, hipStream_t s)
{
    const RankArgs r = rank_args(f, out_rank);
    const int M = f->n_inst;
    {
        ProfScope ps(f, kRankCount, s);
        hipLaunchKernelGGL(k_rank_count, dim3((M + kWave - 1) / kWave, (M + kBlock - 1) / kBlock), dim3(kBlock), 0, s, r);
    }
    {
        ProfScope ps(f, kRankFinal, s);
        hipLaunchKernelGGL(k_rank_final, dim3((f->m_pad + kBlock - 1) / kBlock), dim3(kBlock), 0, s, r);
    }
    if (hipGetLastError() != hipSuccess) return GR_ERR_HIP;
    f->ranks_current = true;
    return GR_OK;
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
    b.tabR = f->tabR; b.tabGH = f->tabGH; b.headGH = f->headGH;
    b.hN = f->hN; b.hD = f->hD; b.act_inst = f->act_inst;
    b.rank_acc = f->rank_acc; b.counters = f->counters;
    b.n_active = in.n_active; b.n_queued = in.n_queued;
    b.n_inst = f->n_inst; b.max_entries = f->max_entries; b.max_len = f->max_len;
    b.pend_cnt = f->pend_cnt; b.pend_prompt = f->pend_prompt; b.pend_len = f->pend_len;
    b.use_pending = in.use_pending;
    b.pend_touched = f->pend_touched; b.only_touched = in.use_pending && in.only_touched;
    b.batch_cap = f->has_cap ? f->batch_cap : nullptr;
    b.lam = f->lam; b.emaQ = f->emaQ; b.emaP = f->emaP; b.emaD = f->emaD;
    const int M = f->n_inst;
    {
        ProfScope ps(f, kBuild, s);
        switch (f->epl) {
            case 1: launch_build<1>(b, M, s); break;
            case 2: launch_build<2>(b, M, s); break;
            case 4: launch_build<4>(b, M, s); break;
            case 8: launch_build<8>(b, M, s); break;
            case 16: launch_build<16>(b, M, s); break;
            default: launch_build<32>(b, M, s); break;
        }
    }
    // the capability order: now if the caller wants to see it, else with the next scoring pass
    f->ranks_current = false;
    f->lam_built = f->lam;
    if (in.out_rank) {
        const int rc = launch_ranks(f, in.out_rank, s);
        if (rc != GR_OK) return rc;
    }
    if (hipGetLastError() != hipSuccess) return GR_ERR_HIP;
    f->has_status = true;
    f->tables_current = true;
    if (!in.use_pending) f->last_in = in;     // what a later feedback routing rebuilds from
    return GR_OK;
}

}  // namespace gr
