// Pair scoring (steps 2 and 3 of the path): Alg. 1 for a batch of requests
// against one snapshot of the instance tables.
//
// T(r,g) = E_g(L_r) + c0_r * kappa_g(L_r) (see common.h), and E, kappa depend on
// the request only through its length.  So a batch is first grouped by length
// (a counting sort over the lengths present), E and kappa are looked up once per
// (distinct length, instance) by binary search in the instance's sorted
// lengths, and every (request, instance) pair then costs one multiply-add, the
// feasibility compare and the running selections of Alg. 1.
//
// Instances are visited in capability order (largest d_g first), 64 per wave
// step, one per lane; the requests of a tile are wave-uniform scalars.  The
// just-enough choice (feasible instance of largest d_g) is then the first set
// bit of the feasibility ballot of the first block that has one; the fallback
// (smallest T) is a per-lane running minimum reduced across the wave at the end.
#include <cfloat>

#include "common.h"

namespace gr {
namespace {

template <bool kMigrate>
__device__ inline bool fetch_len(const ReqSrc& s, int64_t i, int max_len, int& L)
{
    if (kMigrate) {
        if (!s.flag[i]) return false;
        L = s.act_rem[i];
    } else {
        L = s.pred_len[i];
    }
    L = min(max(L, 0), max_len);
    return true;
}

// ------------------------------------------------------------------ grouping by length
// Requests per length: a histogram private to the workgroup in LDS (two 16-bit
// counters per word: a workgroup sees at most kGroupChunk requests), then one
// global atomic per length the workgroup has seen.
template <bool kMigrate>
__global__ __launch_bounds__(kBlock) void k_hist(ReqSrc s, int* __restrict__ len_cnt, int bins, int max_len)
{
    extern __shared__ uint32_t lds[];
    const int tid = threadIdx.x;
    const int nwords = (bins + 1) / 2;
    for (int w = tid; w < nwords; w += kBlock) lds[w] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kGroupChunk;
#pragma unroll
    for (int it = 0; it < kGroupItems; ++it) {
        const int64_t i = base + it * kBlock + tid;
        int L;
        if (i < s.n && fetch_len<kMigrate>(s, i, max_len, L))
            atomicAdd(&lds[L >> 1], (L & 1) ? 0x10000u : 1u);
    }
    __syncthreads();
    for (int w = tid; w < nwords; w += kBlock) {
        const uint32_t v = lds[w];
        if (v & 0xFFFFu) atomicAdd(&len_cnt[2 * w], (int)(v & 0xFFFFu));
        if (v >> 16) atomicAdd(&len_cnt[2 * w + 1], (int)(v >> 16));
    }
}

constexpr int kScanBlock = 1024;

// Inclusive scan over the workgroup; `ws` holds one slot per wave.
__device__ inline unsigned long long block_incl_scan(unsigned long long v, unsigned long long* ws,
                                                     unsigned long long& total)
{
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    v = wave_incl_scan(v);
    __syncthreads();
    if (lane == kWave - 1) ws[wave] = v;
    __syncthreads();
    unsigned long long before = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < kScanBlock / kWave; ++w) {
        const unsigned long long x = ws[w];
        if (w < wave) before += x;
        total += x;
    }
    return v + before;
}

// One workgroup walks the length histogram (copied to LDS; a thread owns a run
// of consecutive lengths): the first slot of each length in grouped order, the
// list of lengths present ("rows"), the first tile of each row (a tile = up to
// kTileReq requests of one length), and the totals.  The histogram is cleared
// for the next call.
__global__ __launch_bounds__(kScanBlock) void k_scan(int* __restrict__ len_cnt, int* __restrict__ len_base,
                                                     int* __restrict__ row_len, int* __restrict__ row_off,
                                                     int* __restrict__ tile_off, int* __restrict__ totals,
                                                     int* __restrict__ out_n, int bins)
{
    extern __shared__ uint32_t lds[];
    int* cnt = reinterpret_cast<int*>(lds);
    __shared__ unsigned long long ws[kScanBlock / kWave];
    const int tid = threadIdx.x;
    for (int i = tid; i < bins; i += kScanBlock) { cnt[i] = len_cnt[i]; len_cnt[i] = 0; }
    __syncthreads();
    const int per = ((bins + kScanBlock - 1) / kScanBlock) | 1;   // odd: no LDS bank conflicts
    const int i0 = min(tid * per, bins), i1 = min(i0 + per, bins);
    unsigned long long mine = 0, rows = 0;     // requests in the low half, tiles in the high half
    for (int i = i0; i < i1; ++i) {
        const unsigned c = (unsigned)cnt[i];
        mine += (unsigned long long)c | ((unsigned long long)((c + kTileReq - 1) / kTileReq) << 32);
        rows += c > 0;
    }
    unsigned long long tot1, tot2;
    unsigned long long run = block_incl_scan(mine, ws, tot1) - mine;
    int u = (int)(block_incl_scan(rows, ws, tot2) - rows);
    for (int i = i0; i < i1; ++i) {
        const unsigned c = (unsigned)cnt[i];
        cnt[i] = (int)(run & 0xFFFFFFFFull);
        if (c) {
            row_len[u] = i;
            row_off[u] = (int)(run & 0xFFFFFFFFull);
            tile_off[u] = (int)(run >> 32);
            ++u;
        }
        run += (unsigned long long)c | ((unsigned long long)((c + kTileReq - 1) / kTileReq) << 32);
    }
    __syncthreads();
    for (int i = tid; i < bins; i += kScanBlock) len_base[i] = cnt[i];
    if (tid == 0) {
        const int n = (int)(tot1 & 0xFFFFFFFFull), U = (int)tot2, NT = (int)(tot1 >> 32);
        row_off[U] = n;
        tile_off[U] = NT;
        totals[0] = n; totals[1] = U; totals[2] = NT;
        if (out_n) *out_n = n;
    }
}

// Requests into grouped order.  Per workgroup: count per length in LDS, reserve
// that many slots of each length with one global atomic, hand the slots out.
template <bool kMigrate>
__global__ __launch_bounds__(kBlock) void k_scatter(ReqSrc s, int* __restrict__ len_base,
                                                    const int* __restrict__ rank, ReqRec* __restrict__ recs,
                                                    int* __restrict__ out_inst, float* __restrict__ out_slack,
                                                    int bins, int max_len, int n_inst)
{
    extern __shared__ uint32_t lds[];
    int* slot = reinterpret_cast<int*>(lds);
    const int tid = threadIdx.x;
    for (int L = tid; L < bins; L += kBlock) slot[L] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kGroupChunk;
    int Ls[kGroupItems];
#pragma unroll
    for (int it = 0; it < kGroupItems; ++it) {
        const int64_t i = base + it * kBlock + tid;
        int L = -1;
        if (i < s.n) {
            if (fetch_len<kMigrate>(s, i, max_len, L)) {
                atomicAdd(&slot[L], 1);
            } else {
                L = -1;
                out_inst[i] = -1;       // not flagged: no migration target
                out_slack[i] = 0.f;
            }
        }
        Ls[it] = L;
    }
    __syncthreads();
    for (int L = tid; L < bins; L += kBlock) {
        const int c = slot[L];
        if (c) slot[L] = atomicAdd(&len_base[L], c);
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kGroupItems; ++it) {
        const int L = Ls[it];
        if (L < 0) continue;
        const int64_t i = base + it * kBlock + tid;
        const int pos = atomicAdd(&slot[L], 1);
        int c0, ex;
        float D;
        if (kMigrate) {
            c0 = s.act_prompt[i] + s.act_gen[i]; D = s.act_budget[i]; ex = s.act_inst[i];
        } else {
            c0 = s.ctx0[i]; D = s.budget[i]; ex = s.exclude ? s.exclude[i] : -1;
        }
        ReqRec r;
        r.c0 = (float)c0; r.D = D;
        r.pex = (ex >= 0 && ex < n_inst) ? rank[ex] : -1;
        r.orig = (int)i;
        recs[pos] = r;
    }
}

// ------------------------------------------------------------------ closed-form lookups
struct MemoArgs {
    const int *totals, *row_len, *order, *hN;
    const double* hQ;
    const ClassCoef* cls;
    const int* inst_class;
    const int* tabR;
    const float *tabG, *tabS;
    float2* memo;
    int n_inst, m_pad, tstride, lds_stride;
};

// (E, kappa) for kMemoU distinct lengths x kMemoP instances (consecutive
// positions of the capability order) per workgroup of kMemoP waves.  A wave
// takes one instance: it copies the instance's sorted lengths to LDS, its lanes
// take the request lengths and find k = #{R_i <= L} by binary search there; the
// tile is turned in LDS so that the table is written in rows of positions.
constexpr int kMemoBlock = kMemoP * kWave;

__global__ __launch_bounds__(kMemoBlock) void k_memo(MemoArgs a)
{
    extern __shared__ uint32_t lds[];
    __shared__ float2 tile[kMemoU][kMemoP + 1];
    const int U = a.totals[1];
    const int u0 = blockIdx.y * kMemoU;
    if (u0 >= U) return;
    const int p0 = blockIdx.x * kMemoP;
    const int tid = threadIdx.x, lane = lane_id(), pi = tid / kWave;
    // this wave's copy, 16 bits per length (lengths are below 32768)
    uint16_t* sR = reinterpret_cast<uint16_t*>(lds) + (size_t)pi * a.lds_stride;
    constexpr int kPerLane = kMemoU / kWave;
    const int p = p0 + pi;
    const int g = p < a.n_inst ? a.order[p] : -1;
    if (g >= 0) {
        const int N = a.hN[g];
        const int* R = a.tabR + (size_t)g * a.tstride;
        for (int k = lane; k <= N; k += kWave) sR[k] = (uint16_t)R[k];
        int Lv[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int u = u0 + lane + kWave * i;
            Lv[i] = u < U ? a.row_len[u] : 0;
        }
        const double q = a.hQ[g];
        const ClassCoef cc = a.cls[a.inst_class[g]];
        const float* G = a.tabG + (size_t)g * a.tstride;
        const float* S = a.tabS + (size_t)g * a.tstride;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        int kk[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            int lo = 0, hi = N;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if ((int)sR[mid] <= Lv[i]) lo = mid; else hi = mid - 1;
            }
            kk[i] = lo;
        }
        float Gv[kPerLane], Sv[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) { Gv[i] = G[kk[i]]; Sv[i] = S[kk[i]]; }
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const double Ld = (double)Lv[i], n1 = (double)(N - kk[i] + 1);
            const double tri = Ld * (Ld - 1.0) * 0.5;
            const double E = q + cc.alpha * Ld + cc.beta * (n1 * Ld) + (double)Gv[i]
                             + cc.gamma * (Ld * (double)Sv[i] + n1 * tri);
            tile[lane + kWave * i][pi] = make_float2((float)E, (float)(cc.delta + cc.gamma * Ld));
        }
    } else {
#pragma unroll
        for (int i = 0; i < kPerLane; ++i)
            tile[lane + kWave * i][pi] = make_float2(__builtin_inff(), 0.f);
    }
    __syncthreads();
    const int col = tid % kMemoP;
#pragma unroll
    for (int it = 0; it < kMemoU * kMemoP / kMemoBlock; ++it) {
        const int ul = tid / kMemoP + (kMemoBlock / kMemoP) * it;
        const int u = u0 + ul;
        if (u < U) a.memo[(size_t)u * a.m_pad + p0 + col] = tile[ul][col];
    }
}

// ------------------------------------------------------------------ Alg. 1 over tiles
struct TileArgs {
    const int *totals, *row_off, *tile_off, *order;
    const ReqRec* recs;
    const float2* memo;
    int* out_inst;
    float* out_slack;
    uint8_t* out_fallback;
    float* out_T;
    int n_inst, m_pad;
};

__device__ inline float readlane_f(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// One step of a wave-wide minimum: combine with the lane selected by a DPP control.
template <int kCtrl, int kRowMask>
__device__ inline float min_dpp(float v)
{
    const int t = __builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), kCtrl, kRowMask, 0xf, false);
    const float o = __int_as_float(t);
    return o < v ? o : v;
}

// Minimum over the 64 lanes (no NaNs among the inputs).  Prefix minima inside
// each row of 16 lanes (row_shr 1, 2, 4, 8), then lane 15 of rows 0 and 2 into
// rows 1 and 3, then lane 31 into rows 2 and 3: lane 63 holds the result.
__device__ inline float wave_min(float v)
{
    v = min_dpp<0x111, 0xf>(v);
    v = min_dpp<0x112, 0xf>(v);
    v = min_dpp<0x114, 0xf>(v);
    v = min_dpp<0x118, 0xf>(v);
    v = min_dpp<0x142, 0xa>(v);
    v = min_dpp<0x143, 0xc>(v);
    return readlane_f(v, kWave - 1);
}

struct TileState {
    float c0[kTileReq];     // same in every lane: tokens to prefill of request j (0 past the tile's last request)
    float D[kTileReq];      // same in every lane: budget of request j; -inf once its instance is found
    float minT[kTileReq];   // per lane: smallest T of request j over the blocks seen
    int minB[kTileReq];     // per lane: the block it was seen in
    unsigned notfound;      // bit j: request j has no feasible instance so far
    int foundP;             // lane j: position of request j's first feasible instance
    float foundT;           // lane j: its T
};

// Request j has feasible instances in block b (lanes `feas`): the first one in
// capability order is its just-enough choice.
__device__ inline void record_found(TileState& st, int j, int b, unsigned long long feas, float T, int lane)
{
    const int fl = __ffsll((long long)feas) - 1;
    const float Tf = readlane_f(T, fl);
    if (lane == j) { st.foundP = b * kWave + fl; st.foundT = Tf; }
    st.notfound &= ~(1u << j);
    st.D[j] = -__builtin_inff();
}

// One block of 64 instances against the tile's requests: per pair one
// multiply-add, the feasibility compare and the running minimum (5 vector
// operations).  Feasibility is only OR-ed here and looked at per request when
// the block has any.
__device__ inline void block_step(TileState& st, int b, float2 cur, int lane)
{
    unsigned long long anyf = 0;
#pragma unroll
    for (int j = 0; j < kTileReq; ++j) {
        const float T = fmaf(st.c0[j], cur.y, cur.x);
        anyf |= __ballot(T <= st.D[j]);
        const bool lt = T < st.minT[j];
        st.minB[j] = lt ? b : st.minB[j];
        st.minT[j] = lt ? T : st.minT[j];
    }
    if (anyf) {
        // rare: recomputed from opaque copies so that nothing of it stays live in the loop above
        asm volatile("" : "+v"(cur.x), "+v"(cur.y));
#pragma unroll
        for (int j = 0; j < kTileReq; ++j) {
            const float T = fmaf(st.c0[j], cur.y, cur.x);
            const unsigned long long feas = __ballot(T <= st.D[j]);
            if (feas) {
                // the first feasible instance in capability order is the just-enough choice
                const int fl = __ffsll((long long)feas) - 1;
                const float Tf = readlane_f(T, fl);
                if (lane == j) { st.foundP = b * kWave + fl; st.foundT = Tf; }
                st.notfound &= ~(1u << j);
                st.D[j] = -__builtin_inff();
            }
        }
    }
}

// Smallest T of one request over the wave: position (ties to the lowest instance) and value.
__device__ inline void wave_argmin(float minT, int minB, const int* __restrict__ order, int& pos, float& val)
{
    const float Tm = wave_min(minT);
    unsigned long long cand = __ballot(minT == Tm && Tm < __builtin_inff());
    int bp = -1, bg = 0x7fffffff;
    while (cand) {
        const int l = __ffsll((long long)cand) - 1;
        cand &= cand - 1;
        const int p = __builtin_amdgcn_readlane(minB, l) * kWave + l;
        const int g = order[p];
        if (g < bg) { bg = g; bp = p; }
    }
    pos = bp;
    val = Tm;
}

// One request on its own against all instances but the one at position `pex`:
// used when the choice made without the exclusion fell on the excluded instance.
__device__ inline void rescan_excluding(const float2* __restrict__ row, int nblk, float c0, float D, int pex,
                                        const int* __restrict__ order, int lane, int& pos, float& val, bool& found)
{
    float minT = __builtin_inff();
    int minB = 0;
    found = false;
    pos = -1;
    val = 0.f;
    for (int b = 0; b < nblk; ++b) {
        const float2 cur = row[b * kWave + lane];
        float T = fmaf(c0, cur.y, cur.x);
        if (b * kWave + lane == pex) T = __builtin_inff();
        const unsigned long long feas = __ballot(T <= D);
        if (feas) {
            const int fl = __ffsll((long long)feas) - 1;
            pos = b * kWave + fl;
            val = readlane_f(T, fl);
            found = true;
            return;
        }
        const bool lt = T < minT;
        minB = lt ? b : minB;
        minT = lt ? T : minT;
    }
    wave_argmin(minT, minB, order, pos, val);
}

// One wave per tile: up to kTileReq requests of one length against all
// instances, 64 instances (one block of the capability order) per step.
// Excluded instances are ignored in the main pass; a request whose choice
// falls on its excluded instance is scored again on its own.
template <bool kWriteT>
__global__ __launch_bounds__(kBlock) void k_tile(TileArgs a)
{
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int NT = a.totals[2], U = a.totals[1];
    // consecutive tiles share a table row: keep them on one XCD (workgroups go round-robin over 8)
    const int per_xcd = gridDim.x >> 3;
    const int bid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    const int t = bid * kWaves + wave;
    if (t >= NT) return;

    // row of this tile: the last u with tile_off[u] <= t, by a 64-way search
    int lo = 0, len = U;
    while (len > 1) {
        const int stride = (len + kWave - 1) / kWave;
        const int idx = lo + lane * stride;
        const bool le = idx < lo + len && a.tile_off[idx] <= t;
        const int cnt = __popcll(__ballot(le));
        const int nlo = lo + (cnt - 1) * stride;
        len = min(stride, lo + len - nlo);
        lo = nlo;
    }
    const int u = lo;
    const int r0 = a.row_off[u] + (t - a.tile_off[u]) * kTileReq;
    const int nreq = min(kTileReq, a.row_off[u + 1] - r0);

    // lanes past the tile's last request carry a dummy that is never feasible and never reported
    ReqRec rec;
    rec.c0 = 0.f; rec.D = -__builtin_inff(); rec.pex = -1; rec.orig = -1;
    if (lane < nreq) rec = a.recs[r0 + lane];
    // padded positions hold T = +inf and must stay infeasible even for D = +inf; a NaN budget is never met
    const float Dc = rec.D > FLT_MAX ? FLT_MAX : rec.D;
    TileState st;
#pragma unroll
    for (int j = 0; j < kTileReq; ++j) {
        st.c0[j] = readlane_f(rec.c0, j);
        st.D[j] = readlane_f(Dc, j);
        // keep both in vector registers: the scalar file is too small for 16 requests
        asm volatile("" : "+v"(st.c0[j]), "+v"(st.D[j]));
        st.minT[j] = __builtin_inff();
        st.minB[j] = 0;
    }
    st.notfound = (1u << nreq) - 1u;
    st.foundP = -1;
    st.foundT = 0.f;

    const float2* __restrict__ row = a.memo + (size_t)u * a.m_pad;
    const int nblk = a.m_pad / kWave;
    float2 next = row[lane];
    for (int b = 0; b < nblk; ++b) {
        const float2 cur = next;
        if (b + 1 < nblk) next = row[(b + 1) * kWave + lane];
        block_step(st, b, cur, lane);
    }

    // requests with no feasible instance fall back to the smallest T
    int bestP = -1;
    float bestT = 0.f;
#pragma unroll
    for (int j = 0; j < kTileReq; ++j) {
        if ((st.notfound >> j) & 1u) {
            int bp;
            float bt;
            wave_argmin(st.minT[j], st.minB[j], a.order, bp, bt);
            if (lane == j) { bestP = bp; bestT = bt; }
        }
    }
    bool found = !((st.notfound >> lane) & 1u);
    int p = found ? st.foundP : bestP;
    float T = found ? st.foundT : bestT;

    // choices that fell on the request's excluded instance
    unsigned long long redo = __ballot(lane < nreq && rec.pex >= 0 && p == rec.pex);
    while (redo) {
        const int j = __ffsll((long long)redo) - 1;
        redo &= redo - 1;
        int rp;
        float rt;
        bool rf;
        rescan_excluding(row, nblk, readlane_f(rec.c0, j), readlane_f(Dc, j),
                         __builtin_amdgcn_readlane(rec.pex, j), a.order, lane, rp, rt, rf);
        if (lane == j) { p = rp; T = rt; found = rf; }
    }

    if (lane < nreq) {
        const int g = p >= 0 ? a.order[p] : -1;
        a.out_inst[rec.orig] = g;
        a.out_slack[rec.orig] = g >= 0 ? rec.D - T : 0.f;
        if (a.out_fallback) a.out_fallback[rec.orig] = !found;
    }

    if (kWriteT) {   // every pair's latency, for checking: same arithmetic, exclusions not applied
        for (int b = 0; b < nblk; ++b) {
            const float2 cur = row[b * kWave + lane];
            const int g_lane = a.order[b * kWave + lane];
            for (int j = 0; j < nreq; ++j) {
                const int orig = __builtin_amdgcn_readlane(rec.orig, j);
                const float Tj = fmaf(readlane_f(rec.c0, j), cur.y, cur.x);
                if (g_lane >= 0) a.out_T[(size_t)orig * a.n_inst + g_lane] = Tj;
            }
        }
    }
}

__global__ void k_set_int(int* p, int v) { *p = v; }

template <typename K>
bool set_lds(K kernel, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess;
}

}  // namespace

int memo_lds_stride(const gr_fleet* f) { return (f->tstride + 1) & ~1; }

size_t memo_lds_bytes(const gr_fleet* f) { return (size_t)kMemoP * memo_lds_stride(f) * 2; }

size_t score_lds_bytes(const gr_fleet* f)
{
    const size_t group = (size_t)f->bins * 4;
    const size_t memo = memo_lds_bytes(f) + sizeof(float2) * kMemoU * (kMemoP + 1);
    return group > memo ? group : memo;
}

int score_prepare(gr_fleet* f)
{
    const size_t hist = (size_t)((f->bins + 1) / 2) * 4, scat = (size_t)f->bins * 4;
    const bool ok = set_lds(k_hist<false>, hist) && set_lds(k_hist<true>, hist) &&
                    set_lds(k_scatter<false>, scat) && set_lds(k_scatter<true>, scat) &&
                    set_lds(k_scan, scat) && set_lds(k_memo, memo_lds_bytes(f));
    return ok ? GR_OK : GR_ERR_HIP;
}

int launch_score(gr_fleet* f, const ReqSrc& src, bool migrate, const ScoreOut& out, hipStream_t s)
{
    const int64_t n = src.n;
    if (n == 0) {
        if (out.n_selected) hipLaunchKernelGGL(k_set_int, dim3(1), dim3(1), 0, s, out.n_selected, 0);
        return hipGetLastError() == hipSuccess ? GR_OK : GR_ERR_HIP;
    }
    const int bins = f->bins;
    const unsigned g_blocks = (unsigned)((n + kGroupChunk - 1) / kGroupChunk);
    const size_t hist_lds = (size_t)((bins + 1) / 2) * 4, scat_lds = (size_t)bins * 4;
    const int off = migrate ? kHistMigrate - kHistRoute : 0;
    {
        ProfScope ps(f, kHistRoute + off, s);
        if (migrate) hipLaunchKernelGGL(k_hist<true>, dim3(g_blocks), dim3(kBlock), hist_lds, s, src, f->len_cnt, bins, f->max_len);
        else hipLaunchKernelGGL(k_hist<false>, dim3(g_blocks), dim3(kBlock), hist_lds, s, src, f->len_cnt, bins, f->max_len);
    }
    {
        ProfScope ps(f, kScanRoute + off, s);
        hipLaunchKernelGGL(k_scan, dim3(1), dim3(kScanBlock), scat_lds, s, f->len_cnt, f->len_base, f->row_len,
                           f->row_off, f->tile_off, f->totals, out.n_selected, bins);
    }
    {
        ProfScope ps(f, kScatterRoute + off, s);
        if (migrate) hipLaunchKernelGGL(k_scatter<true>, dim3(g_blocks), dim3(kBlock), scat_lds, s, src, f->len_base,
                                        f->rank, f->recs, out.inst, out.slack, bins, f->max_len, f->n_inst);
        else hipLaunchKernelGGL(k_scatter<false>, dim3(g_blocks), dim3(kBlock), scat_lds, s, src, f->len_base,
                                f->rank, f->recs, out.inst, out.slack, bins, f->max_len, f->n_inst);
    }
    const int64_t max_rows = n < bins ? n : bins;
    {
        MemoArgs m{};
        m.totals = f->totals; m.row_len = f->row_len; m.order = f->order; m.hN = f->hN; m.hQ = f->hQ;
        m.cls = f->cls; m.inst_class = f->inst_class;
        m.tabR = f->tabR; m.tabG = f->tabG; m.tabS = f->tabS; m.memo = f->memo;
        m.n_inst = f->n_inst; m.m_pad = f->m_pad; m.tstride = f->tstride; m.lds_stride = memo_lds_stride(f);
        ProfScope ps(f, kMemoRoute + off, s);
        hipLaunchKernelGGL(k_memo, dim3(f->m_pad / kMemoP, (unsigned)((max_rows + kMemoU - 1) / kMemoU)),
                           dim3(kMemoBlock), memo_lds_bytes(f), s, m);
    }
    {
        TileArgs t{};
        t.totals = f->totals; t.row_off = f->row_off; t.tile_off = f->tile_off; t.order = f->order;
        t.recs = f->recs; t.memo = f->memo;
        t.out_inst = out.inst; t.out_slack = out.slack; t.out_fallback = out.fallback; t.out_T = out.T;
        t.n_inst = f->n_inst; t.m_pad = f->m_pad;
        const int64_t max_tiles = (n + kTileReq - 1) / kTileReq + max_rows;
        unsigned blocks = (unsigned)((max_tiles + kWaves - 1) / kWaves);
        blocks = (blocks + 7u) & ~7u;
        ProfScope ps(f, kTileRoute + off, s);
        if (out.T) hipLaunchKernelGGL(k_tile<true>, dim3(blocks), dim3(kBlock), 0, s, t);
        else hipLaunchKernelGGL(k_tile<false>, dim3(blocks), dim3(kBlock), 0, s, t);
    }
    return hipGetLastError() == hipSuccess ? GR_OK : GR_ERR_HIP;
}

}  // namespace gr
