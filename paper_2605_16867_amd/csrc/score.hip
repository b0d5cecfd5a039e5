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

// One workgroup walks the length histogram: the first slot of each length in
// grouped order, the list of lengths present ("rows"), the first tile of each
// row (a tile = up to kTileReq requests of one length), and the totals.  The
// histogram is cleared for the next call.
__global__ __launch_bounds__(kScanBlock) void k_scan(int* __restrict__ len_cnt, int* __restrict__ len_base,
                                                     int* __restrict__ row_len, int* __restrict__ row_off,
                                                     int* __restrict__ tile_off, int* __restrict__ totals,
                                                     int* __restrict__ out_n, int bins)
{
    __shared__ unsigned long long ws[kScanBlock / kWave];
    const int tid = threadIdx.x;
    unsigned long long c_req_tile = 0;   // requests in the low half, tiles in the high half
    unsigned long long c_row = 0;
    for (int base = 0; base < bins; base += kScanBlock) {
        const int L = base + tid;
        int c = 0;
        if (L < bins) { c = len_cnt[L]; len_cnt[L] = 0; }
        const unsigned long long tiles = (unsigned)(c + kTileReq - 1) / kTileReq;
        const unsigned long long mine = (unsigned long long)(unsigned)c | (tiles << 32);
        unsigned long long tot1, tot2;
        const unsigned long long in1 = block_incl_scan(mine, ws, tot1);
        const unsigned long long in2 = block_incl_scan(c > 0 ? 1ull : 0ull, ws, tot2);
        const unsigned long long ex1 = in1 - mine + c_req_tile;
        if (L < bins) len_base[L] = (int)(ex1 & 0xFFFFFFFFull);
        if (c > 0) {
            const int u = (int)(in2 - 1 + c_row);
            row_len[u] = L;
            row_off[u] = (int)(ex1 & 0xFFFFFFFFull);
            tile_off[u] = (int)(ex1 >> 32);
        }
        c_req_tile += tot1;
        c_row += tot2;
    }
    if (tid == 0) {
        const int n = (int)(c_req_tile & 0xFFFFFFFFull), U = (int)c_row, NT = (int)(c_req_tile >> 32);
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
    int n_inst, m_pad, tstride;
};

// (E, kappa) for kMemoU distinct lengths x kMemoP instances (consecutive
// positions of the capability order) per workgroup.  A wave takes one instance
// at a time, its lanes the lengths, and finds k = #{R_i <= L} by binary search
// in the instance's sorted lengths; the tile is turned in LDS so that the table
// is written in rows of positions.
__global__ __launch_bounds__(kBlock) void k_memo(MemoArgs a)
{
    __shared__ float2 tile[kMemoU][kMemoP + 1];
    const int U = a.totals[1];
    const int u0 = blockIdx.y * kMemoU;
    if (u0 >= U) return;
    const int p0 = blockIdx.x * kMemoP;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
    constexpr int kPerLane = kMemoU / kWave;
    int Lv[kPerLane];
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
        const int u = u0 + lane + kWave * i;
        Lv[i] = u < U ? a.row_len[u] : 0;
    }
#pragma unroll 1
    for (int j = 0; j < kMemoP / kWaves; ++j) {
        const int pi = wave * (kMemoP / kWaves) + j;
        const int p = p0 + pi;
        const int g = p < a.n_inst ? a.order[p] : -1;
        if (g >= 0) {
            const int N = a.hN[g];
            const double q = a.hQ[g];
            const ClassCoef cc = a.cls[a.inst_class[g]];
            const int* R = a.tabR + (size_t)g * a.tstride;
            const float* G = a.tabG + (size_t)g * a.tstride;
            const float* S = a.tabS + (size_t)g * a.tstride;
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) {
                const int L = Lv[i];
                int lo = 0, hi = N;
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (R[mid] <= L) lo = mid; else hi = mid - 1;
                }
                const double Ld = (double)L, n1 = (double)(N - lo + 1);
                const double tri = Ld * (Ld - 1.0) * 0.5;
                const double E = q + cc.alpha * Ld + cc.beta * (n1 * Ld) + (double)G[lo]
                                 + cc.gamma * (Ld * (double)S[lo] + n1 * tri);
                tile[lane + kWave * i][pi] = make_float2((float)E, (float)(cc.delta + cc.gamma * Ld));
            }
        } else {
#pragma unroll
            for (int i = 0; i < kPerLane; ++i)
                tile[lane + kWave * i][pi] = make_float2(__builtin_inff(), 0.f);
        }
    }
    __syncthreads();
    const int col = tid % kMemoP;
#pragma unroll 4
    for (int it = 0; it < kMemoU * kMemoP / kBlock; ++it) {
        const int ul = tid / kMemoP + (kBlock / kMemoP) * it;
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

__device__ inline float wave_min(float v)
{
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v = fminf(v, __shfl_xor(v, d, kWave));
    return v;
}

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

    int lo = 0, hi = U - 1;                 // row of this tile: last u with tile_off[u] <= t
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (a.tile_off[mid] <= t) lo = mid; else hi = mid - 1;
    }
    const int u = lo;
    const int r0 = a.row_off[u] + (t - a.tile_off[u]) * kTileReq;
    const int nreq = min(kTileReq, a.row_off[u + 1] - r0);

    ReqRec rec;
    rec.c0 = 0.f; rec.D = -__builtin_inff(); rec.pex = -1; rec.orig = -1;
    if (lane < nreq) rec = a.recs[r0 + lane];
    float c0[kTileReq], D[kTileReq], minT[kTileReq];
    int minB[kTileReq];
#pragma unroll
    for (int j = 0; j < kTileReq; ++j) {
        c0[j] = readlane_f(rec.c0, j);
        D[j] = fminf(readlane_f(rec.D, j), FLT_MAX);   // padded positions hold +inf and must stay infeasible
        minT[j] = __builtin_inff();
        minB[j] = 0;
    }
    unsigned notfound = (1u << nreq) - 1u;
    int foundP = -1;         // lane j: position of request j's first feasible instance
    float foundT = 0.f;

    const float2* row = a.memo + (size_t)u * a.m_pad;
    const int nblk = a.m_pad / kWave;
    const int ex_blk = rec.pex >= 0 ? rec.pex / kWave : -1;
    float2 next = row[lane];
    for (int b = 0; b < nblk; ++b) {
        const float2 cur = next;
        if (b + 1 < nblk) next = row[(b + 1) * kWave + lane];
        const unsigned hit = (unsigned)__ballot(ex_blk == b);   // requests whose excluded instance is here
        int g_lane = -1;
        if (kWriteT) g_lane = a.order[b * kWave + lane];
#pragma unroll
        for (int j = 0; j < kTileReq; ++j) {
            if (j < nreq) {
                float T = fmaf(c0[j], cur.y, cur.x);
                if (kWriteT) {
                    const int orig = __builtin_amdgcn_readlane(rec.orig, j);
                    if (g_lane >= 0) a.out_T[(size_t)orig * a.n_inst + g_lane] = T;
                }
                if ((hit >> j) & 1u) {
                    const int ex_lane = __builtin_amdgcn_readlane(rec.pex, j) & (kWave - 1);
                    if (lane == ex_lane) T = __builtin_inff();
                }
                const unsigned long long feas = __ballot(T <= D[j]);
                if (feas && ((notfound >> j) & 1u)) {
                    const int fl = __ffsll((long long)feas) - 1;
                    notfound &= ~(1u << j);
                    const float Tf = readlane_f(T, fl);
                    if (lane == j) { foundP = b * kWave + fl; foundT = Tf; }
                }
                if (T < minT[j]) { minT[j] = T; minB[j] = b; }
            }
        }
    }

    // fallback for requests with no feasible instance: smallest T, ties to the lowest instance
    int bestP = -1;
    float bestT = 0.f;
#pragma unroll
    for (int j = 0; j < kTileReq; ++j) {
        if (j < nreq && ((notfound >> j) & 1u)) {
            const float Tm = wave_min(minT[j]);
            unsigned long long cand = __ballot(minT[j] == Tm && Tm < __builtin_inff());
            int bp = -1, bg = 0x7fffffff;
            while (cand) {
                const int l = __ffsll((long long)cand) - 1;
                cand &= cand - 1;
                const int p = __builtin_amdgcn_readlane(minB[j], l) * kWave + l;
                const int g = a.order[p];
                if (g < bg) { bg = g; bp = p; }
            }
            if (lane == j) { bestP = bp; bestT = Tm; }
        }
    }
    if (lane < nreq) {
        const bool found = !((notfound >> lane) & 1u);
        const int p = found ? foundP : bestP;
        const float T = found ? foundT : bestT;
        const int g = p >= 0 ? a.order[p] : -1;
        a.out_inst[rec.orig] = g;
        a.out_slack[rec.orig] = g >= 0 ? rec.D - T : 0.f;
        if (a.out_fallback) a.out_fallback[rec.orig] = !found;
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

size_t score_lds_bytes(const gr_fleet* f) { return (size_t)f->bins * 4; }

int score_prepare(gr_fleet* f)
{
    const size_t hist = (size_t)((f->bins + 1) / 2) * 4, scat = (size_t)f->bins * 4;
    const bool ok = set_lds(k_hist<false>, hist) && set_lds(k_hist<true>, hist) &&
                    set_lds(k_scatter<false>, scat) && set_lds(k_scatter<true>, scat);
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
        hipLaunchKernelGGL(k_scan, dim3(1), dim3(kScanBlock), 0, s, f->len_cnt, f->len_base, f->row_len,
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
        m.n_inst = f->n_inst; m.m_pad = f->m_pad; m.tstride = f->tstride;
        ProfScope ps(f, kMemoRoute + off, s);
        hipLaunchKernelGGL(k_memo, dim3(f->m_pad / kMemoP, (unsigned)((max_rows + kMemoU - 1) / kMemoU)),
                           dim3(kBlock), 0, s, m);
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
