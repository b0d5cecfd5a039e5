// Pair scoring (steps 2 and 3 of the path): Alg. 1 for a batch of requests
// against one snapshot of the instance tables.
//
// T(r,g) = E_g(L_r) + c0_r * kappa_g(L_r) (see common.h), and E, kappa depend on
// the request only through its length.  So a batch is first grouped by length
// (a counting sort over the lengths present), E is tabulated once per (distinct
// length, instance) from the instance's sorted lengths (by counting: the
// lengths of the batch are sorted too), and every (request, instance) pair then
// costs one multiply-add and half a three-way minimum.
//
// Instances sit in capability order (largest d_g first), 64 per wave step, one
// per lane; the requests of a tile are wave-uniform scalars.  A pair only
// enters its request's running minimum per lane: Alg. 1's feasible set is
// non-empty exactly when the least latency meets the deadline, the just-enough
// choice (feasible instance of largest d_g) is then the first feasible position
// in capability order, found with bounds over runs of 16 positions, and the
// fallback (smallest T) is the position of the minimum.
//
// A batch of a few requests skips grouping and table: a thread per pair with
// its own binary search (k_direct).
#include <cfloat>
#include <mutex>

#include "common.h"

// The running selections of the pair-by-pair pass for callers that may not allocate: a fixed
// array in the library's own device image (each GPU the library runs on holds a copy of it
// until the process ends).  Host code never uses this name as an address: it asks the runtime
// for the array's address on the current device once (static_scratch below) and passes that.
static __device__ __align__(256) unsigned long long scratch[2 * gr::kDirectMax];

namespace gr {
namespace {

// Length of request i (0 <= i < s.n) and whether it takes part (a migration pass scores the flagged
// requests only).  Both reads are in bounds whatever the flag says, so neither waits for the other,
// and a caller that reads several requests has all its loads in flight together.
template <bool kMigrate>
__device__ __forceinline__ bool fetch_len(const ReqSrc& s, int64_t i, int max_len, int& L)
{
    const int raw = kMigrate ? s.act_rem[i] : s.pred_len[i];
    const bool takes_part = !kMigrate || s.flag[i] != 0;
    L = min(max(raw, 0), max_len);
    return takes_part;
}

// ------------------------------------------------------------------ grouping by length
// Requests per length: a histogram private to the workgroup in LDS (two 16-bit
// counters per word: a workgroup sees at most 1024 * kItems < 65536 requests), then one
// global atomic per length the workgroup has seen.
//
// Workgroups past the first `hist_blocks` do something else that has to happen before the
// requests are put in order and costs a launch of its own otherwise: the counting step of the
// capability order (tile b of `rank_bx` x .. tiles, see rank_count_tile; none when rank_bx = 0).
template <bool kMigrate, int kItems>
__global__ __launch_bounds__(kGroupBlock) void k_hist(ReqSrc s, int* __restrict__ len_cnt, int bins, int max_len,
                                                      int hist_blocks, RankArgs ranks, int rank_bx)
{
    extern __shared__ uint32_t lds[];
    if ((int)blockIdx.x >= hist_blocks) {
        const int b = blockIdx.x - hist_blocks;
        rank_count_tile<kGroupBlock>(ranks, b % rank_bx, b / rank_bx, reinterpret_cast<double*>(lds));
        return;
    }
    const int tid = threadIdx.x;
    const int nwords = (bins + 1) / 2;
    for (int w = tid; w < nwords; w += kGroupBlock) lds[w] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * (kGroupBlock * kItems);
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t i = base + it * kGroupBlock + tid;
        int L;
        if (i < s.n && fetch_len<kMigrate>(s, i, max_len, L))
            atomicAdd(&lds[L >> 1], (L & 1) ? 0x10000u : 1u);
    }
    __syncthreads();
    for (int w = tid; w < nwords; w += kGroupBlock) {
        const uint32_t v = lds[w];
        if (v & 0xFFFFu) atomicAdd(&len_cnt[2 * w], (int)(v & 0xFFFFu));
        if (v >> 16) atomicAdd(&len_cnt[2 * w + 1], (int)(v >> 16));
    }
}

constexpr int kScanBlock = 1024;
constexpr int kScanWaves = kScanBlock / kWave;
constexpr int kScanGroups = 16;     // workgroups
constexpr int kScanChunks = 2;      // blocks of 64 lengths per wave
static_assert(kMaxLen + 1 <= kWave * kScanChunks * kScanWaves * kScanGroups, "every length has a lane of some wave");

// Prefix sums over the length histogram: the first slot of each length in
// grouped order, the list of lengths present ("rows") and the row of each such
// length, the first tile of each row (a tile = up to kTileReq requests of one
// length), and the totals.  A wave owns one or two blocks of 64 consecutive
// lengths (lane = length within the block, so every access is a row of
// consecutive addresses).  The histogram is small and sits in L2, so instead
// of passing sums from workgroup to workgroup each workgroup adds up
// everything before its own lengths itself; the last one also has the totals.
// The histogram is left as it is (the scatter clears it for the next call).
// Workgroups past the first kScanGroups finish the capability order (rank_final_item), whose
// counts the previous launch completed.
__global__ __launch_bounds__(kScanBlock) void k_scan(const int* __restrict__ len_cnt, int* __restrict__ len_base,
                                                     int* __restrict__ row_len, int* __restrict__ row_off,
                                                     int* __restrict__ tile_off, int* __restrict__ len_row,
                                                     int* __restrict__ len_ceil, int* __restrict__ totals,
                                                     int* __restrict__ out_n, int bins, RankArgs ranks)
{
    __shared__ int w_req[2][kScanWaves], w_tile[2][kScanWaves], w_rows[2][kScanWaves];
    if (blockIdx.x >= kScanGroups) {
        rank_final_item(ranks, (blockIdx.x - kScanGroups) * kScanBlock + threadIdx.x);
        return;
    }
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int chunks = (bins + kWave - 1) / kWave;
    const int per = (chunks + kScanWaves * kScanGroups - 1) / (kScanWaves * kScanGroups);    // 1 or 2
    const int first = min((int)blockIdx.x * kScanWaves * per * kWave, bins);    // first length of this workgroup
    const auto tiles_of = [](int c) { return (c + kTileReq - 1) / kTileReq; };
    const auto wave_total = [](int v) { return __builtin_amdgcn_readlane(wave_incl_scan_i32(v), kWave - 1); };

    // everything before this workgroup's lengths, a slice per thread
    int b_req = 0, b_tile = 0, b_rows = 0;
#pragma unroll 8
    for (int i = threadIdx.x; i < first; i += kScanBlock) {
        const int c = len_cnt[i];
        b_req += c; b_tile += tiles_of(c); b_rows += c > 0;
    }
    // this wave's own lengths
    int cnt[kScanChunks], m_req = 0, m_tile = 0, m_rows = 0;
#pragma unroll
    for (int k = 0; k < kScanChunks; ++k) {
        const int i = first + (wave * per + k) * kWave + lane;
        cnt[k] = k < per && i < bins ? len_cnt[i] : 0;
        m_req += cnt[k]; m_tile += tiles_of(cnt[k]); m_rows += cnt[k] > 0;
    }
    b_req = wave_total(b_req); b_tile = wave_total(b_tile); b_rows = wave_total(b_rows);
    m_req = wave_total(m_req); m_tile = wave_total(m_tile); m_rows = wave_total(m_rows);
    if (lane == 0) {
        w_req[0][wave] = b_req; w_tile[0][wave] = b_tile; w_rows[0][wave] = b_rows;
        w_req[1][wave] = m_req; w_tile[1][wave] = m_tile; w_rows[1][wave] = m_rows;
    }
    __syncthreads();
    int at_req = 0, at_tile = 0, u = 0, all_req = 0, all_tile = 0, all_rows = 0;
#pragma unroll
    for (int w = 0; w < kScanWaves; ++w) {
        const int before_r = w_req[0][w], before_t = w_tile[0][w], before_u = w_rows[0][w];
        const int own_r = w_req[1][w], own_t = w_tile[1][w], own_u = w_rows[1][w];
        at_req += before_r + (w < wave ? own_r : 0);
        at_tile += before_t + (w < wave ? own_t : 0);
        u += before_u + (w < wave ? own_u : 0);
        all_req += before_r + own_r; all_tile += before_t + own_t; all_rows += before_u + own_u;
    }

    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int k = 0; k < kScanChunks; ++k) {
        const int i = first + (wave * per + k) * kWave + lane;
        const int c = cnt[k];
        const int tiles = tiles_of(c);
        const int req_incl = wave_incl_scan_i32(c), tile_incl = wave_incl_scan_i32(tiles);
        const unsigned long long present = __ballot(c > 0);
        const int row = u + __popcll(present & below);
        if (k < per && i < bins) {
            len_base[i] = at_req + req_incl - c;
            len_ceil[i] = row;          // rows shorter than i = the first row that is at least i long
            if (c) {
                len_row[i] = row;
                row_len[row] = i;
                row_off[row] = at_req + req_incl - c;
                tile_off[row] = at_tile + tile_incl - tiles;
            }
        }
        at_req += __builtin_amdgcn_readlane(req_incl, kWave - 1);
        at_tile += __builtin_amdgcn_readlane(tile_incl, kWave - 1);
        u += __popcll(present);
    }
    if (blockIdx.x == kScanGroups - 1 && threadIdx.x == 0) {      // the last workgroup has seen every length
        row_off[all_rows] = all_req;
        tile_off[all_rows] = all_tile;
        totals[0] = all_req; totals[1] = all_rows; totals[2] = all_tile;
        if (out_n) *out_n = all_req;
    }
}

struct ScatterArgs {
    ReqSrc s;
    int *len_cnt, *len_base;
    const int* rank;
    ReqRec* recs;
    int* out_inst;
    float* out_slack;
    int bins, max_len, n_inst;
};

// Requests into grouped order.  Per workgroup: count per length in LDS, reserve
// that many slots of each length with one global atomic, hand the slots out.
// Workgroup `block` of `blocks`.
template <bool kMigrate, int kItems>
__device__ __forceinline__ void scatter_block(const ScatterArgs& a, int block, int blocks, uint32_t* lds)
{
    const ReqSrc& s = a.s;
    int* const len_cnt = a.len_cnt;
    int* const len_base = a.len_base;
    const int* const rank = a.rank;
    ReqRec* const recs = a.recs;
    int* const out_inst = a.out_inst;
    float* const out_slack = a.out_slack;
    const int bins = a.bins, max_len = a.max_len, n_inst = a.n_inst;
    int* slot = reinterpret_cast<int*>(lds);
    const int tid = threadIdx.x;
    for (int L = tid; L < bins; L += kGroupBlock) slot[L] = 0;
    // the histogram has been turned into slot bases: clear it for the next call
    for (int L = block * kGroupBlock + tid; L < bins; L += blocks * kGroupBlock) len_cnt[L] = 0;
    __syncthreads();
    const int64_t base = (int64_t)block * (kGroupBlock * kItems);
    // Everything a request's record needs is read up front, all requests of the thread together (an
    // index past the batch reads the last request and is dropped below): the reads are in flight
    // while the slots are counted and reserved.
    int Ls[kItems], c0s[kItems], pexs[kItems];
    float Ds[kItems];
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t i = base + it * kGroupBlock + tid, ic = min(i, s.n - 1);
        int L;
        const bool takes_part = fetch_len<kMigrate>(s, ic, max_len, L);
        Ls[it] = i < s.n ? (takes_part ? L : -2) : -1;       // -2: in the batch, not scored
        int ex;
        if (kMigrate) {
            c0s[it] = s.act_prompt[ic] + s.act_gen[ic]; Ds[it] = s.act_budget[ic]; ex = s.act_inst[ic];
        } else {
            c0s[it] = s.ctx0[ic]; Ds[it] = s.budget[ic]; ex = s.exclude ? s.exclude[ic] : -1;
        }
        pexs[it] = ex;
    }
#pragma unroll
    for (int it = 0; it < kItems; ++it) {     // the excluded instance as a position in capability order
        const int ex = pexs[it];
        const int r = rank[min(max(ex, 0), n_inst - 1)];
        pexs[it] = (ex >= 0 && ex < n_inst) ? r : -1;
    }
#pragma unroll
    for (int it = 0; it < kItems; ++it)
        if (Ls[it] >= 0) atomicAdd(&slot[Ls[it]], 1);
    __syncthreads();
    // one global atomic per length the workgroup has seen, eight of a thread's in flight together
    constexpr int kAhead = 8;
    for (int L0 = tid; L0 < bins; L0 += kAhead * kGroupBlock) {
        int c[kAhead], b[kAhead];
#pragma unroll
        for (int k = 0; k < kAhead; ++k) {
            const int L = L0 + k * kGroupBlock;
            c[k] = L < bins ? slot[L] : 0;
        }
#pragma unroll
        for (int k = 0; k < kAhead; ++k) b[k] = c[k] ? atomicAdd(&len_base[L0 + k * kGroupBlock], c[k]) : 0;
#pragma unroll
        for (int k = 0; k < kAhead; ++k)
            if (c[k]) slot[L0 + k * kGroupBlock] = b[k];
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int L = Ls[it];
        const int64_t i = base + it * kGroupBlock + tid;
        if (L >= 0) {
            ReqRec r;
            r.c0 = (float)c0s[it]; r.D = Ds[it]; r.pex = pexs[it]; r.orig = (int)i;
            recs[atomicAdd(&slot[L], 1)] = r;
        } else if (L == -2) {
            out_inst[i] = -1;       // not flagged: no migration target
            out_slack[i] = 0.f;
        }
    }
}

// ------------------------------------------------------------------ closed-form lookups
struct MemoArgs {
    const int *totals, *row_len, *len_ceil, *order, *hN;
    const ClassCoef* cls;
    const int* inst_class;
    const uint16_t* tabR;
    const float2 *tabGH, *headGH;
    float* memo;
    float* grp_min;        // [m_pad / kMemoP][row_cap]
    float2* grp_k;         // [m_pad / kMemoP]
    const float2* posK;
    const int* tile_off;   // [rows + 1] first tile of each row
    int* tile_row;         // [tiles] the row of each tile (written here, for the scoring kernel)
    int n_inst, m_pad, cap, row_cap;
    float keep;      // 1 - weight of the black-box estimate: scales the white-box curvature gamma
};

// E of every (distinct length, instance).  A workgroup of kMemoP waves takes
// kMemoP consecutive positions of the capability order, one instance per wave,
// and a run of consecutive distinct lengths ("rows", ascending), kMemoU at a
// time.  The segment of a length is k = #{R_i <= L}.  Both the instance's
// lengths R and the rows are sorted, so k is found by counting instead of
// searching: every entry is first replaced by the first row that is at least
// as long (a table over all lengths from the grouping pass, looked up once per
// entry); the entries whose row lies in a pass (a handful) each add one to that
// row's counter, and a prefix sum over the pass's counters, carried from pass
// to pass, gives k for every row.  Each pass is turned in LDS, in one of two
// buffers so that one barrier per pass is enough, and written in runs of kMemoP
// positions per length.
constexpr int kMemoBlock = kMemoP * kWave;
constexpr int kMemoTile = kMemoU * (kMemoP + 1);       // floats
static_assert(kMemoU == 4 * kWave, "a lane owns four consecutive counters");
static_assert(kMemoP == 16, "a length's values of one workgroup sit in one row of 16 lanes");

// Workgroup (bx, by) of gx x gy.
__device__ __forceinline__ void memo_block(const MemoArgs& a, int bx, int by, int gx, int gy, uint32_t* lds)
{
    float* tiles = reinterpret_cast<float*>(lds);
    const int U = a.totals[1];
    const int p0 = bx * kMemoP;
    const int tid = threadIdx.x, lane = lane_id(), pi = tid / kWave;
    int* cnt = reinterpret_cast<int*>(tiles + 2 * kMemoTile) + pi * kMemoU;
    uint16_t* sRow = reinterpret_cast<uint16_t*>(tiles + 2 * kMemoTile + kMemoP * kMemoU) + (size_t)pi * a.cap;
    constexpr int kPerLane = kMemoU / kWave;
    const int p = p0 + pi;
    const int g = p < a.n_inst ? a.order[p] : -1;
    // this workgroup's run of rows
    const int per = ((U + gy - 1) / gy + kMemoU - 1) / kMemoU * kMemoU;
    const int ub = by * per, ue = min(ub + per, U);
    int N = 0;
    float2 head = make_float2(0.f, 0.f);
    float gam = 0.f;
    const float2* GH = a.tabGH;
    if (g >= 0) {
        N = a.hN[g];
        head = a.headGH[g];
        gam = a.keep * (float)a.cls[a.inst_class[g]].gamma;
        GH = a.tabGH + (size_t)g * a.cap;
        // the row of each of the instance's sorted lengths (how many rows are shorter), looked up
        // once; from here on the lengths themselves are not needed
        const uint16_t* __restrict__ srcR = a.tabR + (size_t)g * a.cap;
#pragma unroll 4
        for (int e = lane; e < N; e += kWave) sRow[e] = (uint16_t)a.len_ceil[srcR[e]];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // the least delta and gamma of this workgroup's positions, for the scoring kernel's bounds
    if (by == 0 && tid < kMemoP) {
        float2 k = a.posK[p0 + tid];
#pragma unroll
        for (int d = 1; d < kMemoP; d <<= 1) {
            k.x = fminf(k.x, __shfl_xor(k.x, d, kMemoP));
            k.y = fminf(k.y, __shfl_xor(k.y, d, kMemoP));
        }
        if (tid == 0) a.grp_k[bx] = k;
    }

    // entries that belong to rows before the run (the rows are ascending with the entries: the
    // lanes that still find one form a prefix)
    int kb = 0;
    if (g >= 0 && ub > 0 && ub < ue) {
        for (int e = lane;; e += kWave) {
            const unsigned long long m = __ballot(e < N && (int)sRow[min(e, N - 1)] < ub && N > 0);
            kb += __popcll(m);
            if (m != ~0ull) break;
        }
    }

    // the lengths of a pass's rows are fetched one pass ahead: every workgroup reads them from L2,
    // and that latency would otherwise sit in the middle of every pass
    int Lnext[kPerLane];
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
        const int u = ub + lane + kWave * i;
        Lnext[i] = u < ue ? a.row_len[u] : 0;
    }
    int buf = 0;
    for (int u0 = ub; u0 < ue; u0 += kMemoU, buf ^= 1) {
        float* tile = tiles + buf * kMemoTile;
        // the row of every tile, for the scoring kernel: the pass's rows are shared out over the
        // workgroups of this run of rows and their waves (usually one row per workgroup and pass)
        for (int r = bx + gx * pi; r < kMemoU; r += gx * kMemoP) {
            const int u = u0 + r;
            if (u >= ue) break;
            const int t0 = a.tile_off[u], t1 = a.tile_off[u + 1];
            for (int t = t0 + lane; t < t1; t += kWave) a.tile_row[t] = u;
        }
        int Lrow[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            Lrow[i] = Lnext[i];
            const int u = u0 + kMemoU + lane + kWave * i;
            Lnext[i] = u < ue ? a.row_len[u] : 0;
        }
        if (g >= 0) {
            reinterpret_cast<int4*>(cnt)[lane] = make_int4(0, 0, 0, 0);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int hi = min(u0 + kMemoU, U);
            int taken = 0;
            for (int e = kb + lane;; e += kWave) {
                const int row = e < N ? (int)sRow[e] : hi;
                const bool ok = row < hi;
                if (ok) atomicAdd(&cnt[row - u0], 1);
                const unsigned long long m = __ballot(ok);
                taken += __popcll(m);
                if (m != ~0ull) break;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            int4 c = reinterpret_cast<int4*>(cnt)[lane];      // rows 4 lane .. 4 lane + 3 of the pass
            c.y += c.x; c.z += c.y; c.w += c.z;
            const int before = kb + wave_incl_scan_i32(c.w) - c.w;
            c.x += before; c.y += before; c.z += before; c.w += before;
            reinterpret_cast<int4*>(cnt)[lane] = c;           // now k of each row
            kb += taken;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) {
                const int row = lane + kWave * i;
                const int k = cnt[row];
                float2 gh = head;
                if (k > 0) gh = GH[k - 1];
                const float Lf = (float)Lrow[i];
                const float tri = Lf * (Lf - 1.0f) * 0.5f;
                tile[row * (kMemoP + 1) + pi] = fmaf(Lf, gh.y, gh.x) + tri * (gam * (float)(N - k + 1));
            }
        } else {
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) tile[(lane + kWave * i) * (kMemoP + 1) + pi] = __builtin_inff();
        }
        __syncthreads();     // the other buffer was last read before the previous pass's barrier
        const int col = tid % kMemoP;
#pragma unroll
        for (int it = 0; it < kMemoU * kMemoP / kMemoBlock; ++it) {
            const int ul = tid / kMemoP + (kMemoBlock / kMemoP) * it;
            const int u = u0 + ul;
            const float e = tile[ul * (kMemoP + 1) + col];
            if (u < U) a.memo[(size_t)u * a.m_pad + p0 + col] = e;
            // the least of the row's kMemoP values (they sit in one row of 16 lanes), for the
            // scoring kernel's walk in capability order
            // running minimum along the row of 16 lanes (a lane without a source keeps its value):
            // lane 15 ends with all 16.  Written out: the compiler pairs every DPP read with a
            // move and a canonicalising maximum; the s_nops keep the distance a DPP read needs
            // from the instruction that wrote its source.
            float m = e;
            asm volatile("s_nop 1\n\t"
                         "v_min_f32_dpp %0, %0, %0 row_shr:1 row_mask:0xf bank_mask:0xf\n\t"
                         "s_nop 1\n\t"
                         "v_min_f32_dpp %0, %0, %0 row_shr:2 row_mask:0xf bank_mask:0xf\n\t"
                         "s_nop 1\n\t"
                         "v_min_f32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xf\n\t"
                         "s_nop 1\n\t"
                         "v_min_f32_dpp %0, %0, %0 row_shr:8 row_mask:0xf bank_mask:0xf\n\t"
                         "s_nop 1"
                         : "+v"(m));
            if (u < U && col == kMemoP - 1) a.grp_min[(size_t)bx * a.row_cap + u] = m;
        }
    }
}

static_assert(kMemoBlock == kGroupBlock, "the two halves of k_group share a workgroup shape");

// The two kernels between the prefix sums and the tiles do not depend on each other (one puts
// the requests in grouped order, the other tabulates E per distinct length and position), so
// they share a launch and run side by side: workgroups 0 .. memo_blocks - 1 tabulate, the
// others scatter.
template <bool kMigrate, int kItems>
__global__ __launch_bounds__(kGroupBlock) void k_group(ScatterArgs sa, MemoArgs ma, int memo_gx, int memo_gy)
{
    extern __shared__ uint32_t lds[];
    const int memo_blocks = memo_gx * memo_gy;
    if ((int)blockIdx.x < memo_blocks)
        memo_block(ma, blockIdx.x % memo_gx, blockIdx.x / memo_gx, memo_gx, memo_gy, lds);
    else
        scatter_block<kMigrate, kItems>(sa, blockIdx.x - memo_blocks, gridDim.x - memo_blocks, lds);
}

// ------------------------------------------------------------------ Alg. 1 over tiles
struct TileArgs {
    const int *totals, *row_len, *row_off, *tile_off, *order;
    const ReqRec* recs;
    const float* memo;     // [row][m_pad] E of (distinct length, position in capability order)
    const float2* posK;    // [m_pad] (delta, gamma) of the instance at each position
    const float* grp_min;  // [m_pad / kMemoP][row_cap] least E of each run of kMemoP positions
    const float2* grp_k;   // [m_pad / kMemoP] least delta and gamma of each run
    const int* tile_row;   // [tiles] the row of each tile
    int row_cap;
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

// kappa = delta + gamma * L, the same instruction wherever a pair's latency is formed
__device__ inline float kappa_of(float2 dg, float Lf) { return fmaf(dg.y, Lf, dg.x); }

// Wave-wide minima of four registers at once (no NaNs among the inputs): on
// return lane 63 of each holds the minimum over the 64 lanes.  Prefix minima
// inside each row of 16 lanes (row_shr 1, 2, 4, 8), then lane 15 of rows 0 and
// 2 into rows 1 and 3, then lane 31 into rows 2 and 3.  A lane without a
// source keeps its value.  The four chains are interleaved so that a register
// is read through DPP no sooner than three instructions after it was written
// (the hardware asks for two); the leading s_nop covers whatever wrote the
// inputs.
__device__ inline void wave_min4(float& a, float& b, float& c, float& d)
{
#define GR_MIN_STEP(ctrl)                          \
    "v_min_f32_dpp %0, %0, %0 " ctrl "\n\t"        \
    "v_min_f32_dpp %1, %1, %1 " ctrl "\n\t"        \
    "v_min_f32_dpp %2, %2, %2 " ctrl "\n\t"        \
    "v_min_f32_dpp %3, %3, %3 " ctrl "\n\t"
    asm volatile("s_nop 1\n\t"
                 GR_MIN_STEP("row_shr:1 row_mask:0xf bank_mask:0xf")
                 GR_MIN_STEP("row_shr:2 row_mask:0xf bank_mask:0xf")
                 GR_MIN_STEP("row_shr:4 row_mask:0xf bank_mask:0xf")
                 GR_MIN_STEP("row_shr:8 row_mask:0xf bank_mask:0xf")
                 GR_MIN_STEP("row_bcast:15 row_mask:0xa bank_mask:0xf")
                 GR_MIN_STEP("row_bcast:31 row_mask:0xc bank_mask:0xf")
                 "s_nop 1"
                 : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
#undef GR_MIN_STEP
}

__device__ inline float wave_min(float v)
{
    float b = v, c = v, d = v;
    wave_min4(v, b, c, d);
    return readlane_f(v, kWave - 1);
}

// Put a wave-uniform value into lane kLane of a vector register.
template <int kLane>
__device__ inline void writelane(float& dst, float uniform_value)
{
    asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(dst) : "s"(uniform_value), "n"(kLane));
}

template <int kLane>
__device__ inline void writelane(int& dst, int uniform_value)
{
    asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(dst) : "s"(uniform_value), "n"(kLane));
}

// Put a wave-uniform value into the lane whose (wave-uniform) number is only
// known at run time: the lane select travels in m0, the value in a scalar
// register.  m0 belongs to the compiler, so it is saved and put back.
__device__ inline void writelane_at(float& dst, float uniform_value, int uniform_lane)
{
    int saved_m0;
    asm volatile("s_mov_b32 %1, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tv_writelane_b32 %0, %2, m0\n\ts_mov_b32 m0, %1"
                 : "+v"(dst), "=&s"(saved_m0) : "s"(uniform_value), "s"(uniform_lane));
}

__device__ inline void writelane_at(int& dst, int uniform_value, int uniform_lane)
{
    int saved_m0;
    asm volatile("s_mov_b32 %1, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tv_writelane_b32 %0, %2, m0\n\ts_mov_b32 m0, %1"
                 : "+v"(dst), "=&s"(saved_m0) : "s"(uniform_value), "s"(uniform_lane));
}

// Requests kJ0 .. kJ0+3 of a tile: their least latency over the wave and the
// lane that holds it (kWave when several lanes do), left in lanes kJ0 .. kJ0+3
// of Tm and win.
template <int kJ0>
__device__ inline void tile_minima4(const float (&minT)[kTileReq], float& Tm, int& win)
{
    float r0 = minT[kJ0], r1 = minT[kJ0 + 1], r2 = minT[kJ0 + 2], r3 = minT[kJ0 + 3];
    wave_min4(r0, r1, r2, r3);
    const float m0 = readlane_f(r0, kWave - 1), m1 = readlane_f(r1, kWave - 1),
                m2 = readlane_f(r2, kWave - 1), m3 = readlane_f(r3, kWave - 1);
    auto winner = [](unsigned long long cand) {
        return (cand && !(cand & (cand - 1))) ? __ffsll((long long)cand) - 1 : kWave;
    };
    writelane<kJ0>(Tm, m0);
    writelane<kJ0 + 1>(Tm, m1);
    writelane<kJ0 + 2>(Tm, m2);
    writelane<kJ0 + 3>(Tm, m3);
    writelane<kJ0>(win, winner(__ballot(minT[kJ0] == m0)));
    writelane<kJ0 + 1>(win, winner(__ballot(minT[kJ0 + 1] == m1)));
    writelane<kJ0 + 2>(win, winner(__ballot(minT[kJ0 + 2] == m2)));
    writelane<kJ0 + 3>(win, winner(__ballot(minT[kJ0 + 3] == m3)));
}

// All 32 wave-wide minima of a full tile at once (no NaNs among the inputs).
// Five halving steps: the lanes of a pair (lane numbers differing in bit s)
// split the requests they still hold by bit s of the request number, each
// passing the other the half it gives up and keeping the minimum of the half
// it holds; then the two halves of the wave are combined.  On return lane l
// holds the minimum of request l mod 32 over the 64 lanes: 31 + 1 minima
// instead of 32 * 6.
//
// A step's minima are single instructions that read the partner's register
// through DPP, written out here because the compiler would pair every such
// read with a separate move and a canonicalising maximum.  No instruction of a
// group reads what another of the group wrote; the leading s_nop keeps the
// distance the hardware asks for between the instructions that produced the
// inputs and the first DPP read.
__device__ inline float tile_minima_all(const float (&m)[kTileReq], int lane)
{
    const bool b0 = lane & 1, b1 = lane & 2, b4 = lane & 16;
    float r1[16], r2[8], r3[4], r4[2];
    // eight minima: outputs %0-%7, what each lane sends %8-%15, what it keeps %16-%23
#define GR_MIN8(o, sd, kp, ctrl)                                                                                     \
    asm volatile("s_nop 1\n\t"                                                                                       \
                 "v_min_f32_dpp %0, %8, %16 " ctrl "\n\t"                                                            \
                 "v_min_f32_dpp %1, %9, %17 " ctrl "\n\t"                                                            \
                 "v_min_f32_dpp %2, %10, %18 " ctrl "\n\t"                                                           \
                 "v_min_f32_dpp %3, %11, %19 " ctrl "\n\t"                                                           \
                 "v_min_f32_dpp %4, %12, %20 " ctrl "\n\t"                                                           \
                 "v_min_f32_dpp %5, %13, %21 " ctrl "\n\t"                                                           \
                 "v_min_f32_dpp %6, %14, %22 " ctrl "\n\t"                                                           \
                 "v_min_f32_dpp %7, %15, %23 " ctrl                                                                  \
                 : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]), "=&v"(o[4]), "=&v"(o[5]), "=&v"(o[6]),        \
                   "=&v"(o[7])                                                                                       \
                 : "v"(sd[0]), "v"(sd[1]), "v"(sd[2]), "v"(sd[3]), "v"(sd[4]), "v"(sd[5]), "v"(sd[6]), "v"(sd[7]),   \
                   "v"(kp[0]), "v"(kp[1]), "v"(kp[2]), "v"(kp[3]), "v"(kp[4]), "v"(kp[5]), "v"(kp[6]), "v"(kp[7]))
    {   // lane ^ 1
        float keep[16], send[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            keep[k] = b0 ? m[2 * k + 1] : m[2 * k];
            send[k] = b0 ? m[2 * k] : m[2 * k + 1];
        }
        float *o = r1, *sd = send, *kp = keep;
        GR_MIN8(o, sd, kp, "quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf");
        o += 8; sd += 8; kp += 8;
        GR_MIN8(o, sd, kp, "quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf");
    }
    {   // lane ^ 2
        float keep[8], send[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            keep[k] = b1 ? r1[2 * k + 1] : r1[2 * k];
            send[k] = b1 ? r1[2 * k] : r1[2 * k + 1];
        }
        GR_MIN8(r2, send, keep, "quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf");
    }
#undef GR_MIN8
    // lane ^ 4 and lane ^ 8: the lanes that keep the even request of a pair are whole banks of four
    // lanes (0-3 and 8-11 of a row of 16, then 0-7), so each output takes two minima that write
    // only their banks and read the register they keep both here and in the partner: no selects.
    asm volatile("s_nop 1\n\t"
                 "v_min_f32_dpp %0, %4, %4 row_shl:4 row_mask:0xf bank_mask:0x5\n\t"
                 "v_min_f32_dpp %1, %6, %6 row_shl:4 row_mask:0xf bank_mask:0x5\n\t"
                 "v_min_f32_dpp %2, %8, %8 row_shl:4 row_mask:0xf bank_mask:0x5\n\t"
                 "v_min_f32_dpp %3, %10, %10 row_shl:4 row_mask:0xf bank_mask:0x5\n\t"
                 "v_min_f32_dpp %0, %5, %5 row_shr:4 row_mask:0xf bank_mask:0xa\n\t"
                 "v_min_f32_dpp %1, %7, %7 row_shr:4 row_mask:0xf bank_mask:0xa\n\t"
                 "v_min_f32_dpp %2, %9, %9 row_shr:4 row_mask:0xf bank_mask:0xa\n\t"
                 "v_min_f32_dpp %3, %11, %11 row_shr:4 row_mask:0xf bank_mask:0xa"
                 : "=&v"(r3[0]), "=&v"(r3[1]), "=&v"(r3[2]), "=&v"(r3[3])
                 : "v"(r2[0]), "v"(r2[1]), "v"(r2[2]), "v"(r2[3]), "v"(r2[4]), "v"(r2[5]), "v"(r2[6]), "v"(r2[7]));
    asm volatile("s_nop 1\n\t"
                 "v_min_f32_dpp %0, %2, %2 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
                 "v_min_f32_dpp %1, %4, %4 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
                 "v_min_f32_dpp %0, %3, %3 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
                 "v_min_f32_dpp %1, %5, %5 row_ror:8 row_mask:0xf bank_mask:0xc"
                 : "=&v"(r4[0]), "=&v"(r4[1])
                 : "v"(r3[0]), "v"(r3[1]), "v"(r3[2]), "v"(r3[3]));
    const float keep = b4 ? r4[1] : r4[0], send = b4 ? r4[0] : r4[1];
    // lane ^ 16 by a swizzle in bit mode (and 0x1f, or 0, xor 0x10), lane ^ 32 by a permute; both
    // values come back as they were stored, so the minima below need no canonicalising
    float r = __builtin_fminf(keep, __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(send), 0x401F)));
    return __builtin_fminf(r, __shfl_xor(r, 32, kWave));
}

// The lane that holds request kJ's minimum `Tm` (lane kJ of it), kWave when
// several do, into lane kJ of `win`.
template <int kJ>
__device__ inline void tile_winner(const float (&minT)[kTileReq], float Tm, int& win)
{
    const unsigned long long cand = __ballot(minT[kJ] == readlane_f(Tm, kJ));
    writelane<kJ>(win, (cand && !(cand & (cand - 1))) ? __ffsll((long long)cand) - 1 : kWave);
}

template <int kJ, int kEnd>
__device__ inline void tile_winners(const float (&minT)[kTileReq], float Tm, int& win)
{
    if constexpr (kJ < kEnd) {
        tile_winner<kJ>(minT, Tm, win);
        tile_winners<kJ + 1, kEnd>(minT, Tm, win);
    }
}

struct RowView {
    const float* __restrict__ E;       // this length's row of the memo table
    const float* __restrict__ grpE;    // least E of each run of kMemoP positions of the row, run r at grpE[r * grp_stride]
    int grp_stride;
    const float2* __restrict__ grpK;   // least delta and least gamma of each such run (LDS), or null
    const float2* __restrict__ posK;
    const int* __restrict__ order;
    float Lf;
    int nblk;                          // blocks of 64 positions (even)
};

// The walks below visit the blocks of a row in order; each depends on what the
// previous block showed, so their loads are taken a few blocks at a time, the
// next chunk in flight while the current one is looked at.
template <int kN, bool kWithOrder>
struct Chunk {
    float e[kN];
    float2 k[kN];
    int g[kWithOrder ? kN : 1];
};

template <int kN, bool kWithOrder>
__device__ __forceinline__ void load_chunk(const RowView& rv, int b0, int lane, Chunk<kN, kWithOrder>& c)
{
#pragma unroll
    for (int i = 0; i < kN; ++i) {
        const int p = min(b0 + i, rv.nblk - 1) * kWave + lane;    // past the end: the last block again
        c.e[i] = rv.E[p];
        c.k[i] = rv.posK[p];
        if (kWithOrder) c.g[i] = rv.order[p];
    }
}

// First feasible position in capability order for the few requests of a tile
// that have one (bit j of `fm`): blocks in order, the requests still open one
// after the other.  Exclusions are not applied here.
__device__ inline void first_feasible_sparse(const RowView& rv, float rec_c0, float Dc, unsigned long long fm,
                                             int lane, int& foundP, float& foundT)
{
    constexpr int kChunk = 8;
    Chunk<kChunk, false> cur;
    load_chunk(rv, 0, lane, cur);
    for (int b0 = 0; b0 < rv.nblk && fm; b0 += kChunk) {
        Chunk<kChunk, false> nxt;
        load_chunk(rv, b0 + kChunk, lane, nxt);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            if (b0 + i >= rv.nblk) break;
            const float e = cur.e[i], k = kappa_of(cur.k[i], rv.Lf);
            unsigned long long m = fm;
            while (m) {
                const int j = __ffsll((long long)m) - 1;
                m &= m - 1;
                const float T = fmaf(readlane_f(rec_c0, j), k, e);
                const unsigned long long feas = __ballot(T <= readlane_f(Dc, j));
                if (feas) {
                    const int fl = __ffsll((long long)feas) - 1;
                    const float Tf = readlane_f(T, fl);
                    writelane_at(foundP, (b0 + i) * kWave + fl, j);
                    writelane_at(foundT, Tf, j);
                    fm &= ~(1ull << j);
                }
            }
        }
        cur = nxt;
    }
}

// The same when many requests of the tile have a feasible instance: all
// requests against each block, two vector operations per pair; a request that
// is done (or never had one) carries D = -inf.  Looks at the first n_blocks
// blocks and returns the requests still open after them.
__device__ inline unsigned long long first_feasible_dense(const RowView& rv, const float (&c0)[kTileReq], float Dc,
                                                          unsigned long long fm, int n_blocks, int lane, int& foundP,
                                                          float& foundT)
{
    float D[kTileReq];
#pragma unroll
    for (int j = 0; j < kTileReq; ++j) {
        D[j] = ((fm >> j) & 1ull) ? readlane_f(Dc, j) : -__builtin_inff();
        asm volatile("" : "+v"(D[j]));     // 32 more scalars would not fit the scalar file
    }
    unsigned left = (unsigned)fm;
    constexpr int kChunk = 2;
    Chunk<kChunk, false> cur;
    load_chunk(rv, 0, lane, cur);
    for (int b0 = 0; b0 < n_blocks && left; b0 += kChunk) {
        Chunk<kChunk, false> nxt;
        load_chunk(rv, b0 + kChunk, lane, nxt);
        __builtin_amdgcn_sched_barrier(0);
        for (int i = 0; i < kChunk && b0 + i < n_blocks && left; ++i) {
            float e = 0.f;
            float2 kk = make_float2(0.f, 0.f);
#pragma unroll
            for (int c = 0; c < kChunk; ++c)
                if (c == i) { e = cur.e[c]; kk = cur.k[c]; }
            float k = kappa_of(kk, rv.Lf);
            unsigned long long any = 0;
#pragma unroll
            for (int j = 0; j < kTileReq; ++j) any |= __ballot(fmaf(c0[j], k, e) <= D[j]);
            if (any) {
                asm volatile("" : "+v"(e), "+v"(k));   // recomputed: nothing of this branch stays live above
#pragma unroll
                for (int j = 0; j < kTileReq; ++j) {
                    const float T = fmaf(c0[j], k, e);
                    const unsigned long long feas = __ballot(T <= D[j]);
                    if (feas) {
                        const int fl = __ffsll((long long)feas) - 1;
                        const float Tf = readlane_f(T, fl);
                        writelane_at(foundP, (b0 + i) * kWave + fl, j);
                        writelane_at(foundT, Tf, j);
                        left &= ~(1u << j);
                        D[j] = -__builtin_inff();
                    }
                }
            }
        }
        cur = nxt;
    }
    return left;
}

// First feasible position in capability order by bounds: a run of kMemoP
// consecutive positions cannot hold a feasible one unless
// least E + c0 * (least delta + L * least gamma) <= D, and that bound is formed
// with the same two fused multiply-adds as the latency itself, which are
// monotone in every operand (c0, L >= 0), so it never exceeds the latency of a
// position of the run as the main pass computed it.  The bound's two
// request-independent parts are read once per tile (lane = run, 64 runs per
// register pair; runs beyond kBoundRegs * 64 are read again per request).  Per
// request: which runs pass, then from the first such run on 64 positions at
// once until there is a hit.  Instances come slowest first, so most runs
// before the answer fail the bound and are never looked at.
constexpr int kBoundRegs = 4;
constexpr int kRunsPerBlock = kWave / kMemoP;

__device__ inline void first_feasible_bounded(const RowView& rv, float rec_c0, float Dc, unsigned long long fm,
                                              int lane, int& foundP, float& foundT)
{
    const int ngrp = rv.nblk * kRunsPerBlock;
    float gE[kBoundRegs], gK[kBoundRegs];
#pragma unroll
    for (int i = 0; i < kBoundRegs; ++i) {
        const int g = min(i * kWave + lane, ngrp - 1);
        gE[i] = i * kWave + lane < ngrp ? rv.grpE[(size_t)g * rv.grp_stride] : __builtin_inff();     // never passes
        gK[i] = kappa_of(rv.grpK[g], rv.Lf);
    }
    while (fm) {
        const int j = __ffsll((long long)fm) - 1;
        fm &= fm - 1;
        const float c0j = readlane_f(rec_c0, j), Dj = readlane_f(Dc, j);
        bool found = false;
        // looks at 64 positions from run `gi` on (from further back at the end of the row: what lies
        // before the first run that passes is infeasible anyway, its runs failed the bound); all
        // addresses are a scalar start plus the lane
        const auto visit = [&](int gi) {
            const int start = min(gi * kMemoP, rv.nblk * kWave - kWave);
            const float T = fmaf(c0j, kappa_of(rv.posK[start + lane], rv.Lf), rv.E[start + lane]);
            const unsigned long long hit = __ballot(T <= Dj);
            if (hit) {
                const int fl = __ffsll((long long)hit) - 1;
                writelane_at(foundP, start + fl, j);
                writelane_at(foundT, readlane_f(T, fl), j);
                found = true;
            }
        };
        const auto chunk = [&](int g0, float boundE, float boundK) {
            unsigned long long pass = __ballot(fmaf(c0j, boundK, boundE) <= Dj);
            while (pass && !found) {
                const int first = __ffsll((long long)pass) - 1;
                pass &= ~(((1ull << kRunsPerBlock) - 1ull) << first);      // the runs this visit covers
                visit(g0 + first);
            }
        };
#pragma unroll
        for (int i = 0; i < kBoundRegs; ++i)
            if (!found && i * kWave < ngrp) chunk(i * kWave, gE[i], gK[i]);
        for (int g0 = kBoundRegs * kWave; g0 < ngrp && !found; g0 += kWave) {
            const int g = min(g0 + lane, ngrp - 1);
            chunk(g0, g0 + lane < ngrp ? rv.grpE[(size_t)g * rv.grp_stride] : __builtin_inff(), kappa_of(rv.grpK[g], rv.Lf));
        }
    }
}

// Alg. 1 for one request on its own, exactly: every position but `pex`, the
// first feasible one in capability order, else the smallest T with ties to the
// lowest instance index.  The rare cases of the tile pass end here: a choice
// that fell on the excluded instance, equal minima.
__device__ inline void exact_choice(const RowView& rv, float c0, float D, int pex, int lane,
                                    int& pos, float& val, bool& found)
{
    float minT = __builtin_inff();
    int minP = -1, minG = 0x7fffffff;
    found = false;
    constexpr int kChunk = 4;
    Chunk<kChunk, true> cur;
    load_chunk(rv, 0, lane, cur);
    for (int b0 = 0; b0 < rv.nblk; b0 += kChunk) {
        Chunk<kChunk, true> nxt;
        load_chunk(rv, b0 + kChunk, lane, nxt);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            if (b0 + i >= rv.nblk) break;
            const int p = (b0 + i) * kWave + lane;
            const int g = cur.g[i];
            float T = fmaf(c0, kappa_of(cur.k[i], rv.Lf), cur.e[i]);
            if (p == pex || g < 0) T = __builtin_inff();
            const unsigned long long feas = __ballot(T <= D);
            if (feas) {
                const int fl = __ffsll((long long)feas) - 1;
                pos = (b0 + i) * kWave + fl;
                val = readlane_f(T, fl);
                found = true;
                return;
            }
            if (T < minT || (T == minT && g >= 0 && g < minG)) { minT = T; minP = p; minG = g; }
        }
        cur = nxt;
    }
    const float Tm = wave_min(minT);
    unsigned long long cand = __ballot(minT == Tm && Tm < __builtin_inff());
    int bp = -1, bg = 0x7fffffff;
    while (cand) {
        const int l = __ffsll((long long)cand) - 1;
        cand &= cand - 1;
        const int g = __builtin_amdgcn_readlane(minG, l);
        if (g < bg) { bg = g; bp = __builtin_amdgcn_readlane(minP, l); }
    }
    pos = bp;
    val = bp >= 0 ? Tm : 0.f;
}

// Main pass of a tile: T = E + c0 * kappa for the first kN requests against every
// position, folded into each request's running minimum per lane.  Two blocks
// of 64 positions per step, the operands of the next step in flight (two
// register sets taking turns, so that nothing is copied).
// The prefill length of a request is the same in all lanes and normally sits in
// a scalar register.  The vector ALU issues up to two instructions of different
// waves in the four cycles a wave instruction takes, the second one only from
// the simple class (multiply-add, add, logic, move) and, as measured, not next
// to a minimum when it reads a scalar register: with scalar operands only, a
// minimum issues alone and the two multiply-adds of a pair pair up with each
// other (2 slots per 3 instructions instead of 1.5).  So the first kVecReq
// requests of a tile also keep their length in a vector register each, for the
// main pass only: their multiply-adds can go next to the minima.  (All 32 in
// vector registers would cost 32 registers and was no faster.)
constexpr int kVecReq = 16;

template <int kN>
__device__ __forceinline__ void main_pass(const RowView& rv, const float (&c0)[kTileReq], const float (&c0v)[kVecReq],
                                          float (&minT)[kTileReq], int lane)
{
    struct Step { float Ea, Eb; float2 Ka, Kb; };
    // Block starts are wave-uniform.  The table row is read through a buffer descriptor: the
    // address is base + the lane's fixed byte offset + a scalar offset that the scalar unit
    // advances, so a read costs no vector arithmetic (with a plain pointer the compiler folds the
    // lane's offset into a loop-invariant 64-bit vector base and adds the block offset to it with
    // a shift-and-add per step, an instruction of the one-per-slot class).  The coefficient pairs
    // are at the lane's own address plus a scalar offset: a plain add.
    const int lane_e = lane * (int)sizeof(float);
    const __amdgpu_buffer_rsrc_t row = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(rv.E), 0, rv.nblk * kWave * (int)sizeof(float), 0x00020000 /* 32-bit elements */);
    const char* const k_lane = reinterpret_cast<const char*>(rv.posK + (unsigned)lane);
    auto fetch = [&](Step& st, int b) {
        const int e_off = b * (kWave * (int)sizeof(float));
        unsigned k_off = (unsigned)b * (unsigned)(kWave * sizeof(float2));
        asm volatile("" : "+s"(k_off));      // (a scalar, added as it is)
        st.Ea = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(row, lane_e, e_off, 0));
        st.Eb = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(row, lane_e + kWave * (int)sizeof(float), e_off, 0));
        const float2* __restrict__ kb = reinterpret_cast<const float2*>(k_lane + k_off);
        st.Ka = kb[0]; st.Kb = kb[kWave];
    };
    auto fold = [&](const Step& st) {
        const float ka = kappa_of(st.Ka, rv.Lf), kb = kappa_of(st.Kb, rv.Lf);
        // in pairs of requests, one with its length in a vector register and one in a scalar
        // register: four multiply-adds, then the two minima (a minimum right behind the
        // multiply-adds it reads waits for them)
        static_assert(kVecReq * 2 == kTileReq, "request j (vector operand) goes with request j + kVecReq (scalar)");
#pragma unroll
        for (int j = 0; j < (kN < kVecReq ? kN : kVecReq); ++j) {
            const int jv = j, js = j + kVecReq;
            float Ta = fmaf(c0v[jv], ka, st.Ea), Tb = fmaf(c0v[jv], kb, st.Eb);
            if (js < kN) {
                float Ua = fmaf(c0[js], ka, st.Ea), Ub = fmaf(c0[js], kb, st.Eb);
                __builtin_amdgcn_sched_barrier(0);      // (the four multiply-adds stay ahead of the two minima)
                minT[jv] = fminf(fminf(minT[jv], Ta), Tb);
                minT[js] = fminf(fminf(minT[js], Ua), Ub);
            } else {
                minT[jv] = fminf(fminf(minT[jv], Ta), Tb);
            }
        }
    };
    // the prefetch is unconditional (past the end it re-reads the last step), so that the
    // compiler can count exactly how many loads may stay in flight at each use
    Step s0, s1;
    const int last = rv.nblk - 2;
    fetch(s0, 0);
    for (int b = 0; b < rv.nblk; b += 4) {
        fetch(s1, min(b + 2, last));
        __builtin_amdgcn_sched_barrier(0);       // keep the loads ahead of the arithmetic
        fold(s0);
        __builtin_amdgcn_sched_barrier(0);
        fetch(s0, min(b + 4, last));
        __builtin_amdgcn_sched_barrier(0);
        if (b + 2 < rv.nblk) fold(s1);
        __builtin_amdgcn_sched_barrier(0);
    }
}

constexpr int kSparseFeasible = 8;   // up to this many feasible requests of a tile go one by one
constexpr int kDenseBlocks = 2;      // blocks looked at for all requests at once before the bounded walk

constexpr int kXcdRun = 8;     // workgroups in a row that stay on one XCD
constexpr int kSmallTilesFirstBelow = 4 * 256 * 24;   // tiles: four rounds of the chip's 6 waves per SIMD

// One wave per tile: up to kTileReq requests of one length against all
// instances.  Lane = position in capability order within a block of 64; the
// requests' prefill lengths are wave-uniform (scalar registers, and for half of
// them a vector register as well, see kVecReq).
//
// Main pass, per pair: T = E + c0 * kappa (one multiply-add) folded into the
// request's running minimum per lane (one three-way minimum per two pairs).
// Alg. 1's feasible set is non-empty exactly when that minimum is <= D, so the
// feasibility test of every pair is implied; only requests that have a
// feasible instance are looked at again, for their first one in capability
// order (the just-enough choice).  The others take the instance of the minimum,
// found by recomputing the positions of the lane that holds it; equal minima
// (in several lanes or at several positions of one lane) are redone one by one,
// so that ties go to the lowest instance index.  The lanes' own request
// records (budget, excluded instance, index in the caller's arrays) are read
// only after the main pass and the minima.
//
// kW waves per workgroup, six waves per SIMD (80 vector registers: the 32
// running minima, two sets of operands in flight and the epilogue's
// temporaries fit without spilling).  With kW > 4 the workgroup first copies
// the (delta, gamma) pairs of all positions, which every tile reads in full,
// into LDS (and their minima over runs of kMemoP positions, for the bounded
// walk): 24 / kW workgroups of m_pad * 8.5 bytes share a compute unit, and the
// texture path is left to the table rows and the gathers of the search for the
// minimum.
template <bool kWriteT, int kW, int kWavesPerSimd>
__global__ __launch_bounds__(kW * kWave) __attribute__((amdgpu_waves_per_eu(kWavesPerSimd, kWavesPerSimd))) void k_tile(TileArgs a)
{
    // (four waves per workgroup at six per SIMD is the variant without the LDS copy)
    constexpr bool kLdsK = kW > 4 || kWavesPerSimd > 6;
    extern __shared__ float2 lds_posK[];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int NT = a.totals[2];
    // consecutive tiles share a table row: keep them on one XCD (workgroups go round-robin over 8)
    // in runs of kXcdRun workgroups' worth of tiles, dealt to the XCDs in turn: tiles get cheaper
    // towards the long lengths (few requests each), and equal eighths of the tiles are not equal work
    const int groups = (NT + kW - 1) / kW;
    const int seq = blockIdx.x >> 3;
    const int bid = (seq / kXcdRun) * (8 * kXcdRun) + (int)(blockIdx.x & 7) * kXcdRun + seq % kXcdRun;
    if (bid >= groups) return;
    // Tiles come cheapest last (the common lengths first, the rare ones with a few requests each at
    // the end), which lets a launch of many rounds of waves tail off smoothly.  A launch of two or
    // three rounds is better off the other way round: its small tiles are then done next to the
    // large ones instead of adding a round of their own, each a chain of dependent loads long.
    const int idx = bid * kW + wave;
    const int t = NT < kSmallTilesFirstBelow ? NT - 1 - idx : idx;
    float2* lds_grpK = lds_posK + a.m_pad;      // least (delta, gamma) of each run of kMemoP positions
    if (kLdsK) {
        for (int p = threadIdx.x; p < a.m_pad; p += kW * kWave) lds_posK[p] = a.posK[p];
        for (int g = threadIdx.x; g < a.m_pad / kMemoP; g += kW * kWave) lds_grpK[g] = a.grp_k[g];
        __syncthreads();
    }
    if (idx >= NT) return;

    const int u = a.tile_row[t];        // (written by the memo kernel)
    // The row's requests are dealt out to its tiles in turn (request q of the row goes to tile
    // q mod tiles), not in runs of 32: neighbours in grouped order tend to come from one instance,
    // and requests whose answer lands on their own (excluded) instance are redone one by one, which
    // would otherwise pile up in single tiles.
    const int row_begin = a.row_off[u], row_n = a.row_off[u + 1] - row_begin;
    const int row_tiles = a.tile_off[u + 1] - a.tile_off[u], tl = t - a.tile_off[u];
    const int nreq = (row_n - tl + row_tiles - 1) / row_tiles;       // requests q = tl, tl + tiles, ..

    RowView rv;
    rv.E = a.memo + (size_t)u * a.m_pad;
    rv.grpE = a.grp_min + u;
    rv.grp_stride = a.row_cap;
    rv.grpK = kLdsK ? lds_grpK : nullptr;
    rv.posK = kLdsK ? lds_posK : a.posK;
    rv.order = a.order;
    rv.Lf = (float)a.row_len[u];
    rv.nblk = a.m_pad / kWave;

    // the requests' prefill lengths as scalars: read again through the scalar cache (the lanes hold
    // them too, but a read of a lane is a vector instruction of the one-per-slot class); slots past
    // the tile's last request repeat the last one, their results are never used
    float c0[kTileReq], minT[kTileReq];
    const ReqRec* __restrict__ tile_recs = a.recs + row_begin + tl;
#pragma unroll
    for (int j = 0; j < kTileReq; ++j) {
        c0[j] = tile_recs[(size_t)min(j, nreq - 1) * row_tiles].c0;
        minT[j] = __builtin_inff();
    }

    float c0v[kVecReq];
#pragma unroll
    for (int j = 0; j < kVecReq; ++j) {
        c0v[j] = c0[j];
        asm volatile("" : "+v"(c0v[j]));      // (a vector register, whatever the compiler knows about the value)
    }

    // ---- main pass over the requests the tile really has, in fours (most lengths of a batch
    // have only a few requests, and a tile is one length's)
    switch ((nreq + 3) >> 2) {
        case 1: main_pass<4>(rv, c0, c0v, minT, lane); break;
        case 2: main_pass<8>(rv, c0, c0v, minT, lane); break;
        case 3: main_pass<12>(rv, c0, c0v, minT, lane); break;
        case 4: main_pass<16>(rv, c0, c0v, minT, lane); break;
        case 5: main_pass<20>(rv, c0, c0v, minT, lane); break;
        case 6: main_pass<24>(rv, c0, c0v, minT, lane); break;
        case 7: main_pass<28>(rv, c0, c0v, minT, lane); break;
        default: main_pass<32>(rv, c0, c0v, minT, lane); break;
    }

    // ---- per request: the least latency and the lane that holds it (lane j keeps request j's)
    float Tm = __builtin_inff();
    int win = kWave;                 // lane holding the minimum; kWave when several do
    static_assert(kTileReq == 32, "eight groups of four requests");
    if (nreq > 16) {
        Tm = tile_minima_all(minT, lane);
        tile_winners<0, kTileReq>(minT, Tm, win);
    } else {
        tile_minima4<0>(minT, Tm, win);
        if (nreq > 4) tile_minima4<4>(minT, Tm, win);
        if (nreq > 8) tile_minima4<8>(minT, Tm, win);
        if (nreq > 12) tile_minima4<12>(minT, Tm, win);
    }

    // The lanes' own request records (lane j: request j) are only needed from here on: read after
    // the main pass and the minima, they do not sit in registers (or scratch) through them.
    // Lanes past the tile's last request carry a dummy that is never feasible and never reported.
    __builtin_amdgcn_sched_barrier(0);
    ReqRec rec;
    rec.c0 = 0.f; rec.D = -__builtin_inff(); rec.pex = -1; rec.orig = -1;
    const bool mine = lane < nreq;
    if (mine) rec = tile_recs[(size_t)lane * row_tiles];
    // padded positions hold T = +inf and must stay infeasible even for D = +inf; a NaN budget is never met
    const float Dc = rec.D > FLT_MAX ? FLT_MAX : rec.D;

    // ---- requests with a feasible instance: the first one in capability order
    int foundP = -1;
    float foundT = 0.f;
    const unsigned long long fm = __ballot(mine && Tm <= Dc);
    if (fm) {
        // many feasible requests: most have their first feasible instance early or not at all
        // early, so the first blocks are looked at for all of them at once; the rest by bounds
        unsigned long long rest = fm;
        if (__popcll(rest) > kSparseFeasible)
            rest = first_feasible_dense(rv, c0, Dc, rest, kLdsK ? min(kDenseBlocks, rv.nblk) : rv.nblk, lane, foundP, foundT);
        if (rest) {
            if (kLdsK) first_feasible_bounded(rv, rec.c0, Dc, rest, lane, foundP, foundT);
            else first_feasible_sparse(rv, rec.c0, Dc, rest, lane, foundP, foundT);
        }
    }

    // ---- the others: which of the winning lane's positions has T = the minimum.  Lane l looks
    // for request l mod 32 in the blocks of parity l / 32; the earliest block wins.
    const int src = lane & (kTileReq - 1);
    const float s_c0 = __shfl(rec.c0, src, kWave), s_Tm = __shfl(Tm, src, kWave);
    const int s_win = __shfl(win, src, kWave);
    // The block is tracked as a float key, T - min scaled up plus the block number: the key is the
    // block number exactly where T equals the minimum (the difference of two floats is zero only
    // if they are equal, and T >= min) and huge elsewhere; the least key is the earliest such block.
    // That is three instructions of the class that issues two per slot and half a three-way
    // minimum per block, instead of a compare and a select.
    // A second key of the same kind with the block number negated gives the latest such block: the
    // two differ when the lane holds the minimum at more than one position (different instances
    // with the same latency), and then the tie goes to the lowest instance index, one by one.
    int firstB = 0x7fffffff, lastB = -1;
    if (__ballot(mine && foundP < 0)) {
        const int lw = s_win & (kWave - 1), half = lane >> 5;
        const float* __restrict__ pe = rv.E + half * kWave + lw;
        const float2* __restrict__ pk = rv.posK + half * kWave + lw;
        float blk = (float)half, key = 0x1p100f, keyL = 0x1p100f;
#pragma unroll 8
        for (int i = 0; i < rv.nblk / 2; ++i) {       // block 2 i + half
            const float Tc = fmaf(s_c0, kappa_of(pk[i * 2 * kWave], rv.Lf), pe[i * 2 * kWave]);
            const float off = Tc - s_Tm;
            key = fminf(key, fmaf(off, 0x1p100f, blk));
            keyL = fminf(keyL, fmaf(off, 0x1p100f, -blk));     // minus the latest block where T equals the minimum
            blk += 2.0f;
        }
        if (key < 0x1p30f) { firstB = (int)key; lastB = -(int)keyL; }
    }
    firstB = min(firstB, __shfl_xor(firstB, 32, kWave));
    lastB = max(lastB, __shfl_xor(lastB, 32, kWave));
    const int candP = firstB < rv.nblk ? firstB * kWave + (win & (kWave - 1)) : -1;
    // equal minima (in several lanes, or at several positions of one) and a minimum on the
    // excluded instance: one by one
    const bool slow = mine && (foundP >= 0 ? foundP == rec.pex
                                           : (win == kWave || candP < 0 || candP == rec.pex || lastB != firstB));

    int p = foundP >= 0 ? foundP : candP;
    float T = foundP >= 0 ? foundT : Tm;
    bool found = foundP >= 0;

    unsigned long long redo = __ballot(slow);
    while (redo) {
        const int j = __ffsll((long long)redo) - 1;
        redo &= redo - 1;
        int rp;
        float rt;
        bool rf;
        exact_choice(rv, readlane_f(rec.c0, j), readlane_f(Dc, j), __builtin_amdgcn_readlane(rec.pex, j),
                     lane, rp, rt, rf);
        if (lane == j) { p = rp; T = rt; found = rf; }
    }

    if (mine) {
        const int g = p >= 0 ? a.order[p] : -1;
        a.out_inst[rec.orig] = g;
        a.out_slack[rec.orig] = g >= 0 ? rec.D - T : 0.f;
        if (a.out_fallback) a.out_fallback[rec.orig] = !found;
    }

    if (kWriteT) {   // every pair's latency, for checking: same arithmetic, exclusions not applied
        for (int b = 0; b < rv.nblk; ++b) {
            const float e = rv.E[b * kWave + lane], k = kappa_of(rv.posK[b * kWave + lane], rv.Lf);
            const int g_lane = a.order[b * kWave + lane];
            for (int j = 0; j < nreq; ++j) {
                const int orig = __builtin_amdgcn_readlane(rec.orig, j);
                const float Tj = fmaf(readlane_f(rec.c0, j), k, e);
                if (g_lane >= 0) a.out_T[(size_t)orig * a.n_inst + g_lane] = Tj;
            }
        }
    }
}

// ------------------------------------------------------------------ cached prefixes
struct HitArgs {
    const int *ctx0, *pred_len;
    const float* budget;
    const int* exclude;
    const int *hit_off, *hit_inst, *hit_len;
    const int *len_row, *rank, *order;
    const float* memo;
    const float2* posK;
    int* out_inst;
    float* out_slack;
    uint8_t* out_fallback;
    float* out_T;
    int64_t n, n_hits;
    int n_inst, m_pad, max_len;
};

// Eq. 2's hit prefix H_{r,g}, after the pass without it: a cached prefix of h
// tokens on instance g takes delta_g * h off T(r,g) and changes nothing else,
// so Alg. 1's answer can only move to an instance the request has a prefix on.
// One thread per request that has any: the choice made without prefixes
// against the request's own short list.  Feasible set: the earlier position in
// capability order wins; otherwise the smallest T, ties to the lowest index
// (the minimum over all instances is either the old one or among the hits,
// because a hit only lowers its own pair).
__global__ __launch_bounds__(kBlock) void k_hits(HitArgs a)
{
    const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r >= a.n) return;
    const int64_t h0 = min(max((int64_t)a.hit_off[r], (int64_t)0), a.n_hits);
    const int64_t h1 = min(max((int64_t)a.hit_off[r + 1], h0), a.n_hits);
    if (h0 >= h1) return;
    const int L = min(max(a.pred_len[r], 0), a.max_len);
    const int ci = a.ctx0[r];
    const float c0 = (float)ci, Lf = (float)L, D = a.budget[r];
    const float Dc = D > FLT_MAX ? FLT_MAX : D;
    const int ex = a.exclude ? a.exclude[r] : -1;
    const float* __restrict__ rowE = a.memo + (size_t)a.len_row[L] * a.m_pad;

    int feasP = 0x7fffffff, anyG = -1;
    float feasT = 0.f, anyT = __builtin_inff();
    const int g0 = a.out_inst[r];
    if (g0 >= 0) {
        const int p0 = a.rank[g0];
        const float T0 = fmaf(c0, kappa_of(a.posK[p0], Lf), rowE[p0]);
        if (T0 <= Dc) { feasP = p0; feasT = T0; }
        anyG = g0; anyT = T0;
    }
    for (int64_t k = h0; k < h1; ++k) {
        const int g = a.hit_inst[k];
        if (g < 0 || g >= a.n_inst) continue;
        const int h = min(max(a.hit_len[k], 0), max(ci, 0));
        const int p = a.rank[g];
        const float2 dg = a.posK[p];
        const float T = fmaf(-(float)h, dg.x, fmaf(c0, kappa_of(dg, Lf), rowE[p]));
        if (a.out_T) {          // (an instance named twice: the longer prefix, i.e. the smaller T, stays)
            float* t = a.out_T + (size_t)r * a.n_inst + g;
            *t = fminf(*t, T);
        }
        if (g == ex) continue;
        if (T <= Dc && (p < feasP || (p == feasP && T < feasT))) { feasP = p; feasT = T; }
        if (T < anyT || (T == anyT && g < anyG)) { anyT = T; anyG = g; }
    }
    const bool found = feasP != 0x7fffffff;
    const int g = found ? a.order[feasP] : anyG;
    a.out_inst[r] = g;
    a.out_slack[r] = g >= 0 ? D - (found ? feasT : anyT) : 0.f;
    if (a.out_fallback) a.out_fallback[r] = !found;
}

// ------------------------------------------------------------------ small batches, pair by pair
struct DirectArgs {
    const int *ctx0, *pred_len;
    const float* budget;
    const int* exclude;
    const int *order, *hN;
    const ClassCoef* cls;
    const int* inst_class;
    const uint16_t* tabR;
    const float2 *tabGH, *headGH, *posK;
    unsigned long long *best_feasible, *best_any;     // [n] each, all ones on entry
    int* out_inst;
    float* out_slack;
    uint8_t* out_fallback;
    float* out_T;
    int n, n_inst, m_pad, cap, max_len;
    float keep;
};

// a float as an unsigned integer of the same order
__device__ inline uint32_t ordered_bits(float v)
{
    const uint32_t b = __float_as_uint(v);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

__device__ inline float from_ordered_bits(uint32_t u)
{
    return __uint_as_float(u ^ ((u >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

// A batch of a few requests (one arriving request is the paper's own case):
// grouping by length and a table of per-length values would cost more than
// they save, so every pair gets a thread, which finds its segment by a binary
// search over the instance's sorted lengths (Eq. 2's decode term in closed
// form, the same expression as in the memo kernel) and forms T = E + c0 * kappa.
// Thread = position in capability order, blockIdx.y = request.  Alg. 1's two
// selections are two 64-bit minima per request, reduced over the wave and then
// with one atomic each: (position, T) over the feasible pairs, i.e. the first
// feasible instance in capability order, and (T, instance index) over all, i.e.
// the least latency with ties to the lowest index.
__global__ __launch_bounds__(kBlock) void k_direct(DirectArgs a)
{
    const int p = blockIdx.x * kBlock + threadIdx.x, r = blockIdx.y;
    const int L = min(max(a.pred_len[r], 0), a.max_len);
    const float c0 = (float)a.ctx0[r], Lf = (float)L, D = a.budget[r];
    const float Dc = D > FLT_MAX ? FLT_MAX : D;       // padded positions hold +inf and stay infeasible
    const int ex = a.exclude ? a.exclude[r] : -1;
    const int g = p < a.m_pad ? a.order[p] : -1;
    unsigned long long feas = ~0ull, any = ~0ull;
    if (g >= 0) {
        const int N = a.hN[g];
        const uint16_t* __restrict__ R = a.tabR + (size_t)g * a.cap;
        int k = 0;                                    // #{R_i <= L}
        for (int step = a.cap; step >= 1; step >>= 1) {
            const int probe = k + step;
            if (probe <= N && (int)R[probe - 1] <= L) k = probe;
        }
        const float2 gh = k > 0 ? a.tabGH[(size_t)g * a.cap + k - 1] : a.headGH[g];
        const float gam = a.keep * (float)a.cls[a.inst_class[g]].gamma;
        const float tri = Lf * (Lf - 1.0f) * 0.5f;
        const float E = fmaf(Lf, gh.y, gh.x) + tri * (gam * (float)(N - k + 1));
        const float T = fmaf(c0, kappa_of(a.posK[p], Lf), E);
        if (a.out_T) a.out_T[(size_t)r * a.n_inst + g] = T;
        if (g != ex) {
            const unsigned long long tb = ordered_bits(T);
            any = (tb << 32) | (unsigned)g;
            if (T <= Dc) feas = ((unsigned long long)p << 32) | tb;
        }
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        const unsigned long long f2 = __shfl_xor(feas, d, kWave), a2 = __shfl_xor(any, d, kWave);
        feas = f2 < feas ? f2 : feas;
        any = a2 < any ? a2 : any;
    }
    if (lane_id() == 0) {
        if (feas != ~0ull) atomicMin(&a.best_feasible[r], feas);
        if (any != ~0ull) atomicMin(&a.best_any[r], any);
    }
}

// The two selections of each request into Alg. 1's answer; they are set back to all ones.
__global__ __launch_bounds__(kBlock) void k_direct_finish(DirectArgs a)
{
    const int r = blockIdx.x * kBlock + threadIdx.x;
    if (r >= a.n) return;
    const unsigned long long feas = a.best_feasible[r], any = a.best_any[r];
    a.best_feasible[r] = ~0ull;
    a.best_any[r] = ~0ull;
    const bool found = feas != ~0ull;
    int g = -1;
    float T = 0.f;
    if (found) {
        g = a.order[(int)(feas >> 32)];
        T = from_ordered_bits((uint32_t)feas);
    } else if (any != ~0ull) {
        g = (int)(uint32_t)any;
        T = from_ordered_bits((uint32_t)(any >> 32));
    }
    a.out_inst[r] = g;
    a.out_slack[r] = g >= 0 ? a.budget[r] - T : 0.f;
    if (a.out_fallback) a.out_fallback[r] = !found;
}

__global__ void k_set_int(int* p, int v) { *p = v; }

// all ones = "no selection yet", for the first n requests of both halves
__global__ __launch_bounds__(kBlock) void k_fill_ones(unsigned long long* __restrict__ best, int n)
{
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i < n) {
        best[i] = ~0ull;
        best[kDirectMax + i] = ~0ull;
    }
}

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
unsigned long long* scratch_ptr[kMaxDevices];      // the array's address on each device, once asked for

template <typename K>
bool set_lds(K kernel, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess;
}

}  // namespace

size_t memo_lds_bytes(const gr_fleet* f)
{
    return sizeof(float) * 2 * kMemoTile + sizeof(int) * kMemoP * kMemoU + (size_t)kMemoP * f->cap * 2;
}

size_t score_lds_bytes(const gr_fleet* f)
{
    const size_t group = (size_t)f->bins * 4, memo = memo_lds_bytes(f);
    return group > memo ? group : memo;
}

// Dynamic LDS limits of the kernels that take more than the default.  The attribute belongs to
// the kernel, not to a handle: it is set to what the largest handle the library accepts needs
// (hard limits of gr_create), so a later, smaller handle cannot lower it for a live, larger one.
int score_prepare(gr_fleet*)
{
    constexpr size_t hist = (size_t)((kMaxLen + 2) / 2) * 4, scat = (size_t)(kMaxLen + 1) * 4;
    constexpr size_t memo = sizeof(float) * 2 * kMemoTile + sizeof(int) * kMemoP * kMemoU + (size_t)kMemoP * kMaxEntries * 2;
    constexpr size_t group = scat > memo ? scat : memo;
    const bool ok = set_lds(k_hist<false, 4>, hist) && set_lds(k_hist<true, 4>, hist) &&
                    set_lds(k_hist<false, 16>, hist) && set_lds(k_hist<true, 16>, hist) &&
                    set_lds(k_group<false, 4>, group) && set_lds(k_group<true, 4>, group);
    return ok ? GR_OK : GR_ERR_HIP;
}

// Alg. 1 pair by pair for up to kDirectMax requests; `best`: 2 * kDirectMax running selections,
// all ones on entry for the requests of this batch, and left so.
static int launch_direct(gr_fleet* f, const ReqSrc& src, const ScoreOut& out, unsigned long long* best, hipStream_t s)
{
    const int64_t n = src.n;
    DirectArgs d{};
    d.ctx0 = src.ctx0; d.pred_len = src.pred_len; d.budget = src.budget; d.exclude = src.exclude;
    d.order = f->order; d.hN = f->hN; d.cls = f->cls; d.inst_class = f->inst_class;
    d.tabR = f->tabR; d.tabGH = f->tabGH; d.headGH = f->headGH; d.posK = f->posK;
    d.best_feasible = best; d.best_any = best + kDirectMax;
    d.out_inst = out.inst; d.out_slack = out.slack; d.out_fallback = out.fallback; d.out_T = out.T;
    d.n = (int)n; d.n_inst = f->n_inst; d.m_pad = f->m_pad; d.cap = f->cap; d.max_len = f->max_len;
    d.keep = (float)(1.0 - f->lam_built);
    {
        ProfScope ps(f, kDirect, s);
        hipLaunchKernelGGL(k_direct, dim3((f->m_pad + kBlock - 1) / kBlock, (unsigned)n), dim3(kBlock), 0, s, d);
    }
    {
        ProfScope ps(f, kDirectFinish, s);
        hipLaunchKernelGGL(k_direct_finish, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, d);
    }
    return hipGetLastError() == hipSuccess ? GR_OK : GR_ERR_HIP;
}

// Whether a scoring pass on stream `s` has to make the capability order first.
static int ranks_needed(const gr_fleet* f, hipStream_t s, bool* needed)
{
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &capturing) != hipSuccess) return GR_ERR_HIP;
    *needed = !f->ranks_current || capturing != hipStreamCaptureStatusNone;
    return GR_OK;
}

int static_scratch(int device, unsigned long long** out)
{
    if (device < 0 || device >= kMaxDevices) return GR_ERR_TOO_LARGE;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[device]) {
        int current = -1;
        if (hipGetDevice(&current) != hipSuccess || current != device) return GR_ERR_INVALID_ARG;
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GR_ERR_HIP;
        scratch_ptr[device] = static_cast<unsigned long long*>(p);
    }
    *out = scratch_ptr[device];
    return GR_OK;
}

int launch_score_static(gr_fleet* f, const ReqSrc& src, const ScoreOut& out, hipStream_t s)
{
    if (src.n == 0) return GR_OK;
    if (src.n > kDirectMax) return GR_ERR_TOO_LARGE;
    unsigned long long* best = nullptr;
    const int rc = static_scratch(f->device, &best);
    if (rc != GR_OK) return rc;
    // the array keeps whatever the last call on this GPU left (a call that was cut short may
    // have left selections behind): set this batch's slots before use, with a kernel, so that
    // the call can be recorded into a graph
    hipLaunchKernelGGL(k_fill_ones, dim3((unsigned)((src.n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, best, (int)src.n);
    if (hipGetLastError() != hipSuccess) return GR_ERR_HIP;
    bool with_ranks = false;       // the capability order of the current status (two small kernels, no allocation)
    if (ranks_needed(f, s, &with_ranks) != GR_OK) return GR_ERR_HIP;
    if (with_ranks) {
        const int rc2 = launch_ranks(f, nullptr, s);
        if (rc2 != GR_OK) return rc2;
    }
    return launch_direct(f, src, out, best, s);
}

int launch_score(gr_fleet* f, const ReqSrc& src, bool migrate, const ScoreOut& out, hipStream_t s,
                 bool small_batch_ok)
{
    const int64_t n = src.n;
    if (n == 0) {
        if (out.n_selected) hipLaunchKernelGGL(k_set_int, dim3(1), dim3(1), 0, s, out.n_selected, 0);
        return hipGetLastError() == hipSuccess ? GR_OK : GR_ERR_HIP;
    }
    // up to about two million pairs (the default) a thread per pair is cheaper than the five kernels
    // of the grouped pass
    // The capability order of the current status, if nobody has made it yet, comes first.  While
    // the stream is being captured it always does: a recorded pass may be replayed after a status
    // build that was recorded elsewhere.
    bool with_ranks = false;
    if (ranks_needed(f, s, &with_ranks) != GR_OK) return GR_ERR_HIP;
    if (small_batch_ok && !migrate && n <= kDirectMax && n * f->m_pad <= f->small_batch_pairs) {
        if (with_ranks) {
            const int rc = launch_ranks(f, nullptr, s);
            if (rc != GR_OK) return rc;
        }
        return launch_direct(f, src, out, f->direct_best, s);
    }
    // In the grouped pass it rides along with the first two launches.
    const RankArgs ranks = rank_args(f, nullptr);
    const int rank_bx = with_ranks ? (f->n_inst + kWave - 1) / kWave : 0;
    const int rank_blocks = rank_bx * ((f->n_inst + kGroupBlock - 1) / kGroupBlock);
    const int bins = f->bins;
    // Requests per thread of the grouping kernels.  Every workgroup pays a pass over all length
    // bins and one global atomic per length it has seen, so the histogram of a large batch is
    // faster with few large workgroup shares.  The scatter keeps what it has read of its requests
    // in registers until their slots are known: four requests per thread leave room for two
    // workgroups on a compute unit (with eight, the tabulating workgroups that share its launch
    // lose more than the scatter gains: 80 against 62 us on 2.1 M requests).
    const int h_items = n > (int64_t(1) << 20) ? 16 : 4;
    constexpr int kScatterItems = 4;
    const auto blocks_for = [n](int items) {
        return (unsigned)((n + (int64_t)kGroupBlock * items - 1) / ((int64_t)kGroupBlock * items));
    };
    size_t hist_lds = (size_t)((bins + 1) / 2) * 4;
    const size_t scat_lds = (size_t)bins * 4;
    if (hist_lds < kGroupBlock * sizeof(double)) hist_lds = kGroupBlock * sizeof(double);   // (the counting step's competitors)
    const int off = migrate ? kHistMigrate - kHistRoute : 0;
    {
        ProfScope ps(f, kHistRoute + off, s);
#define GR_LAUNCH_HIST(M, I) hipLaunchKernelGGL((k_hist<M, I>), dim3(blocks_for(I) + rank_blocks), dim3(kGroupBlock), hist_lds, s, src, \
                                                f->len_cnt, bins, f->max_len, (int)blocks_for(I), ranks, rank_bx)
        if (migrate) { if (h_items == 16) GR_LAUNCH_HIST(true, 16); else GR_LAUNCH_HIST(true, 4); }
        else { if (h_items == 16) GR_LAUNCH_HIST(false, 16); else GR_LAUNCH_HIST(false, 4); }
#undef GR_LAUNCH_HIST
    }
    {
        ProfScope ps(f, kScanRoute + off, s);
        const int final_blocks = with_ranks ? (f->m_pad + kScanBlock - 1) / kScanBlock : 0;
        hipLaunchKernelGGL(k_scan, dim3(kScanGroups + final_blocks), dim3(kScanBlock), 0, s, f->len_cnt, f->len_base, f->row_len,
                           f->row_off, f->tile_off, f->len_row, f->len_ceil, f->totals, out.n_selected, bins, ranks);
    }
    if (with_ranks) f->ranks_current = true;
    const int64_t max_rows = n < bins ? n : bins;
    {
        ScatterArgs sc{};
        sc.s = src; sc.len_cnt = f->len_cnt; sc.len_base = f->len_base; sc.rank = f->rank; sc.recs = f->recs;
        sc.out_inst = out.inst; sc.out_slack = out.slack; sc.bins = bins; sc.max_len = f->max_len; sc.n_inst = f->n_inst;
        MemoArgs m{};
        m.totals = f->totals; m.row_len = f->row_len; m.len_ceil = f->len_ceil; m.order = f->order; m.hN = f->hN;
        m.cls = f->cls; m.inst_class = f->inst_class;
        m.tabR = f->tabR; m.tabGH = f->tabGH; m.headGH = f->headGH; m.memo = f->memo; m.grp_min = f->grp_min; m.grp_k = f->grp_k; m.posK = f->posK; m.tile_off = f->tile_off; m.tile_row = f->tile_row; m.row_cap = (int)f->row_cap;
        m.n_inst = f->n_inst; m.m_pad = f->m_pad; m.cap = f->cap; m.keep = (float)(1.0 - f->lam_built);
        // every memo workgroup walks all lengths; with few instances the lengths are dealt out to several
        const int gx = f->m_pad / kMemoP;
        const int64_t chunks = (max_rows + kMemoU - 1) / kMemoU;
        int gy = gx >= 512 ? 1 : 512 / gx;
        if (gy > chunks) gy = (int)chunks;
        const size_t memo_lds = memo_lds_bytes(f), lds = scat_lds > memo_lds ? scat_lds : memo_lds;
        ProfScope ps(f, kGroupRoute + off, s);
#define GR_LAUNCH_GROUP(M, I) hipLaunchKernelGGL((k_group<M, I>), dim3(gx * gy + blocks_for(I)), dim3(kGroupBlock), lds, s, sc, m, gx, gy)
        if (migrate) GR_LAUNCH_GROUP(true, kScatterItems);
        else GR_LAUNCH_GROUP(false, kScatterItems);
#undef GR_LAUNCH_GROUP
    }
    {
        TileArgs t{};
        t.totals = f->totals; t.row_len = f->row_len; t.row_off = f->row_off; t.tile_off = f->tile_off;
        t.order = f->order; t.recs = f->recs; t.memo = f->memo; t.posK = f->posK; t.grp_min = f->grp_min; t.grp_k = f->grp_k; t.tile_row = f->tile_row; t.row_cap = (int)f->row_cap;
        t.out_inst = out.inst; t.out_slack = out.slack; t.out_fallback = out.fallback; t.out_T = out.T;
        t.n_inst = f->n_inst; t.m_pad = f->m_pad;
        const int64_t max_tiles = (n + kTileReq - 1) / kTileReq + max_rows;
        // 24 waves per compute unit (6 per SIMD): the coefficient pairs go to LDS when the
        // 24 / kW workgroups resident together have room for a copy each
        const size_t k_bytes = (size_t)(f->m_pad + f->m_pad / kMemoP) * sizeof(float2);
        // (12 waves per workgroup measured 1 % faster than 8 at 4 096 instances, 4 % slower at 1 024.
        // Up to 1 024 instances seven copies fit as well: workgroups of 4 waves at 7 waves per SIMD --
        // a few registers of each lane then live in scratch memory -- are 3 % faster at 1 024
        // instances, where the short rows leave the vector ALU idle a fifth of the time at 6, and
        // 5 % slower at 256, where a tile is a chain of dependent loads and little else.)
        const int kw = (f->m_pad >= 512 && k_bytes <= 8704) ? 7 : k_bytes <= 24576 ? 8 : k_bytes <= 65536 ? 12 : 4;
        const int wg = kw == 7 ? 4 : kw;              // waves per workgroup
        unsigned blocks = (unsigned)((max_tiles + wg - 1) / wg);
        blocks = (blocks + 8u * kXcdRun - 1) / (8u * kXcdRun) * (8u * kXcdRun);
        ProfScope ps(f, kTileRoute + off, s);
#define GR_LAUNCH_TILE(W, E, L) \
        if (out.T) hipLaunchKernelGGL((k_tile<true, W, E>), dim3(blocks), dim3(W * kWave), L, s, t); \
        else hipLaunchKernelGGL((k_tile<false, W, E>), dim3(blocks), dim3(W * kWave), L, s, t)
        if (kw == 7) { GR_LAUNCH_TILE(4, 7, k_bytes); }
        else if (kw == 8) { GR_LAUNCH_TILE(8, 6, k_bytes); }
        else if (kw == 12) { GR_LAUNCH_TILE(12, 6, k_bytes); }
        else { GR_LAUNCH_TILE(4, 6, 0); }
#undef GR_LAUNCH_TILE
    }
    return hipGetLastError() == hipSuccess ? GR_OK : GR_ERR_HIP;
}

int launch_hits(gr_fleet* f, const ReqSrc& src, const int* hit_off, const int* hit_inst, const int* hit_len,
                int64_t n_hits, const ScoreOut& out, hipStream_t s)
{
    if (src.n == 0 || n_hits == 0) return GR_OK;
    HitArgs h{};
    h.ctx0 = src.ctx0; h.pred_len = src.pred_len; h.budget = src.budget; h.exclude = src.exclude;
    h.hit_off = hit_off; h.hit_inst = hit_inst; h.hit_len = hit_len;
    h.len_row = f->len_row; h.rank = f->rank; h.order = f->order; h.memo = f->memo; h.posK = f->posK;
    h.out_inst = out.inst; h.out_slack = out.slack; h.out_fallback = out.fallback; h.out_T = out.T;
    h.n = src.n; h.n_hits = n_hits; h.n_inst = f->n_inst; h.m_pad = f->m_pad; h.max_len = f->max_len;
    ProfScope ps(f, kHitsRoute, s);
    hipLaunchKernelGGL(k_hits, dim3((unsigned)((src.n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, h);
    return hipGetLastError() == hipSuccess ? GR_OK : GR_ERR_HIP;
}

}  // namespace gr
