// Token timelines (Sec. 4.3), statistics pass of disco_eval_migration.
//
// The delivery recurrence delta_t = max(r_t, delta_{t-1} + tau) is a running
// maximum in the shifted domain u_t = r_t - t tau: delta_t = fma(t, tau, M_t),
// M_t = max_{v<=t} u_v.  It does not depend on the pair's TTFT, so a request
// has one timeline per source and kind of hand-off, shared by all the policy
// columns that pick it.  Per-column statistics need, of each timeline, only
// its final maximum M (last delivery fma(n-1, tau, M)) and its hand-off index.
//
// The pass is split so that the one kernel that touches the token array does
// nothing else:
//   k_tl_flags   lane = request: which timelines of the request are not known
//                in closed form and have to be walked (one byte per request)
//   k_tl_walk    the token walk: one wave per request at a time, 256 arrival
//                offsets per step (one 16-byte load per lane, the next two
//                steps and the next request's first one in flight), one fma
//                and one max per token; the lag trigger is only screened by
//                a proven necessary condition; batches of requests are handed
//                out through device-wide counters, since the token count of
//                a batch varies by far more than its mean; leaves 16 bytes
//                per request (TlSummary)
//   k_tl_walk_rest  the requests the screening flags, walked exactly; sources
//                without a token array and slow device sources
//   k_tl_accum   lane = column: per-column totals from the summaries (the pairs with a buffer hand-off are
//                added by the kernel that settles those hand-offs)
//   k_tl_mat     optional per-pair outputs from the summaries
#include <string.h>

#include "disco_tl_walk.h"

namespace {

constexpr int TW_BLOCK = 256;                // 4 waves
constexpr int TW_WAVES = TW_BLOCK / 64;
constexpr int TW_NV = 1;                     // 16-byte vectors per lane and iteration of the general walker

// ---------------------------------------------------------------- flags ----

// The window of a request in the token array starts at the 128-byte boundary at or below its first token, so
// that the 1 KB a wave loads per iteration is eight whole cache lines and no line is fetched by two loads of the
// request: the tokens are read once, and the loads carry the streaming (non-temporal) hint, which this GPU
// serves about a tenth faster than plain loads but which keeps no line for a second touch.
__device__ __forceinline__ int window_lead(const float* first) { return (int)(((uintptr_t)first >> 2) & 31u); }


__global__ __launch_bounds__(256) void k_tl_flags(TraceView tr, i64 n_tok, const disco_policy* __restrict__ pol, int P, float tau,
                                                  unsigned char* __restrict__ wflags, unsigned* __restrict__ counters, int ncounters)
{
    __shared__ disco_policy sp[DISCO_MAX_COLS];
    if (blockIdx.x == 0)                                     // the walk's batch counters start at zero
        for (int w = threadIdx.x; w < ncounters; w += blockDim.x) counters[w] = 0u;
    if ((int)threadIdx.x < P) sp[threadIdx.x] = pol[threadIdx.x];
    __syncthreads();
    const bool mem = tr.arr != nullptr;
    for (i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x; i < tr.n_req; i += (i64)gridDim.x * blockDim.x) {
        const int l = tr.l[i];
        const float s = tr.s[i];
        const float k = tr.k ? tr.k[i] : tr.k_s;
        const float gd = tr.g ? tr.g[i] : tr.g_s;
        const float gap = tr.tbt ? tr.tbt[i] : 0.0f;
        u64 m[TL_KINDS];
        request_sets(sp, P, l, s, __fmaf_rn((float)l, k, tr.c), i, m);
        const bool srv_closed = pure_pacing(!mem, gap, tau);
        unsigned f = 0;
        if (m[TL_SRV_LAG] != 0ull && !srv_closed) f |= WF_LAG;
        // (a buffer hand-off timeline that never hands off is the source's own timeline: the kernel of those
        // pairs takes its final maximum from here instead of walking it)
        if ((m[TL_SRV] | m[TL_SRV_BUF]) != 0ull && !srv_closed) f |= WF_PLAIN;
        if ((m[TL_DEV] | m[TL_DEV_BUF]) != 0ull && !pure_pacing(true, gd, tau)) f |= WF_DEV;
        // the streaming walk loads 16 bytes per lane without bounds checks, from the 128-byte boundary at or below
        // the request's first token: the requests at the very ends of the token array, where such a load could
        // leave it, are left to the general walker
        if (mem && (f & (WF_LAG | WF_PLAIN)) != 0u) {
            const i64 off = tr.off[i];
            if (off + tr.n[i] + 3 > n_tok || off < (i64)window_lead(tr.arr + off)) f |= WF_REDO;
        }
        wflags[i] = (unsigned char)f;
    }
}

// ----------------------------------------------------------------- walk ----

struct WalkRes { int m; float Mlane; float C; };     // hand-off index (-1 none), this lane's partial maximum, u_0

// Four consecutive arrival offsets from an address that is only 4-byte aligned (a request starts anywhere in
// the token array); gfx950 serves such a 16-byte load in one instruction.
typedef float Float4U __attribute__((ext_vector_type(4), aligned(4)));

__device__ __forceinline__ void load4u(const float* __restrict__ arr, i64 g, i64 n_tok, bool safe, float r[4])
{
    if (safe || g + 3 < n_tok) {
        const Float4U v = *reinterpret_cast<const Float4U*>(arr + g);
        r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) r[k] = (g + k < n_tok) ? arr[g + k] : 0.0f;
    }
}

// Arrival offsets of one iteration of a request: vector v of a lane holds the tokens t0 + 256 v + 4 lane .. + 3;
// vectors that start beyond the request are not loaded.  `safe`: every such load of the request lies inside
// the token array.
template <int NV>
__device__ __forceinline__ void load_span(const float* __restrict__ arr, i64 g0, int tk0, int n, i64 n_tok, bool safe,
                                          float out[NV][4])
{
#pragma unroll
    for (int v = 0; v < NV; ++v)
        if (tk0 + 256 * v < n) load4u(arr, g0 + 256 * v, n_tok, safe, out[v]);
}

// What the screening of the lag trigger needs once per launch (see lag_fast_ok).
struct LagConst { float n_max; float c_max; bool kt_ok; };

// Exact evaluation of the lag trigger over one iteration of a walk (rare: only where the screening condition
// holds); it recomputes what it needs from the arrivals, so that the streaming loop keeps nothing alive for it.  r: the arrivals of the iteration as loaded;
// before: this lane's maximum of u over the earlier iterations.  Tokens are taken 256 at a time: running maximum
// before each token, then slot = delta_{t-1} + tau and lag = r_t - slot as defined (Sec. 4.3 pacing).  Returns
// the hand-off index (-1 none) and, after a hand-off, the device's arrival base and gap; imax = this lane's
// maximum of u over the iteration with the device's arrivals spliced in from the hand-off on.
struct ExactOut { int m; float base, g_dev, imax; };

template <int NV>
__device__ __forceinline__ ExactOut lag_exact(const int32_t* __restrict__ pl, const float* __restrict__ pk,
                                                        const float* __restrict__ pg, float k_s, float g_s, float c, i64 i,
                                                        int n, int e0, int lane, float Mlane, const float rin[NV][4],
                                                        float tau, float kt)
{
    const float ninf = -INFINITY;
    const float ntau = -tau;
    const int lane4 = 4 * lane;
    float r[NV][4], u[NV][4], tf[NV][4], iv[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const float t0 = (float)(lane4 + e0 + 256 * v);
        tf[v][0] = t0; tf[v][1] = t0 + 1.0f; tf[v][2] = t0 + 2.0f; tf[v][3] = t0 + 3.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            r[v][q] = rin[v][q];
            asm volatile("" : "+v"(r[v][q]));            // a fresh value: nothing of the streaming loop is kept alive for this path
            u[v][q] = (lane4 + e0 + 256 * v + q < n) ? __fmaf_rn(tf[v][q], ntau, r[v][q]) : ninf;
        }
        iv[v] = fmaxf(fmaxf(u[v][0], u[v][1]), fmaxf(u[v][2], u[v][3]));
    }
    ExactOut o{-1, 0.0f, 0.0f, ninf};
    float before = wave_max_f32(Mlane);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        if (o.m < 0) {
            const int tk0 = lane4 + e0 + 256 * v;
            const float i0 = u[v][0], i1 = fmaxf(i0, u[v][1]), i2 = fmaxf(i1, u[v][2]);
            const float incl = wave_incl_max_dpp(iv[v], lane);
            const float E = fmaxf(wave_prev(incl, ninf), before);
            const float ex[4] = {E, fmaxf(E, i0), fmaxf(E, i1), fmaxf(E, i2)};
            bool trig[4];
            float slot[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                slot[q] = __fmaf_rn(tf[v][q] - 1.0f, tau, ex[q]) + tau;        // delta_{t-1} + tau
                const float lg = r[v][q] - slot[q];
                trig[q] = (unsigned)(tk0 + q - 1) < (unsigned)(n - 1) && lg > kt;      // tokens 1 .. n-1
            }
            const u64 any = __ballot(trig[0] || trig[1] || trig[2] || trig[3]);
            if (any) {
                const int ml = __ffsll((long long)any) - 1;
                const int qf = trig[0] ? 0 : (trig[1] ? 1 : (trig[2] ? 2 : 3));
                const float sl = trig[0] ? slot[0] : (trig[1] ? slot[1] : (trig[2] ? slot[2] : slot[3]));
                const int m = bcast_i(tk0, ml) + bcast_i(qf, ml);
                // hand-off: decided once the token is kappa*tau overdue; the device re-prefills the
                // prompt plus the m tokens already produced, then generates at its own pace
                const int l = pl[i];
                const float k = pk ? pk[i] : k_s;
                const float g_dev = pg ? pg[i] : g_s;
                const float t_dec = bcast_f(sl, ml) + kt;
                const float t_mig = __fmaf_rn((float)(l + m), k, c);
                const float base = t_dec + t_mig;
                o.m = m; o.base = base; o.g_dev = g_dev;
#pragma unroll
                for (int w = v; w < NV; ++w) {
                    const int tw0 = lane4 + e0 + 256 * w;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (tw0 + q >= m) {
                            const float rd = __fmaf_rn((float)(tw0 + q - m + 1), g_dev, base);
                            u[w][q] = (tw0 + q < n) ? __fmaf_rn(tf[w][q], ntau, rd) : ninf;
                        }
                    iv[w] = fmaxf(fmaxf(u[w][0], u[w][1]), fmaxf(u[w][2], u[w][3]));
                }
            } else if (v + 1 < NV) {
                before = fmaxf(before, wave_max_f32(iv[v]));
            }
        }
    }
#pragma unroll
    for (int v = 0; v < NV; ++v) o.imax = fmaxf(o.imax, iv[v]);
    return o;
}

// Walk of one request and source: hand-off index and the per-lane maximum of u over the lane's tokens.
//   mem   arrivals from the CSR token array (first iteration already in `cur`), else t * gap
//   lag   evaluate the lag trigger wherever the necessary condition stated above lag_fast_ok holds, with
//         C = u_0 (a lower bound of every later running maximum)
//   i     the request (its prompt length and device speeds are fetched only when a hand-off fires)
template <int NV>
__device__ __forceinline__ WalkRes walk_request(const TraceView& tr, bool mem, i64 i, int n, i64 off, i64 n_tok, float cur[NV][4],
                                                float gap, bool lag, float tau, float kt, const LagConst& lc, int lane,
                                                float lane4f)
{
    const float ninf = -INFINITY;
    const float ntau = -tau;
    const int lane4 = 4 * lane;
    const i64 gbase = off + lane4;
    const bool safe = mem && off + n + 3 <= n_tok;
    const int lim = n - lane4;                               // tokens of the request from this lane's first one on
    int m = -1;
    float base = 0.0f, g_dev = 0.0f;
    float Mlane = ninf;
    const float C = mem ? bcast_f(cur[0][0], 0) : 0.0f;      // u_0 = r_0
    const bool cheap = lc.kt_ok && (float)n + 2.0f <= lc.n_max && fabsf(C) <= lc.c_max;
    const float thr = C + 0.5f * kt;
#pragma unroll 1
    for (int e0 = 0; e0 < n; e0 += 256 * NV) {
        float r[NV][4], u[NV][4];
        float tf[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) tf[v] = lane4f + (float)(e0 + 256 * v);        // exact: token indices are far below 2^24
        if (m >= 0) {
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int q = 0; q < 4; ++q) r[v][q] = __fmaf_rn((float)(lane4 + e0 + 256 * v + q - m + 1), g_dev, base);
        } else if (mem) {
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int q = 0; q < 4; ++q) r[v][q] = cur[v][q];
            if (e0 + 256 * NV < n)                           // next iteration in flight
                load_span<NV>(tr.arr, gbase + e0 + 256 * NV, lane4 + e0 + 256 * NV, n, n_tok, safe, cur);
        } else {
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int q = 0; q < 4; ++q) r[v][q] = (tf[v] + (float)q) * gap;
        }
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int q = 0; q < 4; ++q) u[v][q] = __fmaf_rn(tf[v] + (float)q, ntau, r[v][q]);
        if (e0 + 256 * NV > n) {                             // the request ends inside this iteration
            const int left = lim - e0;
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int q = 0; q < 4; ++q) u[v][q] = (256 * v + q < left) ? u[v][q] : ninf;
        }
        float imax = ninf;
#pragma unroll
        for (int v = 0; v < NV; ++v) imax = fmaxf(imax, fmaxf(fmaxf(u[v][0], u[v][1]), fmaxf(u[v][2], u[v][3])));
        if (lag && m < 0 && (!cheap || __ballot(imax > thr) != 0ull)) {
            const ExactOut x = lag_exact<NV>(tr.l, tr.k, tr.g, tr.k_s, tr.g_s, tr.c, i, n, e0, lane, Mlane, r, tau, kt);
            m = x.m; base = x.base; g_dev = x.g_dev;
            imax = x.imax;
        }
        Mlane = fmaxf(Mlane, imax);
    }
    return WalkRes{m, Mlane, C};
}

struct WalkArgs {
    float tau, kt;
    int rb;                        // requests per batch (<= TF_RB)
    unsigned char* wflags;
    TlSummary* summary;
    unsigned* counter;             // per queue, 128 bytes apart: positions of the queue handed out so far
    int nqueue;                    // queues: workgroup b and batch j belong to queue b % nqueue, j % nqueue
};

// Batches are handed out dynamically because their token counts differ by far more than their mean (half of
// the requests of a budget sweep need no walk at all, the others have log-normal lengths): a static deal leaves
// the slowest wave with well over 1.5 times the mean.  One device-wide counter would serialise every claim on
// one address (about 10 ns each: longer than a batch takes the chip), so workgroups and batches are dealt
// round-robin to TW_QUEUES queues with a counter each.
constexpr int TW_QUEUES = 32;
constexpr int TW_COUNTER_STRIDE = 32;        // words between the counters of two queues

// Row maxima of a lane's partial maximum -> LDS (lanes 15, 31, 47, 63 hold the maxima of their rows of 16).
__device__ __forceinline__ void put_rows(float v, float* dst4, int lane)
{
    const float ninf = -INFINITY;
    v = fmaxf(v, dpp_mov<0x111>(ninf, v));
    v = fmaxf(v, dpp_mov<0x112>(ninf, v));
    v = fmaxf(v, dpp_mov<0x114>(ninf, v));
    v = fmaxf(v, dpp_mov<0x118>(ninf, v));
    if ((lane & 15) == 15) dst4[lane >> 4] = v;
}

// One 16-byte vector per lane of a window's elements t0 + 4 lane .. + 3 (p: the window's first element; lane4u:
// 4 lane; n: elements of the window).  Lanes beyond the window load nothing; its last vector may reach up to
// three elements past it, which the caller has made sure lie inside the token array, like its first one.  The address is a uniform
// base plus a 32-bit lane offset, which costs no vector arithmetic.
__device__ __forceinline__ void load_vec(const float* __restrict__ p, int t0, unsigned lane4u, int n, float out[4])
{
    const float* q = p + t0;
    if (t0 + 256 <= n || (int)lane4u + t0 < n) {             // (a full iteration: every lane loads)
        const Float4U v = __builtin_nontemporal_load(reinterpret_cast<const Float4U*>(q + lane4u));
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    }
}

// The streaming walk: the server-sourced timeline of every request that has one in the token array, as long as
// nothing but the running maximum is asked of it.  256 tokens per iteration (one 16-byte load per lane), the two
// following iterations of the request and the first one of the next request in flight; per token one fma
// (u_t = r_t - t tau) and one max.  Where a column wants the lag trigger, the maximum so far is compared once
// per round of three iterations with the bound of the necessary condition (see lag_fast_ok): a request that
// passes it could hold a hand-off and is left, flagged WF_REDO, to the kernel behind this one, which evaluates
// the trigger exactly.  Everything per request is either done for the whole batch at once (lane = request) or
// kept in scalar registers.
enum { WP_NOK = 32 };                                        // beside the walk flags in a request's packed word

__global__ __launch_bounds__(TW_BLOCK) void k_tl_walk(TraceView tr, i64 n_tok, WalkArgs a)
{
    __shared__ __align__(16) float red[TW_WAVES][TF_RB][4];   // row maxima per wave and request of the batch
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned lane4u = 4u * (unsigned)lane;
    const float lane4f = (float)lane4u;
    const float ninf = -INFINITY;
    const float tau = a.tau, kt = a.kt, ntau = -a.tau;
    const LagConst lc{262144.0f * (kt / tau), 262144.0f * kt, kt >= tau * 0.0009765625f};
    const float half_kt = 0.5f * kt;
    const int rb = a.rb;
    const i64 nbatch = (tr.n_req + rb - 1) / rb;
    // this wave's queue: position k of queue q is batch q + nqueue k
    const int nqueue = a.nqueue, queue = (int)(blockIdx.x % (unsigned)nqueue);
    unsigned* counter = a.counter + (size_t)queue * TW_COUNTER_STRIDE;
    // lane = request of a batch: output length, token offset, packed word (walk flags; WP_NOK: short enough for
    // the screening), all 0 beyond the batch or trace
    struct Meta { int n; i64 off; unsigned pk; };
    auto load_meta = [&](i64 bt) {
        Meta x{1, 0, 0u};
        const i64 i = bt * rb + lane;
        if (bt < nbatch && lane < rb && i < tr.n_req) {
            x.pk = a.wflags[i];
            x.n = tr.n[i];
            x.off = tr.off[i];
            if (lc.kt_ok && (float)x.n + 2.0f <= lc.n_max) x.pk |= WP_NOK;
        }
        return x;
    };
    unsigned claimed = 0u;
    if (lane == 0) claimed = atomicAdd(counter, 2u);         // the first two positions at once
    const i64 first_pos = (i64)(unsigned)__builtin_amdgcn_readfirstlane((int)claimed);
    i64 cur_id = queue + nqueue * first_pos, nxt_id = queue + nqueue * (first_pos + 1);
    Meta cur = load_meta(cur_id);
    float (*myred)[4] = red[wave];
    // (Choosing a batch's first walk, and issuing its load, while the batch before it is still being walked was
    // tried: the bookkeeping cost a tenth of the kernel's time, more than the latency it hid.)
    while (cur_id < nbatch) {
        const Meta nxt = load_meta(nxt_id);                  // in flight while this batch is walked
        claimed = 0u;
        if (lane == 0 && nxt_id < nbatch) claimed = atomicAdd(counter, 1u);
        u64 todo = __ballot((cur.pk & (WF_LAG | WF_PLAIN)) != 0u && (cur.pk & WF_REDO) == 0u);
        int marks = 0;                                       // lane = request: bit 0 walk again exactly, bit 1 first offset not 0
        // the request about to be walked, in scalars (window length and lead, packed word, window start), its
        // first iteration in `pre`
        float pre[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        int n = 1, mis = 0;                                  // n: elements of the window = lead + tokens of the request
        unsigned pk = 0u;
        const float* p = tr.arr;
        int rq = -1;
        if (todo) {
            rq = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            n = bcast_i(cur.n, rq);
            pk = (unsigned)bcast_i((int)cur.pk, rq);
            const i64 off = (i64)bcast_u64((u64)cur.off, rq);
            mis = window_lead(tr.arr + off);
            p = tr.arr + off - mis; n += mis;
            load_vec(p, 0, lane4u, n, pre);
        }
        while (rq >= 0) {
            const bool lag = (pk & WF_LAG) != 0u;
            // three register sets take turns (no copies: a copy would wait for the load it moves)
            float x[4] = {pre[0], pre[1], pre[2], pre[3]};
            float y[4] = {0.0f, 0.0f, 0.0f, 0.0f}, z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (n > 256) load_vec(p, 256, lane4u, n, y);
            if (n > 512) load_vec(p, 512, lane4u, n, z);
            // the next request: its scalars, and its first iteration in flight
            int rq1 = -1, n1 = 1, mis1 = 0;
            unsigned pk1 = 0u;
            const float* p1 = tr.arr;
            if (todo) {
                rq1 = __ffsll((long long)todo) - 1;
                todo &= todo - 1;
                n1 = bcast_i(cur.n, rq1);
                pk1 = (unsigned)bcast_i((int)cur.pk, rq1);
                const i64 off1 = (i64)bcast_u64((u64)cur.off, rq1);
                mis1 = window_lead(tr.arr + off1);
                p1 = tr.arr + off1 - mis1; n1 += mis1;
                load_vec(p1, 0, lane4u, n1, pre);
            }
            const int mq = mis & 3;
            const float r0 = mq == 0 ? x[0] : (mq == 1 ? x[1] : (mq == 2 ? x[2] : x[3]));
            const float C = bcast_f(r0, mis >> 2);           // u_0 = r_0: element `mis` of the window
            const bool cheap = (pk & WP_NOK) != 0u && fabsf(C) <= lc.c_max;
            const float thr = lag ? C + half_kt : INFINITY;
            bool leave = lag && !cheap;                      // no screening possible: exact evaluation throughout
            float Mlane = ninf;
            float tf = lane4f - (float)mis;                  // this lane's first token index of the iteration (exact in fp32)
            // 256 tokens, arrivals in v, first token index of the lane tq: per-lane maximum, screening
            auto step = [&](const float v[4], float tq, int e) {
                float u0 = __fmaf_rn(tq, ntau, v[0]), u1 = __fmaf_rn(tq + 1.0f, ntau, v[1]);
                float u2 = __fmaf_rn(tq + 2.0f, ntau, v[2]), u3 = __fmaf_rn(tq + 3.0f, ntau, v[3]);
                if (e + 256 > n || e == 0) {                 // the request ends inside this iteration, or the window's lead is in it
                    // element index in the window, less the lead: valid iff in [0, n - mis)
                    const unsigned at = (unsigned)(e + (int)lane4u - mis), cnt = (unsigned)(n - mis);
                    u0 = at < cnt ? u0 : ninf; u1 = at + 1u < cnt ? u1 : ninf; u2 = at + 2u < cnt ? u2 : ninf; u3 = at + 3u < cnt ? u3 : ninf;
                }
                const float imax = fmaxf(fmaxf(u0, u1), fmaxf(u2, u3));
                Mlane = fmaxf(Mlane, imax);
            };
#pragma unroll 1
            for (int e0 = 0; e0 < n && !leave; e0 += 768) {
                step(x, tf, e0);
                if (e0 + 768 < n) load_vec(p, e0 + 768, lane4u, n, x);
                if (e0 + 256 < n) {
                    step(y, tf + 256.0f, e0 + 256);
                    if (e0 + 1024 < n) load_vec(p, e0 + 1024, lane4u, n, y);
                    if (e0 + 512 < n) {
                        step(z, tf + 512.0f, e0 + 512);
                        if (e0 + 1280 < n) load_vec(p, e0 + 1280, lane4u, n, z);
                    }
                }
                // screening once per round of 768 tokens: the maximum so far against the bound
                if (lag) leave = leave || __ballot(Mlane > thr) != 0ull;
                tf += 768.0f;
            }
            put_rows(Mlane, myred[rq], lane);
            const int mark = (leave ? 1 : 0) | ((f2u(C) & 0x7FFFFFFFu) != 0u ? 2 : 0);
            if (mark) marks = lane == rq ? mark : marks;
            rq = rq1; n = n1; pk = pk1; p = p1; mis = mis1;
        }
        __builtin_amdgcn_wave_barrier();                     // the row maxima were written by other lanes of this wave
        {
            const i64 i = cur_id * rb + lane;
            if (lane < rb && i < tr.n_req) {
                TlSummary s{0.0f, (marks & 2) ? -2 : -1, 0.0f, 0.0f};
                if ((cur.pk & (WF_LAG | WF_PLAIN)) != 0u && (cur.pk & WF_REDO) == 0u) {
                    const float4 v = *reinterpret_cast<const float4*>(myred[lane]);
                    s.M_lag = s.M_plain = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
                }
                a.summary[i] = s;
                if (marks & 1) a.wflags[i] = (unsigned char)((cur.pk & (WF_LAG | WF_PLAIN | WF_DEV)) | WF_REDO);
            }
        }
        __builtin_amdgcn_wave_barrier();
        cur = nxt;
        cur_id = nxt_id;
        nxt_id = nxt_id < nbatch ? queue + nqueue * (i64)(unsigned)__builtin_amdgcn_readfirstlane((int)claimed) : nbatch;
    }
}

// Everything the streaming walk leaves: requests it flagged WF_REDO (the lag trigger may fire: exact evaluation,
// and a second walk without hand-off where columns without hand-off share the request), server sources with a
// constant gap that is not pure pacing (no token array), and device sources that are not pure pacing.  Few
// requests; one wave per request and job with the general walker.  `streamed`: the streaming walk has run (else
// every server job is done here).
__global__ __launch_bounds__(TW_BLOCK) void k_tl_walk_rest(TraceView tr, i64 n_tok, WalkArgs a, int streamed)
{
    // row maxima per wave, slot (0 server walk, 1 server walk without hand-off beside a hand-off that fired,
    // 2 device source) and request of the batch
    constexpr int WR_RB = 64;                                // requests per wave and round: one flag byte per lane
    __shared__ __align__(16) float red[TW_WAVES][3][WR_RB][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float lane4f = (float)(4 * lane);
    const float tau = a.tau, kt = a.kt;
    const LagConst lc{262144.0f * (kt / tau), 262144.0f * kt, kt >= tau * 0.0009765625f};
    const bool mem = tr.arr != nullptr;
    float (*myred)[WR_RB][4] = red[wave];
    const i64 nbatch = (tr.n_req + WR_RB - 1) / WR_RB;
    for (i64 bt = (i64)blockIdx.x * TW_WAVES + wave; bt < nbatch; bt += (i64)gridDim.x * TW_WAVES) {
        const i64 first = bt * WR_RB;
        const i64 il = first + lane;
        const bool valid = il < tr.n_req;
        const unsigned f = valid ? a.wflags[il] : 0u;
        const bool srv_here = (f & (WF_LAG | WF_PLAIN)) != 0u && (!streamed || (f & WF_REDO) != 0u);
        u64 todo0 = __ballot(srv_here), todo1 = 0ull;
        u64 todo2 = __ballot((f & WF_DEV) != 0u);
        if ((todo0 | todo2) == 0ull) continue;               // (almost every batch)
        int n_v = 1;
        i64 off_v = 0;
        float gap_v = 0.0f;
        if (srv_here || (f & WF_DEV) != 0u) {
            n_v = tr.n[il];
            if (tr.off) off_v = tr.off[il];
            if (!mem && tr.tbt) gap_v = tr.tbt[il];
        }
        int m_enc = -1;                                      // lane = request
        bool two = false;                                    // a second server walk was needed
        while ((todo0 | todo1 | todo2) != 0ull) {
            const int slot = todo0 ? 0 : (todo1 ? 1 : 2);
            const u64 td = todo0 ? todo0 : (todo1 ? todo1 : todo2);
            const int rq = __ffsll((long long)td) - 1;
            if (slot == 0) todo0 &= todo0 - 1; else if (slot == 1) todo1 &= todo1 - 1; else todo2 &= todo2 - 1;
            const int n = bcast_i(n_v, rq);
            const unsigned fr = (unsigned)bcast_i((int)f, rq);
            const i64 off = (i64)bcast_u64((u64)off_v, rq);
            const bool job_mem = mem && slot < 2;
            const bool lag = slot == 0 && (fr & WF_LAG) != 0u;
            float gap = 0.0f;
            if (slot == 2) gap = tr.g ? tr.g[first + rq] : tr.g_s;
            else if (!mem) gap = bcast_f(gap_v, rq);
            float now[TW_NV][4];
#pragma unroll
            for (int v = 0; v < TW_NV; ++v) { now[v][0] = now[v][1] = now[v][2] = now[v][3] = 0.0f; }
            if (job_mem) load_span<TW_NV>(tr.arr, off + 4 * lane, 4 * lane, n, n_tok, off + n + 3 <= n_tok, now);
            const WalkRes w = walk_request<TW_NV>(tr, job_mem, first + rq, n, off, n_tok, now, gap, lag, tau, kt, lc, lane, lane4f);
            put_rows(w.Mlane, myred[slot][rq], lane);
            if (slot == 0) {
                const bool nz = w.C != 0.0f;
                const int enc = w.m >= 0 ? (w.m | (nz ? (1 << 30) : 0)) : (nz ? -2 : -1);
                m_enc = lane == rq ? enc : m_enc;
                if (w.m >= 0 && (fr & WF_PLAIN) != 0u) todo1 |= 1ull << rq;       // columns without hand-off share the request
            } else if (slot == 1) {
                two = lane == rq ? true : two;
            }
        }
        __builtin_amdgcn_wave_barrier();                     // the row maxima were written by other lanes of this wave
        if (srv_here || (f & WF_DEV) != 0u) {
            auto rowmax = [&](int slot) {
                const float4 x = *reinterpret_cast<const float4*>(myred[slot][lane]);
                return fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
            };
            TlSummary s = a.summary[il];                     // what the streaming walk left (all zero / none without it)
            if (srv_here) {
                s.M_lag = rowmax(0);
                s.m_enc = m_enc;
                s.M_plain = two ? rowmax(1) : s.M_lag;
            }
            if (f & WF_DEV) s.M_dev = rowmax(2);
            a.summary[il] = s;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Summaries of a trace without a token array: nothing streamed, every field at its closed-form value.
__global__ __launch_bounds__(256) void k_tl_summary_clear(i64 n_req, TlSummary* __restrict__ summary)
{
    for (i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x; i < n_req; i += (i64)gridDim.x * blockDim.x)
        summary[i] = TlSummary{0.0f, -1, 0.0f, 0.0f};
}

// ----------------------------------------------------------- accumulate ----

constexpr int TA_BLOCK = 1024;
constexpr int TA_WAVES = TA_BLOCK / 64;

struct AccStaged { int l, n; float s, d; TlSummary sum; };      // 32 bytes, one per request of a wave's batch

struct AccumArgs {
    float tau;
    int P, G;                      // columns, columns rounded up to a power of two
    const TlSummary* summary;
    MigPartial* totals;            // DISCO_NCOPY x 64 device-wide totals
};

// lane = sub * G + column (as in the dispatch passes): a batch of 64 requests is loaded one per lane, staged in
// LDS, and every column lane reads the G requests of its sub-group.  Pairs with a buffer hand-off are left to
// the kernel of that hand-off; n_tot counts the tokens of the pairs handled here.
__global__ __launch_bounds__(TA_BLOCK) void k_tl_accum(TraceView tr, const disco_policy* __restrict__ pol, AccumArgs a)
{
    __shared__ __align__(16) AccStaged stage[TA_BLOCK];
    __shared__ u64 sh[6 * TA_BLOCK];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int G = a.G, P = a.P;
    const int col = lane & (G - 1), sub = lane / G;
    const bool colv = col < P;
    const disco_policy p = pol[colv ? col : 0];
    const int mode = p.mode, mg = p.mig_mode;
    const bool dev_constrained = mode == DISCO_MODE_DEVICE_CONSTRAINED || mode == DISCO_MODE_STOCH_DEVICE;
    const float tau = a.tau;
    u64 acc_s_dec = 0, acc_repre = 0, acc_n = 0, tot_cnt = 0;
    unsigned acc_mig = 0;
    double acc_tlast = 0.0;
    AccStaged* st = stage + wave * 64;
    const i64 nbatch = (tr.n_req + 63) >> 6;
    for (i64 b = (i64)blockIdx.x * TA_WAVES + wave; b < nbatch; b += (i64)gridDim.x * TA_WAVES) {
        const i64 i = b * 64 + lane;
        AccStaged x{0, 1, 0.0f, 0.0f, TlSummary{0.0f, -1, 0.0f, 0.0f}};
        if (i < tr.n_req) {
            x.l = tr.l[i]; x.n = tr.n[i]; x.s = tr.s[i];
            x.d = __fmaf_rn((float)x.l, tr.k ? tr.k[i] : tr.k_s, tr.c);
            x.sum = a.summary[i];
            tot_cnt += (u64)(x.n - 1);
        }
        st[lane] = x;
        __builtin_amdgcn_wave_barrier();                     // the staging area is private to the wave
        const int cnt = (int)((tr.n_req - b * 64 < 64) ? (tr.n_req - b * 64) : 64);
        for (int it = 0; it < G; ++it) {
            const int src = sub * G + it;
            const AccStaged r = st[src];
            unsigned dec; float t;
            dispatch_pair(p, r.l, r.s, r.d, b * 64 + src, dec, t);
            const bool dev = (dec & 4u) != 0u;
            const bool buf = mg == DISCO_MIG_BUFFER && (dev == dev_constrained);
            if (!colv || src >= cnt || buf) continue;
            const bool lag = !dev && mg == DISCO_MIG_LAG;
            const int m = lag ? summary_m(r.sum.m_enc) : -1;
            const float M = dev ? r.sum.M_dev : (lag ? r.sum.M_lag : r.sum.M_plain);
            const float t_last = __fmaf_rn((float)(r.n - 1), tau, M);
            const int nsrc = dev ? 0 : (m >= 0 ? m : r.n);
            acc_s_dec += (u64)nsrc;
            acc_n += (u64)r.n;
            if (m >= 0) { acc_mig += 1u; acc_repre += (u64)r.l + (u64)m; }
            acc_tlast += (double)t_last;
        }
        __builtin_amdgcn_wave_barrier();
    }
    tot_cnt = wave_sum_u64(tot_cnt);
    // fold the request sub-groups of the wave
    for (int mk = G; mk < 64; mk <<= 1) {
        acc_s_dec += shfl_xor_u64(acc_s_dec, mk); acc_repre += shfl_xor_u64(acc_repre, mk); acc_n += shfl_xor_u64(acc_n, mk);
        acc_mig += (unsigned)__shfl_xor((int)acc_mig, mk, 64);
        acc_tlast += shfl_xor_f64(acc_tlast, mk);
    }
    // lane = column (sub-group 0): fold the waves of the workgroup, then add into this workgroup's copy of the totals
    sh[0 * TA_BLOCK + threadIdx.x] = acc_s_dec; sh[1 * TA_BLOCK + threadIdx.x] = acc_n - acc_s_dec;
    sh[2 * TA_BLOCK + threadIdx.x] = acc_repre; sh[3 * TA_BLOCK + threadIdx.x] = (u64)acc_mig;
    sh[4 * TA_BLOCK + threadIdx.x] = tot_cnt; sh[5 * TA_BLOCK + threadIdx.x] = (u64)__double_as_longlong(acc_tlast);
    __syncthreads();
    if ((int)threadIdx.x < P) {
        u64 f[5];
        double tl = 0.0;
        for (int q = 0; q < 5; ++q) f[q] = 0;
        for (int w = 0; w < TA_WAVES; ++w) {
            for (int q = 0; q < 5; ++q) f[q] += sh[q * TA_BLOCK + w * 64 + threadIdx.x];
            tl += __longlong_as_double((long long)sh[5 * TA_BLOCK + w * 64 + threadIdx.x]);
        }
        MigPartial* t = &a.totals[(blockIdx.x % DISCO_NCOPY) * 64 + threadIdx.x];
        atomicAdd((unsigned long long*)&t->s_dec, (unsigned long long)f[0]);
        atomicAdd((unsigned long long*)&t->d_dec, (unsigned long long)f[1]);
        atomicAdd((unsigned long long*)&t->d_repre, (unsigned long long)f[2]);
        atomicAdd((unsigned long long*)&t->migrated, (unsigned long long)f[3]);
        atomicAdd((unsigned long long*)&t->tbt_count, (unsigned long long)f[4]);
        unsafeAtomicAdd(&t->tlast_sum, tl);        // hardware fp64 add; order-dependent in its last bits
    }
}

// ----------------------------------------------------- per-pair outputs ----

struct MatArgs {
    float tau;
    int P;
    const TlSummary* summary;
    const BufSummary* bufsum;      // read when the staged table has a buffer hand-off column
    const unsigned* buffer_flag;
    int32_t* mig_idx; int32_t* n_src_tok; float* t_last; int32_t* delay_num;
};

// lane = request, so that every column is written coalesced.  A pair with a buffer hand-off (its source is the
// constrained endpoint of a column with that hand-off) reads the summary of that hand-off: the source's last
// token is m, the target takes over at m + 1.
__global__ __launch_bounds__(256) void k_tl_mat(TraceView tr, const disco_policy* __restrict__ pol, MatArgs a)
{
    __shared__ disco_policy sp[DISCO_MAX_COLS];
    if ((int)threadIdx.x < a.P) sp[threadIdx.x] = pol[threadIdx.x];
    __syncthreads();
    const bool any_buf = *a.buffer_flag != 0u;
    for (i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x; i < tr.n_req; i += (i64)gridDim.x * blockDim.x) {
        const int l = tr.l[i], n = tr.n[i];
        const float s = tr.s[i];
        const float d = __fmaf_rn((float)l, tr.k ? tr.k[i] : tr.k_s, tr.c);
        const TlSummary sum = a.summary[i];
        BufSummary bs{0.0f, -1, 0, 0, 0.0f, -1, 0, 0};
        if (any_buf) bs = a.bufsum[i];
        for (int j = 0; j < a.P; ++j) {
            unsigned dec; float t;
            dispatch_pair(sp[j], l, s, d, i, dec, t);
            const bool dev = (dec & 4u) != 0u;
            const int mg = sp[j].mig_mode, mode = sp[j].mode;
            const bool dev_constrained = mode == DISCO_MODE_DEVICE_CONSTRAINED || mode == DISCO_MODE_STOCH_DEVICE;
            int m, delay = 0;                                // first token of the target, -1: no hand-off
            float M;
            if (mg == DISCO_MIG_BUFFER && dev == dev_constrained) {
                const int last = summary_m(dev ? bs.m_d : bs.m_s);
                m = last >= 0 ? last + 1 : -1;
                M = dev ? bs.M_d : bs.M_s;
                if (last >= 0) delay = dev ? bs.delay_d : bs.delay_s;
            } else {
                const bool lag = !dev && mg == DISCO_MIG_LAG;
                m = lag ? summary_m(sum.m_enc) : -1;
                M = dev ? sum.M_dev : (lag ? sum.M_lag : sum.M_plain);
            }
            const size_t at = (size_t)j * tr.n_req + i;
            if (a.mig_idx) a.mig_idx[at] = m;
            if (a.n_src_tok) a.n_src_tok[at] = m >= 0 ? m : n;
            if (a.t_last) a.t_last[at] = __fmaf_rn((float)(n - 1), a.tau, M);
            if (a.delay_num) a.delay_num[at] = delay;
        }
    }
}

}  // namespace

// The token walk alone: flags, the streaming walk (traces with a token array), then what it leaves.  With
// events, the streaming kernel's launch is bracketed by them (measurement aid).
void disco_launch_tl_walk(const TraceView& v, i64 n_tok, const disco_policy* pol, int P, float tau, float kt,
                          unsigned char* wflags, void* summary, unsigned* counter, hipStream_t stream,
                          hipEvent_t before, hipEvent_t after)
{
    if (v.n_req <= 0) return;
    i64 fb = (v.n_req + 255) / 256;
    if (fb > 2048) fb = 2048;
    hipLaunchKernelGGL(k_tl_flags, dim3((unsigned)fb), dim3(256), 0, stream, v, n_tok, pol, P, tau, wflags, counter,
                       TW_QUEUES * TW_COUNTER_STRIDE);
    WalkArgs w;
    memset(&w, 0, sizeof(w));
    w.tau = tau; w.kt = kt;
    w.wflags = wflags; w.summary = (TlSummary*)summary; w.counter = counter;
    const bool mem = v.arr != nullptr;
    if (mem) {
        const i64 waves = 2048 * TW_WAVES;         // eight resident workgroups per CU
        w.rb = tl_batch(v.n_req, waves);
        const i64 per_block = (i64)TW_WAVES * w.rb;
        i64 b = (v.n_req + per_block - 1) / per_block;
        if (b > 2048) b = 2048;
        b /= disco_grid_divisor();
        if (b < 1) b = 1;
        w.nqueue = b >= 2 * TW_QUEUES ? TW_QUEUES : 1;
        b -= b % w.nqueue;                         // every queue is served by the same number of workgroups
        if (before) (void)hipEventRecord(before, stream);
        hipLaunchKernelGGL(k_tl_walk, dim3((unsigned)b), dim3(TW_BLOCK), 0, stream, v, n_tok, w);
        if (after) (void)hipEventRecord(after, stream);
    } else {
        hipLaunchKernelGGL(k_tl_summary_clear, dim3((unsigned)fb), dim3(256), 0, stream, v.n_req, (TlSummary*)summary);
    }
    i64 rb_ = (v.n_req + (i64)TW_WAVES * 64 - 1) / ((i64)TW_WAVES * 64);          // 64 requests per wave and round
    if (rb_ < 1) rb_ = 1;
    if (rb_ > 2048) rb_ = 2048;
    hipLaunchKernelGGL(k_tl_walk_rest, dim3((unsigned)rb_), dim3(TW_BLOCK), 0, stream, v, n_tok, w, mem ? 1 : 0);
}

void disco_launch_tl_stats_fast(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                                MigPartial* totals, hipStream_t stream)
{
    disco_launch_tl_walk(v, n_tok, pol, a.P, a.tau, a.kt, a.wflags, a.summary, a.counter, stream, nullptr, nullptr);
    if (v.n_req > 0) {
        AccumArgs c;
        memset(&c, 0, sizeof(c));
        c.tau = a.tau; c.P = a.P;
        c.G = 1;
        while (c.G < a.P) c.G <<= 1;
        c.summary = (const TlSummary*)a.summary;
        c.totals = totals;
        i64 b = ((v.n_req + 63) / 64 + TA_WAVES - 1) / TA_WAVES;
        if (b > 256) b = 256;
        b /= disco_grid_divisor();
        if (b < 1) b = 1;
        hipLaunchKernelGGL(k_tl_accum, dim3((unsigned)b), dim3(TA_BLOCK), 0, stream, v, pol, c);
    }
    // the pairs with a buffer hand-off, if any; its last workgroup turns the totals into the accumulators
    disco_launch_tl_stats_buf(v, n_tok, pol, a, totals, stream);
    if (v.n_req > 0) {
        if (a.mig_idx || a.n_src_tok || a.t_last || a.delay_num) {
            MatArgs m;
            memset(&m, 0, sizeof(m));
            m.tau = a.tau; m.P = a.P; m.summary = (const TlSummary*)a.summary;
            m.bufsum = (const BufSummary*)a.bufsum; m.buffer_flag = a.buffer_flag;
            m.mig_idx = a.mig_idx; m.n_src_tok = a.n_src_tok; m.t_last = a.t_last; m.delay_num = a.delay_num;
            i64 mb = (v.n_req + 255) / 256;
            if (mb > 4096) mb = 4096;
            hipLaunchKernelGGL(k_tl_mat, dim3((unsigned)mb), dim3(256), 0, stream, v, pol, m);
        }
    }
}
