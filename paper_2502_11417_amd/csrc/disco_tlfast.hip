// Token timelines (Sec. 4.3): the class-mode TBT histogram passes of
// disco_reduce_stats and what prepares them once per selection.
//
//   k_tl_assign  lane = request: timelines that the token walk's summaries
//                prove analytic (running maximum never left 0, so
//                delta_t = round(t tau)) are counted per class and length;
//                the others get their histogram row into the request's
//                descriptor and the request into the walk list
//   k_pp_reduce  per-workgroup count slices -> counts per class and length
//   k_tl_hist    one pass over the walk list: a wave walks one request at a
//                time in chunks of 256 tokens, four consecutive tokens per
//                lane (one 16-byte load per lane and chunk, the next chunk's
//                load issued before the current one is used)
//
// The delivery recurrence delta_t = max(r_t, delta_{t-1} + tau) is evaluated
// in the shifted domain u_t = r_t - t tau, where it is a running maximum M_t
// and delta_t = fma(t, tau, M_t).  `max` is exact and associative, so any
// evaluation order gives the sequential definition bit for bit.  The
// histogram walk needs M_t per token: a 4-element scan in registers and a DPP
// scan across the wave; the gaps delta_t - delta_{t-1} go to the LDS
// histogram of the timeline's class.
//
// Lag trigger (token t is overdue by more than kappa tau): evaluated exactly,
// one IEEE fp32 operation at a time in the order of the definition (slot =
// delta_{t-1} + tau, lag = r_t - slot), in every chunk that passes a cheap necessary
// condition (see walk_hist); the other chunks provably cannot trigger.
//
// A timeline is computed once per request and source, never per policy
// column: the recurrence does not depend on the pair's TTFT, so every column
// only picks the timeline of its dispatch winner.
#include <string.h>

#include "disco_tl_walk.h"

namespace {

constexpr int TH_BLOCK = 1024;               // histogram kernel: 16 waves share 64 KB of bins

struct WalkOut { int m; float M; };          // hand-off index (-1 none), running maximum over all tokens

// Histogram walk of one request and source: the delivery of every token and
// the gap in front of it -> sink(key[4]) once per chunk (tokens without a gap
// carry KEY_SKIP).
//   mem    arrivals from the CSR token array (else t * gap)
//   lag    evaluate the lag trigger (server source of a column with hand-off)
//   first  the lane's elements of the first chunk, if `have_first` (loaded ahead by the caller with load_first)
//
// Necessary condition for the trigger.  With C <= M_{t-1} (C = a running
// maximum taken earlier: u_0 in the first chunk, the carried maximum later)
// and monotone rounding,
//   lag_t = fl(r_t - fl(fl((t-1) tau + M_{t-1}) + tau)) <= fl(r_t - fl(fl((t-1) tau + C) + tau)),
// which differs from u_t - C = fl(r_t - t tau) - C by at most four roundings
// of magnitudes below 2 t tau + 2 |C| + kappa tau.  lag_fast_ok bounds t and
// `cheap` bounds |C| so that this error stays below kappa tau / 4; hence
// lag_t > kappa tau implies u_t > C + kappa tau / 2, and a chunk where no
// token satisfies the latter cannot trigger.
template <class Sink>
__device__ __forceinline__ WalkOut walk_hist(bool mem, int n, const float* __restrict__ arr, i64 off, i64 n_tok, int align,
                                             const float first[4], bool have_first, float gap, bool lag, float g_dev, int l,
                                             float k, float c, float tau, float kt, int lane, Sink&& sink)
{
    const float ninf = -INFINITY;
    const float ntau = -tau;
    const int mis = mem ? (int)((off + align) & 3) : 0;      // the window starts at the 16-byte boundary below the request
    const int lane4 = 4 * lane - mis;                        // token index of this lane's first element in chunk 0
    const i64 gbase = off + lane4;
    const int total = n + mis;
    const bool safe = mem && off - mis >= 0 && off + n + 3 <= n_tok;
    const bool fast_ok = lag_fast_ok(n, tau, kt);
    int m = -1;
    float base = 0.0f;
    float carryM = ninf;           // running maximum over the chunks so far
    float carryD = 0.0f;           // delivery of the last token of the previous chunk
    float nxt[4] = {first[0], first[1], first[2], first[3]};
    if (mem && !have_first && lane4 < n) load4s(arr, gbase, n_tok, safe, nxt);
#pragma unroll 1
    for (int e0 = 0; e0 < total; e0 += 256) {
        const int tk0 = lane4 + e0;
        const float tf0 = (float)tk0;
        const float tf[4] = {tf0, tf0 + 1.0f, tf0 + 2.0f, tf0 + 3.0f};
        float r[4], u[4];
        if (m >= 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = __fmaf_rn((float)(tk0 + q - m + 1), g_dev, base);
        } else if (mem) {
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = nxt[q];
            if (e0 + 256 < total && tk0 + 256 < n) load4s(arr, gbase + e0 + 256, n_tok, safe, nxt);   // next chunk in flight
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = tf[q] * gap;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) u[q] = __fmaf_rn(tf[q], ntau, r[q]);
        const bool full = e0 > 0 && e0 + 256 <= total;      // every element of the chunk is a token of the request
        if (!full) {
#pragma unroll
            for (int q = 0; q < 4; ++q) u[q] = ((unsigned)(tk0 + q) < (unsigned)n) ? u[q] : ninf;
        }
        float i0 = u[0], i1 = fmaxf(i0, u[1]), i2 = fmaxf(i1, u[2]), i3 = fmaxf(i2, u[3]);
        bool exact = false;
        if (lag && m < 0) {
            float C = carryM;
            if (e0 == 0) {                                  // u_0 = r_0: element `mis` of lane 0
                const float r0 = mis == 0 ? r[0] : (mis == 1 ? r[1] : (mis == 2 ? r[2] : r[3]));
                C = bcast_f(r0, 0);
            }
            const bool cheap = fast_ok && fabsf(C) <= 262144.0f * kt;
            exact = !cheap || __ballot(i3 > C + 0.5f * kt) != 0ull;
        }
        float E = fmaxf(wave_prev(wave_incl_max_dpp(i3, lane), ninf), carryM);      // running maximum before this lane's tokens
        if (exact) {
            const float ex[4] = {E, fmaxf(E, i0), fmaxf(E, i1), fmaxf(E, i2)};
            bool trig[4];
            float slot[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                slot[q] = __fmaf_rn(tf[q] - 1.0f, tau, ex[q]) + tau;        // delta_{t-1} + tau
                const float lg = r[q] - slot[q];
                trig[q] = (unsigned)(tk0 + q - 1) < (unsigned)(n - 1) && lg > kt;      // tokens 1 .. n-1
            }
            const u64 any = __ballot(trig[0] || trig[1] || trig[2] || trig[3]);
            if (any) {
                const int ml = __ffsll((long long)any) - 1;
                const int qf = trig[0] ? 0 : (trig[1] ? 1 : (trig[2] ? 2 : 3));
                const float sl = trig[0] ? slot[0] : (trig[1] ? slot[1] : (trig[2] ? slot[2] : slot[3]));
                m = bcast_i(tk0, ml) + bcast_i(qf, ml);
                // hand-off: decided once the token is kappa*tau overdue; the device re-prefills the
                // prompt plus the m tokens already produced, then generates at its own pace
                const float t_dec = bcast_f(sl, ml) + kt;
                const float t_mig = __fmaf_rn((float)(l + m), k, c);
                base = t_dec + t_mig;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (tk0 + q >= m) {
                        r[q] = __fmaf_rn((float)(tk0 + q - m + 1), g_dev, base);
                        u[q] = ((unsigned)(tk0 + q) < (unsigned)n) ? __fmaf_rn(tf[q], ntau, r[q]) : ninf;
                    }
                i0 = u[0]; i1 = fmaxf(i0, u[1]); i2 = fmaxf(i1, u[2]); i3 = fmaxf(i2, u[3]);
                E = fmaxf(wave_prev(wave_incl_max_dpp(i3, lane), ninf), carryM);
            }
        }
        const float M0 = fmaxf(E, i0), M1 = fmaxf(E, i1), M2 = fmaxf(E, i2), M3 = fmaxf(E, i3);
        const float d0 = __fmaf_rn(tf[0], tau, M0), d1 = __fmaf_rn(tf[1], tau, M1);
        const float d2 = __fmaf_rn(tf[2], tau, M2), d3 = __fmaf_rn(tf[3], tau, M3);
        const float p0 = wave_prev(d3, carryD);
        unsigned key[4] = {f2u(d0 - p0), f2u(d1 - d0), f2u(d2 - d1), f2u(d3 - d2)};
        if (!full) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                key[q] = ((unsigned)(tk0 + q - 1) < (unsigned)(n - 1)) ? key[q] : KEY_SKIP;     // tokens 1 .. n-1 have a gap
        }
        sink(key);
        carryM = bcast_f(M3, 63);
        carryD = bcast_f(d3, 63);
    }
    return WalkOut{m, carryM};
}

// The lane's elements of the first chunk of a request's token window (see walk_hist).
__device__ __forceinline__ void load_first(const float* __restrict__ arr, i64 off, int n, i64 n_tok, int align, int lane,
                                           float out[4])
{
    const int mis = (int)((off + align) & 3);
    if (4 * lane - mis < n) load4(arr, off - mis + 4 * lane, n_tok, out);
}

// ------------------------------------------------------------- histogram ---

// What every histogram pass needs to know of a request, worked out once per selection (k_tl_assign): the LDS
// row of each of its timelines (device source, server source, server source with the lag trigger, the two buffer
// hand-off kinds; one byte each in the order of the TL_ kinds, 0xFF = nothing to walk: no such timeline, or one
// that is histogrammed analytically).  The kernel below walks the first three kinds.
constexpr u64 DESC_NONE5 = 0xFFFFFFFFFFull;
constexpr unsigned DESC_NONE = 0xFFFFFFu;

// Analytic timelines per class and length, counted per workgroup in LDS (two 16-bit counts per word, a workgroup
// sees at most 65535 requests) for the first PP_LDS_CLS classes and stored as one slice per workgroup; classes
// beyond that (tables of many columns) are counted in device memory directly.
constexpr int PP_LDS_CLS = 16;
constexpr int PP_WORDS = DISCO_PP_NMAX / 2 + 1;              // words per class: lengths 0 .. DISCO_PP_NMAX
constexpr int AS_BLOCK = 1024;

__global__ __launch_bounds__(AS_BLOCK) void k_tl_assign(TraceView tr, const disco_policy* __restrict__ pol, int P,
                                                        const TlSummary* __restrict__ summary,
                                                        const BufSummary* __restrict__ bufsum, SelState* S,
                                                        u64* __restrict__ desc_out, unsigned* __restrict__ list,
                                                        unsigned* __restrict__ slices, unsigned* __restrict__ ppcnt,
                                                        unsigned* __restrict__ dhist, int use_lds)
{
    __shared__ unsigned cnt[PP_LDS_CLS * PP_WORDS];          // 128 KB
    __shared__ unsigned s_nw[2], s_base[2];                  // [0] long requests (front of the list), [1] the others (back)
    __shared__ u64 s_cls[DISCO_MAX_CLS];
    __shared__ signed char s_slot[DISCO_MAX_CLS];
    __shared__ disco_policy spol[DISCO_MAX_COLS];
    const TlSel* tl = &S->tl;
    if (tl->fallback) return;                                // per-slot histograms: the general kernel walks everything
    const int ncls = tl->ncls;
    const int nlds = use_lds ? (ncls < PP_LDS_CLS ? ncls : PP_LDS_CLS) : 0;
    if ((int)threadIdx.x < P) spol[threadIdx.x] = pol[threadIdx.x];
    if (threadIdx.x < DISCO_MAX_CLS) { s_cls[threadIdx.x] = tl->cls_mask[threadIdx.x]; s_slot[threadIdx.x] = tl->cls_slot[threadIdx.x]; }
    for (int i = threadIdx.x; i < nlds * PP_WORDS; i += AS_BLOCK) cnt[i] = 0u;
    if (threadIdx.x < 2) s_nw[threadIdx.x] = 0u;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    // a contiguous share of the requests per workgroup (at most 65535, see the launch)
    const i64 per = (tr.n_req + gridDim.x - 1) / gridDim.x;
    const i64 lo = (i64)blockIdx.x * per;
    const i64 hi = lo + per < tr.n_req ? lo + per : tr.n_req;
    u64 wmask = 0ull, lmask = 0ull;                          // bit r: this thread's request of round r has tokens to walk / is long
    int round = 0;
    for (i64 i = lo + threadIdx.x; i < hi; i += AS_BLOCK, ++round) {
        const int l = tr.l[i], n = tr.n[i];
        const float s = tr.s[i];
        const float k = tr.k ? tr.k[i] : tr.k_s;
        const TlSummary sm = summary[i];
        u64 m[TL_KINDS];
        request_sets(spol, P, l, s, __fmaf_rn((float)l, k, tr.c), i, m);
        u64 desc = DESC_NONE5;
        BufSummary bs{0.0f, -1, 0, 0, 0.0f, -1, 0, 0};
        if ((m[TL_SRV_BUF] | m[TL_DEV_BUF]) != 0ull) {
            bs = bufsum[i];
            // migrated requests by number of delayed tokens, per column (those without one are implied by the
            // migration count)
#pragma unroll
            for (int kind = TL_SRV_BUF; kind <= TL_DEV_BUF; ++kind) {
                const int me = kind == TL_SRV_BUF ? bs.m_s : bs.m_d;
                const int dl = kind == TL_SRV_BUF ? bs.delay_s : bs.delay_d;
                if (m[kind] == 0ull || summary_m(me) < 0 || dl <= 0) continue;
                const int bin = dl < DISCO_DELAY_BINS - 1 ? dl : DISCO_DELAY_BINS - 1;
                for (u64 left = m[kind]; left != 0ull; left &= left - 1ull)
                    atomicAdd(&dhist[(size_t)(__ffsll((long long)left) - 1) * DISCO_DELAY_BINS + bin], 1u);
            }
        }
#pragma unroll
        for (int kind = 0; kind < TL_KINDS; ++kind) {
            if (m[kind] == 0ull) continue;
            const int c = cls_find(s_cls, ncls, m[kind]);
            if (c < 0) { S->tl.error = 1; continue; }        // a set the classification did not see: never expected
            if (kind < TL_SRV_BUF ? timeline_is_analytic(kind, n, sm) : buf_timeline_is_analytic(kind, n, bs)) {
                if (c < nlds) atomicAdd(&cnt[c * PP_WORDS + (n >> 1)], 1u << (16 * (n & 1)));
                else atomicAdd(&ppcnt[(size_t)c * (DISCO_PP_NMAX + 1) + n], 1u);
            } else {
                const int sl = s_slot[c];
                if (sl < 0) { S->tl.error = 1; continue; }
                desc = (desc & ~(0xFFull << (8 * kind))) | ((u64)(unsigned)sl << (8 * kind));
            }
        }
        desc_out[i] = desc;
        const bool walk = desc != DESC_NONE5, lng = n >= WALK_LONG_TOKENS;
        if (walk) wmask |= 1ull << round;
        if (walk && lng) lmask |= 1ull << round;
        const u64 wb = __ballot(walk);
        if (wb) {
            const u64 lb = __ballot(walk && lng);
            if (lane == __ffsll((long long)wb) - 1) {
                if (lb) atomicAdd(&s_nw[0], (unsigned)__popcll(lb));
                if (wb & ~lb) atomicAdd(&s_nw[1], (unsigned)__popcll(wb & ~lb));
            }
        }
    }
    __syncthreads();
    // the requests with tokens to walk go to a device-wide list (any order: the histograms are sums), a range of it
    // per workgroup
    const unsigned nw0 = s_nw[0], nw1 = s_nw[1];
    __syncthreads();
    if (threadIdx.x == 0) {
        s_base[0] = nw0 ? atomicAdd(&S->tl.nlist, nw0) : 0u;
        s_base[1] = nw1 ? atomicAdd(&S->tl.nlist_back, nw1) : 0u;
        s_nw[0] = 0u; s_nw[1] = 0u;
    }
    __syncthreads();
    if (nw0 | nw1) {
        round = 0;
        for (i64 i = lo + threadIdx.x; i < hi; i += AS_BLOCK, ++round) {
            const bool w = (wmask >> round) & 1ull, lng = (lmask >> round) & 1ull;
            const u64 wb = __ballot(w);
            if (!wb) continue;
            const u64 lb = __ballot(w && lng), sb = wb & ~lb;
            const int leader = __ffsll((long long)wb) - 1;
            unsigned at0 = 0u, at1 = 0u;
            if (lane == leader) {
                if (lb) at0 = atomicAdd(&s_nw[0], (unsigned)__popcll(lb));
                if (sb) at1 = atomicAdd(&s_nw[1], (unsigned)__popcll(sb));
            }
            at0 = (unsigned)bcast_i((int)at0, leader);
            at1 = (unsigned)bcast_i((int)at1, leader);
            const u64 below = (1ull << lane) - 1ull;
            if (w && lng) list[s_base[0] + at0 + (unsigned)__popcll(lb & below)] = (unsigned)i;
            if (w && !lng) list[(size_t)tr.n_req - 1 - (s_base[1] + at1 + (unsigned)__popcll(sb & below))] = (unsigned)i;
        }
    }
    unsigned* mine = slices + (size_t)blockIdx.x * PP_LDS_CLS * PP_WORDS;
    for (int i = threadIdx.x; i < nlds * PP_WORDS; i += AS_BLOCK) mine[i] = cnt[i];
}

// ppcnt[c][n] += sum over the workgroup slices.  Workgroup = (class, 256 words of two lengths each); four groups
// of threads share the slices and meet in LDS.
__global__ __launch_bounds__(1024) void k_pp_reduce(const SelState* S, int nslices, const unsigned* __restrict__ slices,
                                                    unsigned* __restrict__ ppcnt, int use_lds)
{
    __shared__ unsigned part[2][1024];
    const TlSel* tl = &S->tl;
    const int c = blockIdx.x;
    if (tl->fallback || !use_lds || c >= tl->ncls || c >= PP_LDS_CLS) return;
    const int w = blockIdx.y * 256 + (threadIdx.x & 255), grp = threadIdx.x >> 8;
    unsigned even = 0u, odd = 0u;
    if (w < PP_WORDS) {
#pragma unroll 8
        for (int b = grp; b < nslices; b += 4) {
            const unsigned v = slices[((size_t)b * PP_LDS_CLS + c) * PP_WORDS + w];
            even += v & 0xFFFFu; odd += v >> 16;
        }
    }
    part[0][threadIdx.x] = even; part[1][threadIdx.x] = odd;
    __syncthreads();
    if (grp == 0 && w < PP_WORDS) {
        for (int g = 1; g < 4; ++g) { even += part[0][threadIdx.x + 256 * g]; odd += part[1][threadIdx.x + 256 * g]; }
        unsigned* row = ppcnt + (size_t)c * (DISCO_PP_NMAX + 1);
        if (even) row[2 * w] += even;
        if (odd && 2 * w + 1 <= DISCO_PP_NMAX) row[2 * w + 1] += odd;
    }
}

// One histogram pass of the class-mode TBT selection: the descriptors say which timelines have tokens to walk
// (few: the others were counted analytically once) and the walk list names their requests.
__global__ __launch_bounds__(TH_BLOCK, 8) void k_tl_hist(TraceView tr, i64 n_tok, int align, HistArgs a)
{
    __shared__ __align__(16) unsigned smem[DISCO_TL_HIST_WORDS];
    const TlSel* tl = &a.S->tl;
    const int width = tl->width;
    if (width <= 0 || tl->fallback) return;       // selection finished, or per-slot histograms (other kernel)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ncls = tl->ncls, nwalk = tl->nwalk;
    HistCtx h;
    h.hist = smem; h.width = width; h.shift = tl->shift; h.up = h.shift + width;
    h.G = tl->G < DISCO_MAX_GRP ? tl->G : DISCO_MAX_GRP;
    h.stride = (unsigned)nwalk << width;
    h.key_lo = tl->key_lo; h.key_cap = tl->window ? (1u << tl->window) : 0xFFFFFFFFu;
    for (int k = 0; k < DISCO_MAX_GRP; ++k) h.grp_prefix[k] = tl->grp_prefix[k];
    const int words = (h.G * nwalk) << width;
    for (int i = threadIdx.x; i < words; i += TH_BLOCK) smem[i] = 0u;
    __syncthreads();
    const float tau = a.tau, kt = a.kt;
    const bool mem = tr.arr != nullptr;
    // the walk list is shared out in batches of rb entries (lane = entry) so that every wave gets some
    const i64 nwaves = (i64)gridDim.x * (TH_BLOCK / 64);
    const i64 nfront = (i64)tl->nlist, nlist = nfront + (i64)tl->nlist_back;
    i64 rb = (nlist + nwaves - 1) / nwaves;
    rb = rb < 1 ? 1 : (rb > 64 ? 64 : rb);
    // wave w of a round takes the entries w, w + W, ... (lane = which of them), W = waves x rounds needed
    const i64 nround = (nlist + rb * nwaves - 1) / (rb * nwaves);
    for (i64 rnd = 0; rnd < nround; ++rnd) {
        const i64 gw = (i64)blockIdx.x * (TH_BLOCK / 64) + wave;
        const i64 j = rnd * rb * nwaves + gw + (i64)lane * nwaves;
        const bool mine = lane < rb && j < nlist;
        const i64 i = mine ? (i64)walk_list_entry(a.list, tr.n_req, nfront, j) : 0;
        const unsigned desc = mine ? (unsigned)(a.desc[i] & 0xFFFFFFull) : DESC_NONE;
        u64 walkers = __ballot(desc != DESC_NONE);
        if (!walkers) continue;
        // the fields of the requests that are walked
        int l_v = 0, n_v = 1;
        float k_v = tr.k_s, gd_v = tr.g_s, gap_v = 0.0f;
        i64 off_v = 0;
        if (desc != DESC_NONE) {
            l_v = tr.l[i]; n_v = tr.n[i];
            if (tr.k) k_v = tr.k[i];
            if (tr.g) gd_v = tr.g[i];
            if (tr.off) off_v = tr.off[i];
            if (tr.tbt) gap_v = tr.tbt[i];
        }
        const u64 memw = mem ? __ballot((desc & 0xFFFF00u) != 0xFFFF00u) : 0ull;     // requests that read the token array
        float pre[4] = {0.f, 0.f, 0.f, 0.f};
        {
            const int r0 = __ffsll((long long)walkers) - 1;
            if ((memw >> r0) & 1ull) load_first(tr.arr, (i64)bcast_u64((u64)off_v, r0), bcast_i(n_v, r0), n_tok, align, lane, pre);
        }
        while (walkers) {
            const int rq = __ffsll((long long)walkers) - 1;
            walkers &= walkers - 1;
            const unsigned dsc = (unsigned)bcast_i((int)desc, rq);
            const int n = bcast_i(n_v, rq), l = bcast_i(l_v, rq);
            const float gd = bcast_f(gd_v, rq);
            const float cur[4] = {pre[0], pre[1], pre[2], pre[3]};
            bool have = (memw >> rq) & 1ull;
            if (walkers) {                          // the next request's first chunk is loaded while this one is walked
                const int r1 = __ffsll((long long)walkers) - 1;
                if ((memw >> r1) & 1ull)
                    load_first(tr.arr, (i64)bcast_u64((u64)off_v, r1), bcast_i(n_v, r1), n_tok, align, lane, pre);
            }
#pragma unroll 1
            for (int variant = 2; variant >= 0; --variant) {
                const unsigned sl = (dsc >> (8 * variant)) & 0xFFu;
                if (sl == 0xFFu) continue;
                const unsigned row_base = sl << width;
                auto sink = [&](const unsigned key[4]) { hist_keys(h, key, row_base, lane); };
                const bool dev = variant == 0;
                const float gap = dev ? gd : bcast_f(gap_v, rq);
                const bool from_mem = !dev && mem;
                const i64 off = from_mem ? (i64)bcast_u64((u64)off_v, rq) : 0;
                walk_hist(from_mem, n, tr.arr, off, n_tok, align, cur, from_mem && have, gap, variant == 2, gd, l,
                          bcast_f(k_v, rq), tr.c, tau, kt, lane, sink);
                if (from_mem) have = false;
            }
        }
    }
    __syncthreads();
    // LDS rows (group, walked class) -> device-wide rows (group, class)
    const unsigned dmask = (1u << width) - 1u;
    for (int i = threadIdx.x; i < words; i += TH_BLOCK) {
        const unsigned cnt = smem[i];
        if (!cnt) continue;
        const int row = i >> width;
        const int g = row / nwalk, sl = row - g * nwalk;
        const int c = tl->slot_cls[sl];
        atomicAdd(&a.ghist[((size_t)(g * ncls + c) << width) | ((unsigned)i & dmask)], cnt);
    }
}

}  // namespace

// Once per selection, after the classification: descriptors of all requests, analytic timelines counted per class
// and length.  `slices`: scratch for the workgroup slices (slices_bytes).
void disco_launch_tl_assign(const TraceView& v, const disco_policy* pol, int P, const void* summary, SelState* S,
                            const void* bufsum, u64* desc, unsigned* list, unsigned* slices, size_t slices_bytes,
                            unsigned* ppcnt, unsigned* dhist, hipStream_t stream)
{
    if (v.n_req <= 0) return;
    i64 b = (v.n_req + 49151) / 49152;             // at most 65535 requests per workgroup: 16-bit counts in LDS
    if (b < 250) b = 250;                          // one workgroup per CU (128 KB of LDS each); at most 64 rounds per thread
    const i64 fit = (i64)(slices_bytes / ((size_t)PP_LDS_CLS * PP_WORDS * sizeof(unsigned)));
    int use_lds = 1;
    // tens of millions of requests (or the testing aid that shrinks the grids): counts in device memory
    if (b > fit || disco_grid_divisor() > 1) { b = (v.n_req + 65535) / 65536; use_lds = 0; }
    hipLaunchKernelGGL(k_tl_assign, dim3((unsigned)b), dim3(AS_BLOCK), 0, stream, v, pol, P, (const TlSummary*)summary,
                       (const BufSummary*)bufsum, S, desc, list, slices, ppcnt, dhist, use_lds);
    hipLaunchKernelGGL(k_pp_reduce, dim3(PP_LDS_CLS, (PP_WORDS + 255) / 256), dim3(1024), 0, stream, (const SelState*)S, (int)b, (const unsigned*)slices,
                       ppcnt, use_lds);
}

void disco_launch_tl_hist_fast(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                               hipStream_t stream)
{
    (void)pol;
    HistArgs h;
    memset(&h, 0, sizeof(h));
    h.tau = a.tau; h.kt = a.kt; h.P = a.P; h.pass = a.pass;
    h.S = a.S; h.ghist = a.ghist;
    h.desc = a.desc; h.list = a.list;
    i64 b = (v.n_req + TH_BLOCK / 64 - 1) / (TH_BLOCK / 64);      // at most one request per wave
    if (b < 1) b = 1;
    // two resident workgroups per CU; the passes after the second normally have nothing to do (the launch returns
    // at once) and get a small grid, which makes the empty launch cheaper and a needed one merely slower
    const i64 cap = a.pass < 2 ? 512 : 64;
    if (b > cap) b = cap;
    b /= disco_grid_divisor();
    if (b < 1) b = 1;
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_tl_hist, dim3((unsigned)b), dim3(TH_BLOCK), 0, stream, v, n_tok, align, h);
}
