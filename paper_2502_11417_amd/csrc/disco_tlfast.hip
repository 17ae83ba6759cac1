// Token timelines (Sec. 4.3), streaming kernels: the statistics pass of
// disco_eval_migration and the class-mode TBT histogram passes of
// disco_reduce_stats.
//
// One wave walks one request at a time in chunks of 256 tokens, four
// consecutive tokens per lane (one 16-byte load per lane and chunk, the next
// chunk's load issued before the current one is used).  The delivery
// recurrence delta_t = max(r_t, delta_{t-1} + tau) is evaluated in the shifted
// domain u_t = r_t - t tau, where it is a running maximum M_t and
// delta_t = fma(t, tau, M_t).  `max` is exact and associative, so any
// evaluation order gives the sequential definition bit for bit.
//
//   statistics pass: only the last delivery fma(n-1, tau, M_{n-1}) and the
//     hand-off index are needed, so a chunk costs one fma and one max per
//     token and the wave reduces its lanes once per request.
//   histogram pass: M_t per token by a 4-element scan in registers and a DPP
//     scan across the wave; the gaps delta_t - delta_{t-1} go to the LDS
//     histogram of the timeline's class.
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

__global__ __launch_bounds__(TH_BLOCK, 8) void k_tl_hist(TraceView tr, i64 n_tok, int align, const disco_policy* __restrict__ pol,
                                                      HistArgs a)
{
    __shared__ __align__(16) unsigned smem[DISCO_TL_HIST_WORDS];
    __shared__ u64 s_cls[DISCO_MAX_CLS];
    __shared__ signed char s_slot[DISCO_MAX_CLS];
    __shared__ disco_policy spol[DISCO_MAX_COLS];
    const TlSel* tl = &a.S->tl;
    const int width = tl->width;
    if (width <= 0 || tl->fallback) return;       // selection finished, or per-slot histograms (other kernel)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int P = a.P, ncls = tl->ncls, nwalk = tl->nwalk;
    HistCtx h;
    h.hist = smem; h.width = width; h.shift = tl->shift; h.up = h.shift + width;
    h.G = tl->G < DISCO_MAX_GRP ? tl->G : DISCO_MAX_GRP;
    h.stride = (unsigned)nwalk << width;
    h.key_lo = tl->key_lo; h.key_cap = tl->window ? (1u << tl->window) : 0xFFFFFFFFu;
    for (int k = 0; k < DISCO_MAX_GRP; ++k) h.grp_prefix[k] = tl->grp_prefix[k];
    if ((int)threadIdx.x < P) spol[threadIdx.x] = pol[threadIdx.x];
    if (threadIdx.x < DISCO_MAX_CLS) { s_cls[threadIdx.x] = tl->cls_mask[threadIdx.x]; s_slot[threadIdx.x] = tl->cls_slot[threadIdx.x]; }
    const int words = (h.G * nwalk) << width;
    for (int i = threadIdx.x; i < words; i += TH_BLOCK) smem[i] = 0u;
    __syncthreads();
    const float tau = a.tau, kt = a.kt;
    const bool mem = tr.arr != nullptr;
    const bool count_pp = a.pass == 0;
    const i64 nwaves = (i64)gridDim.x * (TH_BLOCK / 64);
    const int rb = a.rb;
    const i64 nbatch = (tr.n_req + rb - 1) / rb;
    for (i64 bt = (i64)blockIdx.x * (TH_BLOCK / 64) + wave; bt < nbatch; bt += nwaves) {
        const Batch b = load_batch(tr, spol, P, bt * rb, lane, rb, a.summary);
        // lane = request: LDS row of each of the three timelines, 0xFF = nothing to walk
        unsigned desc = 0xFFFFFFu;
        {
#pragma unroll
            for (int kind = 0; kind < 3; ++kind) {
                if (b.m[kind] == 0ull) continue;
                const int c = cls_find(s_cls, ncls, b.m[kind]);
                const bool analytic = timeline_is_analytic(kind, b.n, b.sum);
                if (c < 0) { a.S->tl.error = 1; continue; }        // a set the classification did not see: never expected
                if (analytic) {
                    if (count_pp) atomicAdd(&a.ppcnt[(size_t)c * (DISCO_PP_NMAX + 1) + b.n], 1u);
                } else {
                    const int sl = s_slot[c];
                    if (sl < 0) { a.S->tl.error = 1; continue; }
                    desc = (desc & ~(0xFFu << (8 * kind))) | ((unsigned)sl << (8 * kind));
                }
            }
        }
        u64 walkers = __ballot(desc != 0xFFFFFFu);
        const u64 memw = mem ? __ballot((desc & 0xFFFF00u) != 0xFFFF00u) : 0ull;     // requests that read the token array
        float pre[4] = {0.f, 0.f, 0.f, 0.f};
        if (walkers) {
            const int r0 = __ffsll((long long)walkers) - 1;
            if ((memw >> r0) & 1ull) load_first(tr.arr, (i64)bcast_u64((u64)b.off, r0), bcast_i(b.n, r0), n_tok, align, lane, pre);
        }
        while (walkers) {
            const int rq = __ffsll((long long)walkers) - 1;
            walkers &= walkers - 1;
            const unsigned dsc = (unsigned)bcast_i((int)desc, rq);
            const int n = bcast_i(b.n, rq), l = bcast_i(b.l, rq);
            const float gd = bcast_f(b.gd, rq);
            const float cur[4] = {pre[0], pre[1], pre[2], pre[3]};
            bool have = (memw >> rq) & 1ull;
            if (walkers) {                          // the next request's first chunk is loaded while this one is walked
                const int r1 = __ffsll((long long)walkers) - 1;
                if ((memw >> r1) & 1ull)
                    load_first(tr.arr, (i64)bcast_u64((u64)b.off, r1), bcast_i(b.n, r1), n_tok, align, lane, pre);
            }
#pragma unroll 1
            for (int variant = 2; variant >= 0; --variant) {
                const unsigned sl = (dsc >> (8 * variant)) & 0xFFu;
                if (sl == 0xFFu) continue;
                const unsigned row_base = sl << width;
                auto sink = [&](const unsigned key[4]) { hist_keys(h, key, row_base, lane); };
                const bool dev = variant == 0;
                const float gap = dev ? gd : bcast_f(b.gap, rq);
                const bool from_mem = !dev && mem;
                const i64 off = from_mem ? (i64)bcast_u64((u64)b.off, rq) : 0;
                walk_hist(from_mem, n, tr.arr, off, n_tok, align, cur, from_mem && have, gap, variant == 2, gd, l,
                          bcast_f(b.k, rq), tr.c, tau, kt, lane, sink);
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

void disco_launch_tl_hist_fast(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                               hipStream_t stream)
{
    HistArgs h;
    memset(&h, 0, sizeof(h));
    h.tau = a.tau; h.kt = a.kt; h.P = a.P; h.pass = a.pass;
    h.S = a.S; h.ghist = a.ghist; h.ppcnt = a.ppcnt;
    h.summary = (const TlSummary*)a.summary;
    h.rb = tl_batch(v.n_req, 512 * (TH_BLOCK / 64));
    const i64 per_block = (i64)(TH_BLOCK / 64) * h.rb;
    i64 b = (v.n_req + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > 512) b = 512;                      // two resident workgroups per CU
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_tl_hist, dim3((unsigned)b), dim3(TH_BLOCK), 0, stream, v, n_tok, align, pol, h);
}
