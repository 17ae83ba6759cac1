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
// with the oracle's operations, in the first chunk of a request and in every
// later chunk that passes a cheap necessary condition (see `walk`).
//
// A timeline is computed once per request and source, never per policy
// column: the recurrence does not depend on the pair's TTFT, so every column
// only picks the timeline of its dispatch winner.
#include <string.h>

#include "disco_tl_device.h"

namespace {

constexpr int TF_RB = 16;                    // requests per wave batch
constexpr int TS_BLOCK = 256;                // statistics kernel: 4 waves, no histogram
constexpr int TH_BLOCK = 1024;               // histogram kernel: 16 waves share 64 KB of bins
constexpr unsigned KEY_SKIP = 0x80000000u;   // a key with the sign bit never matches a prefix

struct WalkOut { int m; float M; };          // hand-off index (-1 none), running maximum over all tokens

// Walks the timeline of one request and source.
//   mem    arrivals from the CSR token array (else t * gap)
//   lag    evaluate the lag trigger (server source of a column with hand-off)
//   HIST   per-token deliveries and gap keys -> sink(key[4]), invalid tokens flagged KEY_SKIP
//
// Necessary condition for the trigger in chunks after the first.  With
// C <= M_{t-1} (C = a running maximum taken earlier) and monotone rounding,
//   lag_t = fl(r_t - fl(fl((t-1) tau + M_{t-1}) + tau)) <= fl(r_t - fl(fl((t-1) tau + C) + tau)),
// which differs from u_t - C = fl(r_t - t tau) - C by at most four roundings
// of magnitudes below 2 t tau + 2 |C| + kappa tau.  `fast_ok` bounds t and
// `c_ok` bounds |C| so that this error stays below kappa tau / 4; hence
// lag_t > kappa tau implies u_t > C + kappa tau / 2, and a chunk where no
// token satisfies the latter cannot trigger.
//   first  the lane's elements of the first chunk, if `have_first` (loaded ahead by the caller with load_first)
template <bool HIST, class Sink>
__device__ __forceinline__ WalkOut walk(bool mem, int n, const float* __restrict__ arr, i64 off, i64 n_tok, int align,
                                        const float first[4], bool have_first, float gap, bool lag, float g_dev, int l, float k, float c, float tau, float kt, bool fast_ok,
                                        int lane, Sink&& sink)
{
    const float ninf = -INFINITY;
    const float ntau = -tau;
    const int mis = mem ? (int)((off + align) & 3) : 0;      // the window starts at the 16-byte boundary below the request
    const i64 gbase = off - mis + 4 * lane;
    const int total = n + mis;
    int m = -1;
    float base = 0.0f;
    float Mlane = ninf;            // !HIST: per-lane maximum of u over the chunks so far
    float carryM = ninf;           // HIST: maximum over the chunks so far; !HIST: maximum of the first chunk
    float carryD = 0.0f;           // HIST: delivery of the last token of the previous chunk
    float nxt[4] = {first[0], first[1], first[2], first[3]};
    if (mem && !have_first && 4 * lane - mis < n) load4(arr, gbase, n_tok, nxt);
#pragma unroll 1
    for (int e0 = 0; e0 < total; e0 += 256) {
        const int tk0 = e0 + 4 * lane - mis;                 // token index of this lane's first element
        float r[4], tf[4], u[4];
        bool val[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            tf[q] = (float)(tk0 + q);
            val[q] = (unsigned)(tk0 + q) < (unsigned)n;
        }
        if (m >= 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = __fmaf_rn((float)(tk0 + q - m + 1), g_dev, base);
        } else if (mem) {
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = nxt[q];
            if (e0 + 256 < total && tk0 + 256 < n) load4(arr, gbase + e0 + 256, n_tok, nxt);   // next chunk in flight
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = tf[q] * gap;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) u[q] = val[q] ? __fmaf_rn(tf[q], ntau, r[q]) : ninf;
        float i0 = u[0], i1 = fmaxf(i0, u[1]), i2 = fmaxf(i1, u[2]), i3 = fmaxf(i2, u[3]);
        bool exact = false;
        if (lag && m < 0) {
            const bool c_ok = fabsf(carryM) <= 262144.0f * kt;
            exact = e0 == 0 || !fast_ok || !c_ok || __ballot(i3 > carryM + 0.5f * kt) != 0ull;
        }
        float E = ninf;            // running maximum over every token before this lane's first
        if (HIST || exact) {
            const float before = HIST ? carryM : wave_max_f32(Mlane);
            const float incl = wave_incl_max_dpp(i3, lane);
            E = fmaxf(wave_prev(incl, ninf), before);
        }
        if (exact) {
            const float ex[4] = {E, fmaxf(E, i0), fmaxf(E, i1), fmaxf(E, i2)};
            bool trig[4];
            float slot[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                slot[q] = __fmaf_rn(tf[q] - 1.0f, tau, ex[q]) + tau;        // delta_{t-1} + tau
                const float lg = r[q] - slot[q];
                trig[q] = val[q] && tk0 + q >= 1 && lg > kt;
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
                        u[q] = val[q] ? __fmaf_rn(tf[q], ntau, r[q]) : ninf;
                    }
                i0 = u[0]; i1 = fmaxf(i0, u[1]); i2 = fmaxf(i1, u[2]); i3 = fmaxf(i2, u[3]);
                if (HIST) {
                    const float incl = wave_incl_max_dpp(i3, lane);
                    E = fmaxf(wave_prev(incl, ninf), carryM);
                }
            }
        }
        if (HIST) {
            const float M0 = fmaxf(E, i0), M1 = fmaxf(E, i1), M2 = fmaxf(E, i2), M3 = fmaxf(E, i3);
            const float d0 = __fmaf_rn(tf[0], tau, M0), d1 = __fmaf_rn(tf[1], tau, M1);
            const float d2 = __fmaf_rn(tf[2], tau, M2), d3 = __fmaf_rn(tf[3], tau, M3);
            const float p0 = wave_prev(d3, carryD);
            unsigned key[4] = {f2u(d0 - p0), f2u(d1 - d0), f2u(d2 - d1), f2u(d3 - d2)};
#pragma unroll
            for (int q = 0; q < 4; ++q)
                key[q] = ((unsigned)(tk0 + q - 1) < (unsigned)(n - 1)) ? key[q] : KEY_SKIP;     // tokens 1 .. n-1 have a gap
            sink(key);
            carryM = bcast_f(M3, 63);
            carryD = bcast_f(d3, 63);
        } else {
            Mlane = fmaxf(Mlane, i3);
            if (lag && e0 == 0) carryM = wave_max_f32(i3);
        }
    }
    return WalkOut{m, HIST ? carryM : wave_max_f32(Mlane)};
}

// The lane's elements of the first chunk of a request's token window (see walk).
__device__ __forceinline__ void load_first(const float* __restrict__ arr, i64 off, int n, i64 n_tok, int align, int lane,
                                           float out[4])
{
    const int mis = (int)((off + align) & 3);
    if (4 * lane - mis < n) load4(arr, off - mis + 4 * lane, n_tok, out);
}

// Per-request fields of a wave batch, lane = request (lanes >= TF_RB idle).
struct Batch {
    int l, n;
    float k, gd, gap;
    i64 off;
    u64 m[3];
};

__device__ __forceinline__ Batch load_batch(const TraceView& tr, const disco_policy* spol, int P, i64 first, int lane)
{
    Batch b;
    const i64 i = first + lane;
    const bool v = lane < TF_RB && i < tr.n_req;
    b.l = 0; b.n = 1; b.k = tr.k_s; b.gd = tr.g_s; b.gap = 0.0f; b.off = 0;
    float s = 0.0f;
    if (v) {
        b.l = tr.l[i]; b.n = tr.n[i]; s = tr.s[i];
        if (tr.k) b.k = tr.k[i];
        if (tr.g) b.gd = tr.g[i];
        if (tr.off) b.off = tr.off[i];
        if (tr.tbt) b.gap = tr.tbt[i];
    }
    request_sets(spol, P, b.l, s, __fmaf_rn((float)b.l, b.k, tr.c), b.m);
    if (!v) b.m[0] = b.m[1] = b.m[2] = 0ull;
    return b;
}

// Can chunks after the first use the necessary condition of the lag trigger?
__device__ __forceinline__ bool lag_fast_ok(int n, float tau, float kt)
{
    return (float)n + 2.0f <= 262144.0f * (kt / tau) && kt >= tau * 0.0009765625f;
}

// ------------------------------------------------------------ statistics ---

struct StatsArgs {
    float tau, kt;
    int P;
    int32_t* mig_idx; int32_t* n_src_tok; float* t_last;
    MigPartial* totals;            // DISCO_NCOPY x 64 device-wide totals
};

__global__ __launch_bounds__(TS_BLOCK) void k_tl_stats(TraceView tr, i64 n_tok, int align, const disco_policy* __restrict__ pol,
                                                       StatsArgs a)
{
    __shared__ disco_policy spol[DISCO_MAX_COLS];
    __shared__ u64 sh[6 * TS_BLOCK];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int P = a.P;
    if ((int)threadIdx.x < P) spol[threadIdx.x] = pol[threadIdx.x];
    __syncthreads();
    // lane = column: tokens decoded by the server, re-prefilled tokens, hand-offs, sum of last deliveries;
    // the number of tokens and of gaps is the same for every column (wave-uniform)
    u64 acc_s_dec = 0, acc_repre = 0, tot_n = 0, tot_cnt = 0;
    unsigned acc_mig = 0;
    double acc_tlast = 0.0;
    const float tau = a.tau, kt = a.kt;
    const bool mem = tr.arr != nullptr;
    auto nosink = [](const unsigned*) {};
    const i64 nwaves = (i64)gridDim.x * (TS_BLOCK / 64);
    const i64 nbatch = (tr.n_req + TF_RB - 1) / TF_RB;
    for (i64 bt = (i64)blockIdx.x * (TS_BLOCK / 64) + wave; bt < nbatch; bt += nwaves) {
        const Batch b = load_batch(tr, spol, P, bt * TF_RB, lane);
        const int cnt = (int)((tr.n_req - bt * TF_RB < TF_RB) ? (tr.n_req - bt * TF_RB) : TF_RB);
        const u64 memw = mem ? __ballot((b.m[1] | b.m[2]) != 0ull) : 0ull;     // requests that read the token array
        float pre[4] = {0.f, 0.f, 0.f, 0.f};
        if (memw & 1ull) load_first(tr.arr, (i64)bcast_u64((u64)b.off, 0), bcast_i(b.n, 0), n_tok, align, lane, pre);
#pragma unroll 1
        for (int rq = 0; rq < cnt; ++rq) {
            const i64 i = bt * TF_RB + rq;
            const int n = bcast_i(b.n, rq), l = bcast_i(b.l, rq);
            const float gd = bcast_f(b.gd, rq);
            const u64 mask_dev = bcast_u64(b.m[0], rq), mask_plain = bcast_u64(b.m[1], rq), mask_lag = bcast_u64(b.m[2], rq);
            const float cur[4] = {pre[0], pre[1], pre[2], pre[3]};
            bool have = (memw >> rq) & 1ull;
            if ((memw >> (rq + 1)) & 1ull)          // the next request's first chunk is loaded while this one is walked
                load_first(tr.arr, (i64)bcast_u64((u64)b.off, rq + 1), bcast_i(b.n, rq + 1), n_tok, align, lane, pre);
            tot_n += (u64)n;
            tot_cnt += (u64)(n - 1);
            WalkOut res_lag{-1, 0.0f};
            bool lag_done = false;
            // order lag, plain, device; a lag run that never fired is also the plain result
#pragma unroll 1
            for (int variant = 2; variant >= 0; --variant) {
                const u64 mask = variant == 2 ? mask_lag : (variant == 1 ? mask_plain : mask_dev);
                if (!mask) continue;
                WalkOut res;
                const bool dev = variant == 0;
                const float gap = dev ? gd : bcast_f(b.gap, rq);
                const bool from_mem = !dev && mem;
                if (variant == 1 && lag_done && res_lag.m < 0) {
                    res = res_lag;
                } else if (!from_mem && pure_pacing(true, gap, tau)) {
                    res = WalkOut{-1, 0.0f};
                } else {
                    const i64 off = from_mem ? (i64)bcast_u64((u64)b.off, rq) : 0;
                    res = walk<false>(from_mem, n, tr.arr, off, n_tok, align, cur, from_mem && have, gap, variant == 2, gd, l,
                                      bcast_f(b.k, rq), tr.c, tau, kt, lag_fast_ok(n, tau, kt), lane, nosink);
                    if (from_mem) have = false;
                }
                if (variant == 2) { res_lag = res; lag_done = true; }
                if ((mask >> lane) & 1ull) {
                    const float t_last = __fmaf_rn((float)(n - 1), tau, res.M);
                    const int nsrc = dev ? 0 : ((res.m >= 0) ? res.m : n);
                    acc_s_dec += (u64)nsrc;
                    if (res.m >= 0) { acc_mig += 1u; acc_repre += (u64)l + (u64)res.m; }
                    acc_tlast += (double)t_last;
                    if (a.mig_idx) a.mig_idx[(size_t)lane * tr.n_req + i] = res.m;
                    if (a.n_src_tok) a.n_src_tok[(size_t)lane * tr.n_req + i] = dev ? n : nsrc;
                    if (a.t_last) a.t_last[(size_t)lane * tr.n_req + i] = t_last;
                }
            }
        }
    }
    // lane = column: fold the waves of the workgroup, then add into this workgroup's copy of the totals
    sh[0 * TS_BLOCK + threadIdx.x] = acc_s_dec; sh[1 * TS_BLOCK + threadIdx.x] = tot_n - acc_s_dec;
    sh[2 * TS_BLOCK + threadIdx.x] = acc_repre; sh[3 * TS_BLOCK + threadIdx.x] = (u64)acc_mig;
    sh[4 * TS_BLOCK + threadIdx.x] = tot_cnt; sh[5 * TS_BLOCK + threadIdx.x] = (u64)__double_as_longlong(acc_tlast);
    __syncthreads();
    if ((int)threadIdx.x < P) {
        u64 f[5];
        double tl = 0.0;
        for (int q = 0; q < 5; ++q) f[q] = 0;
        for (int w = 0; w < TS_BLOCK / 64; ++w) {
            for (int q = 0; q < 5; ++q) f[q] += sh[q * TS_BLOCK + w * 64 + threadIdx.x];
            tl += __longlong_as_double((long long)sh[5 * TS_BLOCK + w * 64 + threadIdx.x]);
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

// Totals -> accumulators; puts the totals back to zero for the next pass.
__global__ void k_tl_stats_fin(int P, MigPartial* totals, disco_accum* acc)
{
    const int c = threadIdx.x;
    if (c >= P) return;
    MigPartial x{0, 0, 0, 0, 0, 0.0, {0, 0}};
    for (int k = 0; k < DISCO_NCOPY; ++k) {
        MigPartial* t = &totals[k * 64 + c];
        x.s_dec += t->s_dec; x.d_dec += t->d_dec; x.d_repre += t->d_repre; x.migrated += t->migrated;
        x.tbt_count += t->tbt_count; x.tlast_sum += t->tlast_sum;
        *t = MigPartial{0, 0, 0, 0, 0, 0.0, {0, 0}};
    }
    disco_accum* o = &acc[c];
    o->m_s_dec = (i64)x.s_dec; o->m_d_dec = (i64)x.d_dec; o->m_d_repre = (i64)x.d_repre;
    o->n_migrated = (i64)x.migrated; o->tbt_count = (i64)x.tbt_count; o->tlast_sum = x.tlast_sum;
}

// ------------------------------------------------------------- histogram ---

struct HistArgs {
    float tau, kt;
    int P, pass;
    SelState* S;
    unsigned* ghist;
    unsigned* ppcnt;
};

// Digit of this pass and the rows of the LDS histogram.
struct HistCtx {
    unsigned* hist;
    int shift, width, up, G;
    unsigned stride;               // words per prefix group = nwalk << width
    unsigned grp_prefix[DISCO_MAX_GRP];
};

// Every key of the chunk goes to the histogram row (prefix group of the key,
// class of the timeline).  The bin shared by most of the wave is counted with
// ballots and added once; the rest is added lane by lane.
__device__ __forceinline__ void hist_keys(const HistCtx& h, const unsigned key[4], unsigned row_base, int lane)
{
    const unsigned dmask = (1u << h.width) - 1u;
    unsigned idx[4];
    bool pend[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const unsigned hi = key[q] >> h.up;                      // up <= 31: the sign flag of skipped keys stays in
        unsigned g = 0;
        bool hit = hi == h.grp_prefix[0];
        if (h.G > 1) {
#pragma unroll
            for (int k = 1; k < DISCO_MAX_GRP; ++k) {
                const bool hk = k < h.G && hi == h.grp_prefix[k] && !hit;
                g = hk ? (unsigned)k : g;
                hit = hit || hk;
            }
        }
        pend[q] = hit;
        idx[q] = g * h.stride + row_base + ((key[q] >> h.shift) & dmask);
    }
    const u64 todo = __ballot(pend[0] || pend[1] || pend[2] || pend[3]);
    if (!todo) return;
    const int leader = __ffsll((long long)todo) - 1;
    const unsigned mine = pend[0] ? idx[0] : (pend[1] ? idx[1] : (pend[2] ? idx[2] : idx[3]));
    const unsigned i0 = (unsigned)bcast_i((int)mine, leader);
    unsigned cnt = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const bool same = pend[q] && idx[q] == i0;
        cnt += (unsigned)__popcll(__ballot(same));
        pend[q] = pend[q] && !same;
    }
    if (lane == leader) atomicAdd(&h.hist[i0], cnt);
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (pend[q]) atomicAdd(&h.hist[idx[q]], 1u);
}

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
    const i64 nbatch = (tr.n_req + TF_RB - 1) / TF_RB;
    for (i64 bt = (i64)blockIdx.x * (TH_BLOCK / 64) + wave; bt < nbatch; bt += nwaves) {
        const Batch b = load_batch(tr, spol, P, bt * TF_RB, lane);
        // lane = request: LDS row of each of the three timelines, 0xFF = nothing to walk
        unsigned desc = 0xFFFFFFu;
        {
            const bool short_n = b.n >= 0 && b.n <= DISCO_PP_NMAX;
#pragma unroll
            for (int kind = 0; kind < 3; ++kind) {
                if (b.m[kind] == 0ull) continue;
                const int c = cls_find(s_cls, ncls, b.m[kind]);
                const bool analytic = short_n && (kind == 0 ? pure_pacing(true, b.gd, tau) : pure_pacing(!mem, b.gap, tau));
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
                walk<true>(from_mem, n, tr.arr, off, n_tok, align, cur, from_mem && have, gap, variant == 2, gd, l,
                           bcast_f(b.k, rq), tr.c, tau, kt, lag_fast_ok(n, tau, kt), lane, sink);
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

void disco_launch_tl_stats_fast(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                                MigPartial* totals, hipStream_t stream)
{
    StatsArgs s;
    memset(&s, 0, sizeof(s));
    s.tau = a.tau; s.kt = a.kt; s.P = a.P;
    s.mig_idx = a.mig_idx; s.n_src_tok = a.n_src_tok; s.t_last = a.t_last;
    s.totals = totals;
    const i64 per_block = (i64)(TS_BLOCK / 64) * TF_RB;
    i64 b = (v.n_req + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > 2048) b = 2048;                    // eight resident workgroups per CU
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_tl_stats, dim3((unsigned)b), dim3(TS_BLOCK), 0, stream, v, n_tok, align, pol, s);
    hipLaunchKernelGGL(k_tl_stats_fin, dim3(1), dim3(64), 0, stream, a.P, totals, a.acc);
}

void disco_launch_tl_hist_fast(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                               hipStream_t stream)
{
    HistArgs h;
    memset(&h, 0, sizeof(h));
    h.tau = a.tau; h.kt = a.kt; h.P = a.P; h.pass = a.pass;
    h.S = a.S; h.ghist = a.ghist; h.ppcnt = a.ppcnt;
    const i64 per_block = (i64)(TH_BLOCK / 64) * TF_RB;
    i64 b = (v.n_req + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > 512) b = 512;                      // two resident workgroups per CU
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_tl_hist, dim3((unsigned)b), dim3(TH_BLOCK), 0, stream, v, n_tok, align, pol, h);
}
